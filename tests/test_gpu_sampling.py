"""GPU parity of sampling-mode verification (Sec. 4.3, sampling strategies) against the oracle,
through the C ABI: same uniforms, same forced schedule, round by round; then the distribution of
what the library emits against the full model's distribution as the oracle computes it; and the
cold limit, which must reproduce greedy decoding."""
import numpy as np
import pytest
from scipy import stats

import oracle as orc
import sb_inputs as si
from helpers import gpu_model, gpu_params, linear_T, NearTies, all_accept_weights
from oracle import Oracle, OrcParams

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12247_amd as sb
    return sb


def _peaked(shape_kw, seed=91, scale=14.0, vocab=1024):
    """Tiny model with a peaked final distribution whose drafts are the full model's likeliest token."""
    shape = si.tiny_shape(n_layers=5, n_exit_heads=3, vocab=vocab, **shape_kw)
    w = si.make_weights(shape, seed, gain_jitter=0.1)
    w["final_norm"] = (w["final_norm"] * scale).astype(np.float32)
    # layers past the first add nothing and the exit heads are the final head: a draft is the full
    # model's most likely token, so that it is accepted with that token's probability
    return shape, all_accept_weights(shape, w, 1)


def _near_boundary(P, u_acc, u_draw, x, tok_gpu, tol=1e-4):
    """Is the GPU's decision for this row explained by a uniform within tol of a boundary of the
    oracle's distribution P: the acceptance threshold P[x], or an edge of the drawn token's cell
    of the cumulative distribution (without x)?"""
    if x >= 0 and abs(u_acc - P[x]) <= tol:
        return True
    Q = P.copy()
    if x >= 0:
        Q[x] = 0.0
    tot = Q.sum()
    if tot <= 0 or tok_gpu < 0 or Q[tok_gpu] <= 0:
        return False
    cdf = np.cumsum(Q) / tot
    return cdf[tok_gpu] - Q[tok_gpu] / tot - tol <= u_draw <= cdf[tok_gpu] + tol


@pytest.mark.parametrize("variant,vocab", [("fp32", 1024), ("bf16", 1024), ("bf16", 4112), ("bf16", 32000),
                                            # above 32768 the kernel keeps the remaining weights in memory: a tail of 16 tokens
                                            # (most threads own none of it), one full group of sixteen loads plus a ragged rest
                                            ("bf16", 32784), ("bf16", 32768 + 17 * 1024 + 16), ("bf16", 128256)])
@pytest.mark.parametrize("temp,top_p", [(1.0, 1.0), (0.3, 1.0), (1.0, 0.9), (0.7, 0.5)])
def test_sampling_decisions_follow_the_rule_on_the_librarys_own_logits(sb, variant, vocab, temp, top_p):
    """The decision part alone, in one precision: the oracle's distribution and inverse-CDF draw are
    applied to the logits the library itself computed (parity tap), with the same uniforms; accepted
    drafts, acceptance probabilities, the drawn token and the emitted count must be the library's.
    (The logits themselves are compared with the oracle's elsewhere.)  A uniform within 1e-5 of a
    boundary of that distribution may fall on the other side: counted, at most one per run."""
    B = si.configs.BF16
    kw = dict() if variant == "fp32" else dict(weight_dtype=B, kv_dtype=B, d_ffn=768)
    shape, w = _peaked(kw, vocab=vocab)
    gm = gpu_model(shape, w, 256)
    prompt = si.make_prompt(shape.vocab, 9, 503)
    U = np.random.default_rng(5).random(2 * 256).astype(np.float32)
    fe = [1, 2, 3, 1, 0, 2, 2, 3, 1, 1, 1, 1] * 20
    pg = sb.Params(3, 4, linear_T(3), 0.5, forced_exit=fe, sample_temperature=temp, top_p=top_p, sample_u=U)
    gsn = gm.session()
    gsn.debug_enable(True)
    gsn.prefill(prompt)
    flagged, accepted, drawn = 0, 0, 0
    for rnd in range(30):
        drafts = []
        while True:
            rg = gsn.draft_step(pg)
            if rg["exit_layer"]:
                drafts.append(rg["token"])
            if rg["status"] != sb.EXITED:
                break
        c0 = gsn.committed_len()
        vg = gsn.verify(pg)
        M = vg["n_rows"]
        m, toks = 0, []
        for i in range(M):
            P = orc.sample_dist(gsn.debug_logits(0, i).astype(np.float64), temp, top_p)
            pos = c0 + i
            x = drafts[i] if i < len(drafts) else -1
            if x >= 0:
                assert abs(vg["accept_prob"][i] - P[x]) <= 2e-6 + 1e-5 * P[x], (rnd, i)
            if x >= 0 and U[2 * pos] < P[x]:
                toks.append(x); m += 1
                continue
            toks.append(orc.sample_token(P, float(U[2 * pos + 1]), x))
            break
        want = (m, min(m + 1, M), toks[: min(m + 1, M)])
        got = (vg["n_matched"], vg["n_emit"], vg["tokens"][: vg["n_emit"]])
        if want != got:
            i = min(m, vg["n_matched"])
            P = orc.sample_dist(gsn.debug_logits(0, i).astype(np.float64), temp, top_p)
            assert _near_boundary(P, U[2 * (c0 + i)], U[2 * (c0 + i) + 1], drafts[i] if i < len(drafts) else -1,
                                  vg["tokens"][i], tol=1e-5), (rnd, want, got)
            flagged += 1
        assert all(t == -1 for t in vg["tokens"][vg["n_emit"]:])
        accepted += vg["n_matched"]
        drawn += vg["n_emit"] - vg["n_matched"]
    assert flagged <= 1 and accepted > 0 and drawn > 0, (flagged, accepted, drawn)


@pytest.mark.parametrize("variant", ["fp32", "bf16"])
@pytest.mark.parametrize("temp,top_p", [(1.0, 1.0), (0.3, 1.0), (1.0, 0.9)])
def test_sampling_rounds_match_the_oracle(sb, variant, temp, top_p):
    """End to end against the oracle's rounds (its own logits, in double): several short runs with
    the same uniforms and schedule.  Here the two sides' logits differ by rounding, and a draw is
    sensitive to that wherever a uniform lies within 1e-3 (the tolerance of a confidence) of a
    boundary of the distribution: such a row ends its run and is counted."""
    B = si.configs.BF16
    kw = dict() if variant == "fp32" else dict(weight_dtype=B, kv_dtype=B, d_ffn=768)
    shape, w = _peaked(kw, vocab=1024)
    om, gm = Oracle(shape, w, 256), gpu_model(shape, w, 256)
    fe = [1, 2, 3, 1, 0, 2, 2, 3, 1, 1, 1, 1] * 20
    ties, boundary, rounds, accepted, drawn = NearTies(), 0, 0, 0, 0
    for trial in range(6):
        prompt = si.make_prompt(shape.vocab, 9, 503 + trial)
        U = np.random.default_rng(5 + trial).random(2 * 256).astype(np.float32)
        po = OrcParams(3, 4, linear_T(3), 0.5, forced_exit=fe, sample_temperature=temp, top_p=top_p, sample_u=U)
        pg = sb.Params(3, 4, linear_T(3), 0.5, forced_exit=fe, sample_temperature=temp, top_p=top_p, sample_u=U)
        osn, gsn = om.session(), gm.session()
        if osn.prefill(prompt) != gsn.prefill(prompt):
            ties.flag(f"trial {trial} prefill", osn.verify_logits(0), gsn.prefill(prompt))
            continue
        for rnd in range(10):
            drafts, stop = [], False
            while True:
                ro, rg = osn.draft_step(po), gsn.draft_step(pg)
                assert (ro["status"], ro["exit_layer"]) == (rg["status"], rg["exit_layer"])
                if ro["token"] != rg["token"]:
                    ties.flag(f"trial {trial} round {rnd} draft", osn.head_logits(), rg["token"])
                    stop = True
                    break
                if ro["exit_layer"]:
                    drafts.append(ro["token"])
                if ro["status"] != orc.EXITED:
                    break
            if stop:
                break
            c0 = osn.committed_len()
            vo, vg = osn.verify(po), gsn.verify(pg)
            assert (vo["n_rows"], vo["n_drafts"], vo["align_layer"]) == (vg["n_rows"], vg["n_drafts"], vg["align_layer"])
            first_diff = min(vo["n_matched"], vg["n_matched"])
            for i in range(min(first_diff + 1, len(drafts))):      # rows examined on both sides
                assert abs(vg["accept_prob"][i] - osn.verify_dist(i)[drafts[i]]) <= 1e-3, (trial, rnd, i)
            if (vo["n_matched"], vo["n_emit"], vo["tokens"][: vo["n_emit"]]) != (vg["n_matched"], vg["n_emit"], vg["tokens"][: vg["n_emit"]]):
                i, pos = first_diff, c0 + first_diff
                x = drafts[i] if i < len(drafts) else -1
                assert _near_boundary(osn.verify_dist(i), U[2 * pos], U[2 * pos + 1], x, vg["tokens"][i], tol=1e-3), (trial, rnd, vo, vg)
                boundary += 1
                break
            assert gsn.committed_len() == osn.committed_len()
            rounds += 1
            accepted += vo["n_matched"]
            drawn += vo["n_emit"] - vo["n_matched"]
    assert rounds >= 40 and len(ties.flags) + boundary <= 3, (rounds, ties.flags, boundary)
    assert accepted > 0 and drawn > 0


@pytest.mark.parametrize("temp,top_p", [(1.0, 1.0), (0.6, 0.9)])
def test_library_output_is_distributed_as_the_full_models_samples(sb, temp, top_p):
    """Chi-square of the first token the library's rounds emit (fresh uniforms every round)
    against the distribution the ORACLE computes from the full model's logits."""
    B = si.configs.BF16
    shape, w = _peaked(dict(weight_dtype=B, kv_dtype=B, d_ffn=768), vocab=64)
    om, gm = Oracle(shape, w, 64), gpu_model(shape, w, 64)
    prompt = si.make_prompt(shape.vocab, 7, 501)
    osn = om.session()
    first = osn.prefill(prompt)
    _, z1 = osn.step(first)
    p1 = orc.sample_dist(z1, temp, top_p)
    a = int(np.argmax(p1))
    gsn = gm.session()
    assert gsn.prefill(prompt) == first
    P0, V, N = len(prompt), shape.vocab, 2000
    g = np.random.default_rng(78)
    c1 = np.zeros(V)
    n_acc = 0
    for it in range(N):
        U = g.random(2 * 64).astype(np.float32)
        p = sb.Params(3, 4, linear_T(3), 0.5, forced_exit=[1, 2, 3, 1], sample_temperature=temp, top_p=top_p, sample_u=U)
        gsn.rewind(P0, first)
        while gsn.draft_step(p)["status"] == sb.EXITED:
            pass
        v = gsn.verify(p)
        c1[v["tokens"][0]] += 1
        n_acc += v["n_matched"] >= 1
    assert 0.05 * N < n_acc < 0.98 * N
    big = p1 * N >= 5
    obs = np.append(c1[big], c1[~big].sum())
    exp = np.append(p1[big] * N, p1[~big].sum() * N)
    keep = exp > 0
    assert obs[~keep].sum() == 0                       # nothing outside the nucleus
    stat = ((obs[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    assert stats.chi2.sf(stat, keep.sum() - 1) > 1e-3
    assert abs(c1[a] / N - p1[a]) < 0.05


def test_cold_sampling_reproduces_greedy_decoding(sb):
    B = si.configs.BF16
    shape, w = _peaked(dict(weight_dtype=B, kv_dtype=B, d_ffn=768), scale=3.0)
    gm = gpu_model(shape, w, 160)
    prompt = si.make_prompt(shape.vocab, 11, 505)
    fe = si.forced_exit_schedule(5, 300, 0, 3)
    U = np.random.default_rng(2).random(2 * 160).astype(np.float32)
    ref, st_ref = gm.session().generate(prompt, 40, gpu_params(3, 4, 0.5, forced_exit=fe))
    out, st = gm.session().generate(prompt, 40, sb.Params(3, 4, linear_T(3), 0.5, forced_exit=fe, sample_temperature=1e-4,
                                                          sample_u=U))
    assert out.tolist() == ref.tolist()
    assert st["accept_hist"] == st_ref["accept_hist"] and st["rounds"] == st_ref["rounds"]
    # and free-running sampled generation runs through sb_generate (every token in the vocabulary, rounds counted)
    out, st = gm.session().generate(prompt, 40, sb.Params(3, 4, linear_T(3), 0.5, forced_exit=fe, sample_temperature=0.8,
                                                          top_p=0.95, sample_u=U))
    assert len(out) == 40 and out.min() >= 0 and out.max() < shape.vocab and st["emitted"] >= 39


def test_sampling_parameter_errors(sb):
    shape, w = _peaked(dict())
    gm = gpu_model(shape, w, 160)
    s = gm.session()
    s.prefill(si.make_prompt(shape.vocab, 5, 1))
    U = np.zeros(400, np.float32)
    for kw in (dict(sample_temperature=-1.0), dict(sample_temperature=1.0), dict(sample_temperature=1.0, top_p=0.0, sample_u=U),
               dict(sample_temperature=1.0, top_p=1.5, sample_u=U)):
        with pytest.raises(sb.SbError) as e:
            s.draft_step(sb.Params(2, 2, linear_T(2), 0.5, **kw))
        assert e.value.code == sb.EINVAL
    p = sb.Params(2, 2, linear_T(2), 0.5, forced_exit=[1, 1], sample_temperature=1.0, sample_u=np.zeros(6, np.float32))
    while s.draft_step(p)["status"] == sb.EXITED:
        pass
    with pytest.raises(sb.SbError) as e:
        s.verify(p)
    assert e.value.code == sb.EINVAL and s.open_rows() == 2        # refused before anything was changed
