"""GPU parity at the full shapes of workloads C2-C5 (sb_inputs.CONFIGS), in the launch
configuration bench.py times (MFMA projections, forced exit schedule with draft
injection, second stream for the exit heads).

What the oracle can afford at these sizes is a short sequence: it scores the
library's output position by position (teacher forcing) on a 12-token prompt.  The
properties that hold at any size are checked at the real lengths: speculative
output == the library's own greedy output, bit for bit, and the accept schedule is
realised exactly."""
import numpy as np
import pytest

import oracle as orc
import sb_inputs as si
from helpers import teacher_forced_check
from oracle import Oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def sb():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2604_12247_amd as sb
    return sb


def _spec_params(sb, wl, greedy, n_rounds_hint):
    accepts = si.accept_schedule(wl.sched_seed, n_rounds_hint, wl.w_max)
    fd, rounds = si.injection_schedule(greedy, accepts, wl.w_max, wl.shape.vocab)
    fe = si.forced_exit_schedule(wl.sched_seed, len(fd), wl.exit_lo, wl.d_max)
    return sb.Params(wl.d_max, wl.w_max, wl.temperatures(), wl.threshold, forced_exit=fe, forced_draft=fd), accepts


def _run_config(sb, name, prompt_len, gen_len, n_oracle_prompt=12, n_oracle_gen=10):
    import torch
    wl = si.CONFIGS[name]
    shape = wl.shape
    print(f"[fullsize] {wl.name}: generating weights", flush=True)
    w = si.make_weights(shape, wl.weight_seed)
    max_seq = (prompt_len + gen_len + 4 * wl.w_max + 31) // 16 * 16
    gm = sb.Model(shape, w, max_seq)
    prompt = si.make_prompt(shape.vocab, prompt_len, wl.prompt_seed)
    s = gm.session()
    first = s.prefill(prompt)
    print(f"[fullsize] {wl.name}: prefill of {prompt_len} done", flush=True)
    n_ar = gen_len + 2 * wl.w_max
    G, st_ar = s.decode(n_ar, sb.Params(0, 1, [], wl.threshold))
    greedy = [first] + G.tolist()
    p_spec, accepts = _spec_params(sb, wl, greedy, 2 * gen_len)
    s.rewind(prompt_len, first)
    out, st = s.decode(gen_len, p_spec)
    # (1) identical to the library's own greedy decoding at the real length
    assert out.tolist() == greedy[1:gen_len + 1]
    # (2) every round emitted what the schedule says (the last one may be cut by gen_len)
    want = np.bincount(accepts[: st["rounds"]], minlength=sb.SB_MAX_W + 1)[: sb.SB_MAX_W + 1]
    got = np.array(st["accept_hist"])
    assert np.abs(got - want).sum() <= 2, (got, want)
    assert st["drafts"] == st["rounds"] * wl.w_max and st["exit_hist"][0] == 0
    assert min(i for i, v in enumerate(st["exit_hist"]) if v) >= wl.exit_lo
    # (3) a second run gives the same bits
    s.rewind(prompt_len, first)
    out2, _ = s.decode(gen_len, p_spec)
    assert out2.tolist() == out.tolist()
    del s
    # (4) the oracle scores a short sequence produced by the same path
    sp = prompt[:n_oracle_prompt]
    s2 = gm.session()
    f2 = s2.prefill(sp)
    G2, _ = s2.decode(n_oracle_gen + wl.w_max, sb.Params(0, 1, [], wl.threshold))
    g2 = [f2] + G2.tolist()
    p2, _ = _spec_params(sb, wl, g2, 4 * n_oracle_gen)
    s2.rewind(n_oracle_prompt, f2)
    o2, _ = s2.decode(n_oracle_gen, p2)
    assert o2.tolist() == g2[1:n_oracle_gen + 1]
    print(f"[fullsize] {wl.name}: oracle scoring {n_oracle_prompt}+{n_oracle_gen} positions", flush=True)
    om = Oracle(shape, w, 64)
    # At these shapes fp32 arithmetic itself sits 3e-3 rms (up to 1.6e-2) from the double oracle's
    # logits after 32 random-init layers, whichever projection kernel runs (the all-fp32 vector
    # path included): an oracle gap below 2e-2 can flip the arg max and is flagged, not failed.
    flagged, n = teacher_forced_check(om, sp, [f2] + o2.tolist(), gap_tol=2e-2)
    assert flagged <= 1, flagged
    # first exit-head evaluation of a draft step against the oracle: logits, arg max, confidence
    s2.rewind(n_oracle_prompt, f2)
    s2.debug_enable(True)
    osn = om.session()
    osn.prefill(sp)
    po = orc.OrcParams(wl.d_max, wl.w_max, wl.temperatures(), wl.threshold, forced_exit=[2, 0])
    pg = sb.Params(wl.d_max, wl.w_max, wl.temperatures(), wl.threshold, forced_exit=[2, 0])
    ro, rg = osn.draft_step(po), s2.draft_step(pg)
    assert (ro["status"], ro["exit_layer"]) == (rg["status"], rg["exit_layer"]) == (sb.EXITED, 2)
    zo, zg = osn.head_logits(), s2.debug_logits(2)
    assert np.max(np.abs(zg - zo)) <= 2e-2 * np.max(np.abs(zo))
    assert abs(ro["confidence"] - rg["confidence"]) <= 1e-3
    srt = np.sort(zo)
    if srt[-1] - srt[-2] >= 1e-2:
        assert ro["token"] == rg["token"]
    del osn, om
    return st_ar, st


def test_c2_7b_full_shape(sb):
    _run_config(sb, "C2", prompt_len=512, gen_len=192)


def test_c3_7b_long_context(sb):
    # 4096-token prompt in the paged cache, w_max = 8: verify attention over > 4100 keys
    _run_config(sb, "C3", prompt_len=4096, gen_len=96)


def test_c4_13b_full_shape(sb):
    _run_config(sb, "C4", prompt_len=256, gen_len=96)


def test_c5_8b_gqa_large_vocab(sb):
    _run_config(sb, "C5", prompt_len=256, gen_len=96)


def test_long_context_attention_kernel_against_oracle(sb):
    """Attention alone at 4100+ keys (33 chunks), sampled heads checked by the oracle."""
    import torch as T
    g = np.random.default_rng(11)
    Hq, Hkv, hd, M, n_ctx = 32, 32, 128, 8, 4100
    n_tot = n_ctx + M
    n_pages = (n_tot + 15) // 16 + 2
    rows = (Hq + 2 * Hkv) * hd
    qkv = (g.standard_normal((n_tot, rows)) * 1.3).astype(np.float32)
    pool = T.empty(2 * n_pages * Hkv * 16 * hd * 2, dtype=T.uint8, device="cuda")
    pool.fill_(0xFF)
    table = T.from_numpy(g.permutation(n_pages).astype(np.int32)).cuda()
    c, s = sb.rope_table(hd, 1e4, n_pages * 16)
    cd, sd = T.from_numpy(c).cuda(), T.from_numpy(s).cuda()
    pos = 0
    out = None
    while pos < n_tot:
        m = min(8, n_ctx - pos) if pos < n_ctx else M
        o = sb.op_attention(T.from_numpy(qkv[pos:pos + m]).cuda(), Hq, Hkv, hd, sb.BF16, pool, table, 0, cd, sd, pos)
        pos += m
        out = o
    out = out.cpu().numpy()
    def rnd(a):
        return si.bf16_to_f32(si.round_to_bf16(a.astype(np.float32)))
    for h in (0, 13, 31):
        K = np.stack([rnd(orc.rope_apply(qkv[t, (Hq + h) * hd:(Hq + h + 1) * hd], t, 1e4)) for t in range(n_tot)])
        V = rnd(qkv[:, (Hq + Hkv + h) * hd:(Hq + Hkv + h + 1) * hd])
        for r in (0, 7):
            p = n_ctx + r
            q = orc.rope_apply(qkv[p, h * hd:(h + 1) * hd], p, 1e4)
            ref = orc.attention_head(q, K[:p + 1], V[:p + 1])
            assert np.max(np.abs(out[r, h * hd:(h + 1) * hd] - ref)) <= 2e-5
