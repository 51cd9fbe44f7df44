"""GPU parity at the full shapes of workloads C2-C5 (sb_inputs.CONFIGS), in the launch
configuration bench.py times (MFMA projections, forced exit schedule with draft
injection, second stream for the exit heads).

The oracle scores the library's output position by position (teacher forcing) on a
sample it can afford: a prompt of several 128-row passes plus 128 generated positions
per workload.  The properties that hold at any size are checked at the workloads' own
prompt lengths: speculative output == the library's own greedy output, bit for bit, and
the accept schedule is realised exactly."""
import numpy as np
import pytest

import oracle as orc
import sb_inputs as si
from helpers import teacher_forced_check, progress, NearTies
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


# Oracle scoring at full size: prompt and generated positions the oracle teacher-forces per
# workload (the prompts span several 128-row passes plus a ragged tail; C3's spans nine).
ORACLE_SAMPLE = {"C2": (300, 128), "C3": (1040, 128), "C4": (272, 128), "C5": (272, 128)}
# positions also scored by the float build of the oracle (same weights; C2 and C3 share theirs)
ORACLE32_POSITIONS = {"C2": 128}
GAP_RULE = 1e-2     # an arg-max difference is a flagged near-tie below this oracle gap ...
GAP_HARD = 2e-2     # ... tolerated (counted as "wide") up to this one, a failure above


def _score(om, sp, toks, label):
    rep = {}
    teacher_forced_check(om, sp, toks, gap_tol=GAP_HARD, report=rep, every=64)
    wide = [g for g in rep["gaps"] if g >= GAP_RULE]
    progress(f"[fullsize] {label}: scored {rep['scored']} positions, {rep['flagged']} flagged "
             f"(largest gap {max(rep['gaps'], default=0.0):.4g}), {len(wide)} of them at or above {GAP_RULE}, "
             f"{rep['close_positions']} positions with an oracle top-2 gap below {GAP_HARD}")
    return rep, wide


def _run_config(sb, name, prompt_len, gen_len):
    import torch
    wl = si.CONFIGS[name]
    shape = wl.shape
    n_oracle_prompt, n_oracle_gen = ORACLE_SAMPLE[name]
    progress(f"[fullsize] {wl.name}: generating weights")
    w = si.make_weights(shape, wl.weight_seed)
    max_seq = (prompt_len + gen_len + 4 * wl.w_max + 31) // 16 * 16
    gm = sb.Model(shape, w, max_seq)
    prompt = si.make_prompt(shape.vocab, prompt_len, wl.prompt_seed)
    s = gm.session()
    first = s.prefill(prompt)
    progress(f"[fullsize] {wl.name}: prefill of {prompt_len} done")
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
    # (4) the oracle scores a sequence produced by the same path: a prompt of several 128-row
    # passes, then speculative decoding with the workload's schedule
    sp = prompt[:n_oracle_prompt]
    s2 = gm.session()
    f2 = s2.prefill(sp)
    G2, _ = s2.decode(n_oracle_gen + wl.w_max, sb.Params(0, 1, [], wl.threshold))
    g2 = [f2] + G2.tolist()
    p2, _ = _spec_params(sb, wl, g2, 4 * n_oracle_gen)
    s2.rewind(n_oracle_prompt, f2)
    o2, st2 = s2.decode(n_oracle_gen, p2)
    assert o2.tolist() == g2[1:n_oracle_gen + 1]
    assert st2["drafts"] == st2["rounds"] * wl.w_max
    oseq = (n_oracle_prompt + n_oracle_gen + 31) // 16 * 16
    progress(f"[fullsize] {wl.name}: oracle scoring {n_oracle_prompt}+{n_oracle_gen} positions")
    om = Oracle(shape, w, oseq)
    # Rule: the library's token is the oracle's arg max, or the oracle's gap between the two is
    # below 1e-2 (flagged).  After 32-40 random-init layers fp32 arithmetic itself sits up to
    # 1.6e-2 from the double oracle's logits (the all-fp32 vector path included), so a gap in
    # [1e-2, 2e-2) is counted separately and at most one per sequence is tolerated; the counts
    # and the largest gap are printed.
    rep, wide = _score(om, sp, [f2] + o2.tolist(), f"{wl.name} vs double oracle")
    assert len(wide) <= 1 and rep["flagged"] <= max(2, rep["close_positions"]), rep
    if name in ORACLE32_POSITIONS:
        n32 = ORACLE32_POSITIONS[name]
        om32 = Oracle(shape, w, oseq, bits=32)
        rep32, wide32 = _score(om32, sp, ([f2] + o2.tolist())[:n32], f"{wl.name} vs float oracle")
        assert len(wide32) <= 1, rep32
        del om32
    # first exit-head evaluation of a draft step against the oracle: logits, arg max, confidence
    osn = om.session()
    osn.prefill(sp[:12])
    s3 = gm.session()
    s3.debug_enable(True)
    s3.prefill(sp[:12])
    po = orc.OrcParams(wl.d_max, wl.w_max, wl.temperatures(), wl.threshold, forced_exit=[2, 0])
    pg = sb.Params(wl.d_max, wl.w_max, wl.temperatures(), wl.threshold, forced_exit=[2, 0])
    ro, rg = osn.draft_step(po), s3.draft_step(pg)
    assert (ro["status"], ro["exit_layer"]) == (rg["status"], rg["exit_layer"]) == (sb.EXITED, 2)
    zo, zg = osn.head_logits(), s3.debug_logits(2)
    assert np.max(np.abs(zg - zo)) <= 2e-2 * np.max(np.abs(zo))
    assert abs(ro["confidence"] - rg["confidence"]) <= 1e-3
    if ro["token"] != rg["token"]:
        NearTies(GAP_RULE).flag("exit head of a draft step", zo, rg["token"])
    del osn, om
    if name in BATCH_CHECK:
        _batch_check(sb, gm, wl, prompt)
    return st_ar, st


# workloads whose model also decodes a batch (MHA at 7B, GQA with the 128256-row heads at 8B)
BATCH_CHECK = ("C2", "C5")


def _batch_check(sb, gm, wl, prompt):
    """Four sequences with contexts of 1 to 5 attention chunks decoded together, speculative with
    forced schedules and greedy: each must be bit-identical to its own single-sequence run."""
    B, w_max, n_new = 4, 2, 24
    lens = [40, 300, min(len(prompt), 512), 130]
    prompts = [prompt[:n] for n in lens]
    P = []
    for b in range(B):
        fe = si.forced_exit_schedule(wl.sched_seed + 7 * b, 4 * n_new, wl.exit_lo, wl.d_max)
        fd = np.where(np.random.default_rng(b).random(4 * n_new) < 0.4, 11 + b, -1).astype(np.int32)
        P.append(sb.Params(wl.d_max, w_max, wl.temperatures(), wl.threshold, forced_exit=fe, forced_draft=fd))
    alone = []
    for b in range(B):
        s = gm.session()
        f = s.prefill(prompts[b])
        o, st = s.decode(n_new, P[b])
        alone.append(([f] + o.tolist(), st))
        del s
    sess = [gm.session() for _ in range(B)]
    firsts = [s.prefill(p) for s, p in zip(sess, prompts)]
    outs = sb.Batch(sess).decode(n_new, P)
    for b in range(B):
        assert [firsts[b]] + outs[b].tolist() == alone[b][0], b
        st = sess[b].stats()
        assert st["accept_hist"] == alone[b][1]["accept_hist"] and st["exit_hist"] == alone[b][1]["exit_hist"], b
    for s, f, n in zip(sess, firsts, lens):
        s.rewind(n, f)
    g_batch = sb.Batch(sess).decode(n_new, [sb.Params(0, 1, [], wl.threshold)] * B)
    for b in range(B):   # speculative == greedy for every sequence, and the batch's greedy == the spec run alone
        assert g_batch[b].tolist() == alone[b][0][1:], b
    progress(f"[fullsize] {wl.name}: batch of {B} (contexts {lens}) equals the single-sequence runs")


def test_c2_7b_full_shape(sb):
    _run_config(sb, "C2", prompt_len=512, gen_len=512)


def test_c3_7b_long_context(sb):
    # 4096-token prompt in the paged cache, w_max = 8: verify attention over > 4100 keys
    _run_config(sb, "C3", prompt_len=4096, gen_len=256)


def test_c4_13b_full_shape(sb):
    _run_config(sb, "C4", prompt_len=1024, gen_len=1024)


def test_c5_8b_gqa_large_vocab(sb):
    _run_config(sb, "C5", prompt_len=2048, gen_len=1024)


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
