"""GPU parity of the single kernels against the CPU oracle, through the C ABI.
Sizes span several tiles and ragged tails; the oracle is double precision."""
import numpy as np
import pytest

import oracle as orc
import sb_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def T():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def _dev(T, a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return T.from_numpy(a).cuda()


def _rand_w(g, N, K, bf16, std=0.02):
    w = (g.standard_normal((N, K)) * std).astype(np.float32)
    return si.round_to_bf16(w) if bf16 else w


def _oracle_rows(W, x):
    return np.stack([orc.matvec(W, x[m].astype(np.float64)) for m in range(x.shape[0])])


@pytest.mark.parametrize("M,d", [(1, 256), (3, 4096), (8, 5120), (2, 688)])
def test_rmsnorm(T, M, d):
    import paper_2604_12247_amd as sb
    g = np.random.default_rng(M * 1000 + d)
    x = g.standard_normal((M, d)).astype(np.float32) * 0.3
    gain = (1 + 0.1 * g.standard_normal(d)).astype(np.float32)
    out = sb.op_rmsnorm(_dev(T, x), _dev(T, gain), 1e-6).cpu().numpy()
    ref = np.stack([orc.rmsnorm(x[m], gain, 1e-6) for m in range(M)])
    assert np.max(np.abs(out - ref)) <= 2e-6 * np.max(np.abs(ref))


VALU_CASES = [  # (N, K, bf16): N ragged against the 16-row block, K ragged against the 512 stride
    (50, 688, False), (768, 256, False), (1024, 256, True), (100, 4096, True), (4096, 11008, True),
    (37, 2056, False),
]


@pytest.mark.parametrize("N,K,bf16", VALU_CASES)
@pytest.mark.parametrize("M", [1, 3, 8])
def test_gemv_valu(T, N, K, bf16, M):
    import paper_2604_12247_amd as sb
    g = np.random.default_rng(N + K + M)
    W = _rand_w(g, N, K, bf16)
    x = g.standard_normal((M, K)).astype(np.float32)
    y = sb.op_gemv(_dev(T, W), _dev(T, x), sb.PROJ_VALU).cpu().numpy()
    ref = _oracle_rows(W, x)
    assert np.max(np.abs(y - ref)) <= 1e-5 * np.max(np.abs(ref)) + 1e-7


MFMA_CASES = [(16, 128), (64, 256), (4096, 4096), (12288, 4096), (4096, 11008), (32000, 4096), (48, 384),
              (15024, 256),      # two row tiles per block, an odd number of tiles: the last block owns one
              (4096, 14336),
              (6144, 4096), (5120, 5120), (5120, 13824)]   # between 4096 and 8192 output rows: one tile per block, four waves


@pytest.mark.parametrize("N,K", MFMA_CASES)
@pytest.mark.parametrize("M", [1, 5, 8])
def test_gemv_mfma(T, N, K, M):
    import paper_2604_12247_amd as sb
    g = np.random.default_rng(N + K + M + 1)
    W = _rand_w(g, N, K, True)
    x = g.standard_normal((M, K)).astype(np.float32)
    Wd = _dev(T, W)
    y = sb.op_gemv(Wd, _dev(T, x), sb.PROJ_MFMA).cpu().numpy()
    ref = _oracle_rows(W, x)
    # activations carry 16 mantissa bits (two bf16 parts): error ~ 2^-17 per term
    assert np.max(np.abs(y - ref)) <= 3e-5 * np.max(np.abs(ref)) + 1e-7
    # the tile-packed copy of the weights gives the same bits
    yp = sb.op_gemv(sb.op_repack(Wd), _dev(T, x), sb.PROJ_MFMA_PACKED).cpu().numpy()
    assert np.array_equal(yp, y)


GEMM_CASES = [(16, 128, 1), (48, 384, 5), (4096, 4096, 128), (12288, 4096, 37), (4096, 11008, 64), (22016, 4096, 128),
              (4112, 256, 17), (8192 + 80, 512, 97), (32000, 4096, 128)]


@pytest.mark.parametrize("N,K,M", GEMM_CASES)
def test_prompt_pass_gemm(T, N, K, M):
    """The projection of the prompt passes (up to 128 rows, k splits added in order) against the
    double-precision product of the same bf16 weights; unwritten rows of the scratch hold NaN."""
    import paper_2604_12247_amd as sb
    g = np.random.default_rng(N + K + M + 2)
    W = _rand_w(g, N, K, True)
    x = g.standard_normal((M, K)).astype(np.float32)
    Wp = sb.op_repack(_dev(T, W))
    scratch = T.empty(sb.lib().sb_op_gemm_scratch_bytes(N, K), dtype=T.uint8, device="cuda")
    scratch.fill_(0xFF)
    y = sb.op_gemm(Wp, _dev(T, x), scratch).cpu().numpy()
    ref = _oracle_rows(W, x)
    assert np.all(np.isfinite(y))
    assert np.max(np.abs(y - ref)) <= 3e-5 * np.max(np.abs(ref)) + 1e-7
    # a row's result does not depend on the rows beside it
    if M > 3:
        y3 = sb.op_gemm(Wp, _dev(T, x[:3]), scratch).cpu().numpy()
        assert np.array_equal(y3, y[:3])


GATE_UP_SHAPES = [(64, 256, 3), (11008, 4096, 1), (11008, 4096, 6), (14336, 4096, 8)]
GATE_UP_CASES = [(k, *c) for k in ("valu", "mfma", "mfma_packed") for c in GATE_UP_SHAPES] + [("valu", 1000, 512, 5)]


@pytest.mark.parametrize("kernel,N,K,M", GATE_UP_CASES)   # (the MFMA kernels take whole 16-row tiles: no ragged N there)
def test_gate_up_swiglu(T, kernel, N, K, M):
    """The gate/up sweep with its SwiGLU epilogue as the decode path runs it, against the oracle's
    mat-vec and SwiGLU, at the 7B and 8B FFN shapes and a ragged one."""
    import paper_2604_12247_amd as sb
    g = np.random.default_rng(N + K + M)
    W = _rand_w(g, 2 * N, K, True, std=0.03)
    x = g.standard_normal((M, K)).astype(np.float32)
    kid = {"valu": sb.PROJ_VALU, "mfma": sb.PROJ_MFMA, "mfma_packed": sb.PROJ_MFMA_PACKED}[kernel]
    Wd = _dev(T, W)
    if kernel == "mfma_packed":
        Wd = sb.op_repack(Wd)
    u = sb.op_gate_up(Wd, _dev(T, x), kid).cpu().numpy()
    for m in range(M):
        ref = orc.swiglu(orc.matvec(W, x[m].astype(np.float64)))
        scale = np.max(np.abs(ref))
        assert np.max(np.abs(u[m] - ref)) <= 1e-4 * scale, (m, np.max(np.abs(u[m] - ref)), scale)


@pytest.mark.parametrize("kernel", ["valu", "mfma", "mfma_packed"])
def test_gemv_row_result_does_not_depend_on_m(T, kernel):
    """A row's output is bit-identical whether it is computed alone or with others."""
    import paper_2604_12247_amd as sb
    k = {"valu": sb.PROJ_VALU, "mfma": sb.PROJ_MFMA, "mfma_packed": sb.PROJ_MFMA_PACKED}[kernel]
    g = np.random.default_rng(5)
    for N, K in ((4096, 4096), (1024, 11008), (32000, 256), (6144, 512), (15360, 256)):
        W = _dev(T, _rand_w(g, N, K, True))
        if kernel == "mfma_packed":
            W = sb.op_repack(W)
        x = g.standard_normal((8, K)).astype(np.float32)
        y8 = sb.op_gemv(W, _dev(T, x), k).cpu().numpy()
        for M in (1, 2, 5):
            yM = sb.op_gemv(W, _dev(T, x[:M]), k).cpu().numpy()
            assert np.array_equal(yM, y8[:M]), (N, K, M)
        # and a row does not care which slot it sits in
        y1 = sb.op_gemv(W, _dev(T, x[3:4]), k).cpu().numpy()
        assert np.array_equal(y1[0], y8[3])


@pytest.mark.parametrize("kernel", ["valu", "mfma", "mfma_packed"])
@pytest.mark.parametrize("N,K,M", [(1024, 256, 1), (32000, 4096, 1), (32000, 4096, 6), (128256, 512, 2), (128256, 4096, 3),
                                   (15024, 256, 3)])   # an odd number of 16-row tiles, two per block
def test_head_argmax_and_confidence(T, kernel, N, K, M):
    import paper_2604_12247_amd as sb
    k = {"valu": sb.PROJ_VALU, "mfma": sb.PROJ_MFMA, "mfma_packed": sb.PROJ_MFMA_PACKED}[kernel]
    g = np.random.default_rng(N + K + M)
    W = _rand_w(g, N, K, True, std=0.05)
    x = g.standard_normal((M, K)).astype(np.float32)
    Wd = sb.op_repack(_dev(T, W)) if kernel == "mfma_packed" else _dev(T, W)
    for Tl in (2.0, 1.0):
        am, cf, z = sb.op_head(Wd, _dev(T, x), Tl, k, want_logits=True)
        am, cf, z = am.cpu().numpy(), cf.cpu().numpy(), z.cpu().numpy()
        ref = _oracle_rows(W, x)
        assert np.max(np.abs(z - ref)) <= 2e-2 * np.max(np.abs(ref))
        assert np.max(np.abs(z - ref)) <= 1e-4 * np.max(np.abs(ref))      # what the kernels actually reach
        for m in range(M):
            o_am, o_cf = orc.act(ref[m], Tl)
            top2 = np.sort(ref[m])[-2:]
            if top2[1] - top2[0] >= 1e-2:
                assert am[m] == o_am
            assert am[m] == int(np.argmax(z[m]))      # consistent with its own logits, lowest index
            assert abs(cf[m] - o_cf) <= 1e-3
            assert abs(cf[m] - o_cf) <= 1e-5 + 1e-4 * o_cf


def test_head_ties_take_lowest_index(T):
    import paper_2604_12247_amd as sb
    # identical weight rows give exactly equal logits in any arithmetic
    g = np.random.default_rng(9)
    row = si.round_to_bf16((g.standard_normal(256) * 0.05).astype(np.float32))
    W = si.round_to_bf16((g.standard_normal((1024, 256)) * 0.001).astype(np.float32))
    x = si.bf16_to_f32(row).astype(np.float32)[None, :] * 4
    for rows in ((700, 33), (5, 1000), (512, 511)):
        W2 = W.copy()
        for r in rows:
            W2[r] = row
        for k in (sb.PROJ_VALU, sb.PROJ_MFMA, sb.PROJ_MFMA_PACKED):
            Wd = sb.op_repack(_dev(T, W2)) if k == sb.PROJ_MFMA_PACKED else _dev(T, W2)
            am, cf, _ = sb.op_head(Wd, _dev(T, x), 1.0, k)
            assert int(am.cpu()[0]) == min(rows)


def _attention_case(T, Hq, Hkv, hd, kv_bf16, n_ctx, M, base, shuffle, seed, oracle=True):
    """Append n_ctx + M rows in passes, then compare the last pass's output rows."""
    import paper_2604_12247_amd as sb
    g = np.random.default_rng(seed)
    kvd = sb.BF16 if kv_bf16 else sb.FP32
    n_tot = n_ctx + M
    n_pages = (n_tot + 15) // 16 + 1
    rows = (Hq + 2 * Hkv) * hd
    qkv = g.standard_normal((n_tot, rows)).astype(np.float32)
    es = 2 if kv_bf16 else 4
    pool = T.empty(3 * 2 * n_pages * Hkv * 16 * hd * es, dtype=T.uint8, device="cuda")
    pool.fill_(0xFF)     # NaN patterns: unwritten cache must never leak into a result
    order = g.permutation(n_pages).astype(np.int32) if shuffle else np.arange(n_pages, dtype=np.int32)
    table = _dev(T, order)
    c, s = sb.rope_table(hd, base, n_pages * 16)
    cd, sd = _dev(T, c), _dev(T, s)
    layer = 1
    pos = 0
    out = None
    passes = [8] * (n_ctx // 8) + ([n_ctx % 8] if n_ctx % 8 else []) + [M]
    scratch = T.empty(sb.lib().sb_op_attention_scratch_bytes(Hq, hd, kvd, n_pages), dtype=T.uint8, device="cuda")
    for m in passes:
        q = _dev(T, qkv[pos:pos + m])
        o = sb.op_attention(q, Hq, Hkv, hd, kvd, pool, table, layer, cd, sd, pos, scratch)
        if pos + m == n_tot:
            out = o.cpu().numpy()
        pos += m
    if not oracle:
        return None, out
    # oracle: rotate, round K/V as the cache does, attend
    def rnd(a):
        return si.bf16_to_f32(si.round_to_bf16(a.astype(np.float32))) if kv_bf16 else a.astype(np.float32)
    K = np.zeros((n_tot, Hkv, hd), np.float32); V = np.zeros_like(K)
    for t in range(n_tot):
        for h in range(Hkv):
            K[t, h] = rnd(orc.rope_apply(qkv[t, (Hq + h) * hd:(Hq + h + 1) * hd], t, base))
            V[t, h] = rnd(qkv[t, (Hq + Hkv + h) * hd:(Hq + Hkv + h + 1) * hd])
    G = Hq // Hkv
    worst = 0.0
    for r in range(M):
        p = n_ctx + r
        for h in range(Hq):
            q = orc.rope_apply(qkv[p, h * hd:(h + 1) * hd], p, base)
            ref = orc.attention_head(q, K[:p + 1, h // G], V[:p + 1, h // G])
            got = out[r, h * hd:(h + 1) * hd]
            worst = max(worst, float(np.max(np.abs(got - ref))))
    return worst, out


ATT_CASES = [  # Hq, Hkv, hd, kv_bf16, n_ctx, M, rope base, shuffled pages
    (4, 4, 64, False, 0, 1, 1e4, False),       # a single key
    (4, 4, 64, False, 29, 4, 1e4, True),
    (4, 2, 64, True, 130, 8, 1e4, True),       # crosses a chunk boundary inside the pass
    (8, 8, 128, True, 300, 6, 1e4, True),
    (8, 2, 128, True, 257, 6, 5e5, True),      # GQA, two query groups
    (2, 2, 128, False, 70, 3, 1e4, False),     # fp32 cache with 64-key chunks
    (8, 8, 128, True, 1018, 6, 1e4, True),     # eight whole 128-key chunks at the last row
    (8, 8, 128, True, 1020, 6, 1e4, True),     # the pass's rows straddle a chunk boundary
    (4, 2, 64, True, 1000, 8, 5e5, True),      # two query heads per kv head, sixteen query columns, head_dim 64, long context
    (8, 8, 128, True, 63, 3, 1e4, False),      # shorter than one chunk
    (8, 8, 128, True, 1030, 5, 1e4, True),     # nine chunks, the last one nearly empty
    (2, 1, 128, True, 65532, 4, 1e4, True),    # the longest context the kernels take: 512 chunks, 4096 shuffled pages
    (32, 32, 128, True, 3300, 6, 1e4, True),   # 32 x 26 blocks: more than the chip holds at once
    (16, 16, 64, True, 8300, 3, 1e4, True),    # 16 x 65 blocks, head_dim 64
    (32, 1, 64, True, 200, 3, 1e4, True),      # one kv head for 32 query heads: six 16-query groups per block
    (16, 1, 128, False, 90, 5, 1e4, False),    # the same on the fp32-cache kernel
]


@pytest.mark.parametrize("case", ATT_CASES)
def test_rope_append_attention(T, case):
    """One call per pass: rotary embedding, KV append and attention over the paged cache."""
    worst, _ = _attention_case(T, *case, seed=sum(int(x) for x in case[:6]))
    assert worst <= 2e-5, worst


def _check_rotated_k_cache(Kc, Ko):
    """Cached K (bf16 bits) against the oracle's.  The kernel rotates in float, the oracle in double:
    a value within float error of a rounding boundary may land on the neighbouring bf16 value (one
    unit in the last place, about 1 element in 30 000), and where the two products of the rotation
    cancel almost completely the float error (<= 2^-22 of the operands, here < 3e-6) can be a few units
    of the tiny result.  Nothing else may differ."""
    dk = np.abs(Kc.astype(np.int32) - Ko.astype(np.int32))
    da = np.abs(si.bf16_to_f32(Kc).astype(np.float64) - si.bf16_to_f32(Ko).astype(np.float64))
    assert not np.any((dk > 1) & (da > 3e-6)), (int(dk.max()), float(da.max()))
    assert (dk != 0).mean() <= 1e-3, float((dk != 0).mean())


PROMPT_ATT_CASES = [  # Hq, Hkv, hd, rows already cached, rows of this call, rope base
    (4, 4, 64, 0, 1, 1e4),          # a single key
    (4, 4, 64, 0, 70, 1e4),         # two query blocks, one chunk
    (4, 2, 64, 37, 200, 1e4),       # GQA, a cached prefix, chunk boundary inside a query block
    (6, 2, 128, 0, 150, 5e5),       # group of 3: query blocks straddle rows
    (8, 8, 128, 130, 333, 1e4),     # several chunks, ragged last block and last page
    (16, 1, 128, 40, 100, 1e4),     # one kv head for 16 query heads: a row fills a wave's 16 queries
]


@pytest.mark.parametrize("case", PROMPT_ATT_CASES)
def test_prompt_attention(T, case):
    """All rows of a prompt pass in one call (running soft-max per query): every output row and the
    cache it leaves against the oracle's attention, rows before pos0 cached by the per-pass kernel."""
    import paper_2604_12247_amd as sb
    Hq, Hkv, hd, n_ctx, M, base = case
    g = np.random.default_rng(5 + sum(int(x) for x in case[:5]))
    n_tot = n_ctx + M
    n_pages = (n_tot + 15) // 16 + 1
    rows = (Hq + 2 * Hkv) * hd
    qkv = (g.standard_normal((n_tot, rows)) * 1.2).astype(np.float32)
    pool = T.empty(2 * 2 * n_pages * Hkv * 16 * hd * 2, dtype=T.uint8, device="cuda")
    pool.fill_(0xFF)
    table = _dev(T, g.permutation(n_pages).astype(np.int32))
    c, s = sb.rope_table(hd, base, n_pages * 16)
    cd, sd = _dev(T, c), _dev(T, s)
    for pos in range(0, n_ctx, 8):
        sb.op_attention(_dev(T, qkv[pos:min(pos + 8, n_ctx)]), Hq, Hkv, hd, sb.BF16, pool, table, 1, cd, sd, pos)
    out = sb.op_prompt_attention(_dev(T, qkv[n_ctx:]), Hq, Hkv, hd, pool, table, 1, cd, sd, n_ctx).cpu().numpy()
    # a decode-style pass after it reads the cache the call left
    nxt = (g.standard_normal((1, rows))).astype(np.float32)
    after = sb.op_attention(_dev(T, nxt), Hq, Hkv, hd, sb.BF16, pool, table, 1, cd, sd, n_tot).cpu().numpy()

    # The cache first.  V is a plain rounding of the input: exact.  K is rounded after the rotation:
    # equal to the oracle's but for float rounding (_check_rotated_k_cache).  The attention below is
    # then checked against the oracle's attention over the keys the cache holds.
    raw = pool.view(T.int16).cpu().numpy().view(np.uint16).reshape(2, 2, n_pages, Hkv, 16 * hd)
    tbl = table.cpu().numpy()
    Kc = np.zeros((n_tot + 1, Hkv, hd), np.uint16); Vc = np.zeros_like(Kc)
    for t in range(n_tot + 1):
        pg = tbl[t // 16]
        for h in range(Hkv):
            Kc[t, h] = raw[1, 0, pg, h].reshape(16, hd)[t % 16]
            Vc[t, h] = raw[1, 1, pg, h].reshape(hd, 16)[:, t % 16]
    allq = np.concatenate([qkv, nxt])
    Ko = np.zeros_like(Kc); Vo = np.zeros_like(Kc)
    for t in range(n_tot + 1):
        for h in range(Hkv):
            Ko[t, h] = si.round_to_bf16(orc.rope_apply(allq[t, (Hq + h) * hd:(Hq + h + 1) * hd], t, base).astype(np.float32))
            Vo[t, h] = si.round_to_bf16(allq[t, (Hq + Hkv + h) * hd:(Hq + Hkv + h + 1) * hd])
    assert np.array_equal(Vc, Vo)
    _check_rotated_k_cache(Kc, Ko)
    K, V = si.bf16_to_f32(Kc), si.bf16_to_f32(Vc)
    G = Hq // Hkv
    worst = 0.0
    check_rows = range(M) if M <= 80 else sorted(set(list(range(0, M, 7)) + [63, 64, 127, 128, M - 2, M - 1]) & set(range(M)))
    for r in check_rows:
        p = n_ctx + r
        for h in range(Hq):
            q = orc.rope_apply(qkv[p, h * hd:(h + 1) * hd], p, base)
            ref = orc.attention_head(q, K[:p + 1, h // G], V[:p + 1, h // G])
            worst = max(worst, float(np.max(np.abs(out[r, h * hd:(h + 1) * hd] - ref))))
    assert worst <= 2e-5, worst
    for h in range(Hq):
        q = orc.rope_apply(nxt[0, h * hd:(h + 1) * hd], n_tot, base)
        ref = orc.attention_head(q, K[:, h // G], V[:, h // G])
        assert np.max(np.abs(after[0, h * hd:(h + 1) * hd] - ref)) <= 2e-5


@pytest.mark.parametrize("hd,n_ctx,M", [(128, 2048 + 40, 2048), (64, 0, 2048 + 77)])
def test_prompt_attention_wide_form(T, hd, n_ctx, M):
    """Launches large enough for the form with 32 queries per wave (32 kv heads x >= 2048 queries): sampled
    heads and rows against the oracle's attention over the keys the cache holds, cache of those heads
    checked as above.  The prefix, where there is one, is itself written by a call of the same kind."""
    import paper_2604_12247_amd as sb
    Hq = Hkv = 32
    base = 1e4
    g = np.random.default_rng(900 + hd)
    n_tot = n_ctx + M
    n_pages = (n_tot + 15) // 16 + 3
    rows = (Hq + 2 * Hkv) * hd
    qkv = (g.standard_normal((n_tot, rows)) * 1.2).astype(np.float32)
    pool = T.empty(2 * n_pages * Hkv * 16 * hd * 2, dtype=T.uint8, device="cuda")
    pool.fill_(0xFF)
    table = _dev(T, g.permutation(n_pages).astype(np.int32))
    c, s = sb.rope_table(hd, base, n_pages * 16)
    cd, sd = _dev(T, c), _dev(T, s)
    if n_ctx:
        sb.op_prompt_attention(_dev(T, qkv[:n_ctx]), Hq, Hkv, hd, pool, table, 0, cd, sd, 0)
    out = sb.op_prompt_attention(_dev(T, qkv[n_ctx:]), Hq, Hkv, hd, pool, table, 0, cd, sd, n_ctx).cpu().numpy()
    raw = pool.view(T.int16).cpu().numpy().view(np.uint16).reshape(2, n_pages, Hkv, 16 * hd)
    tbl = table.cpu().numpy()
    for h in (0, 13, 31):
        Kc = np.stack([raw[0, tbl[t // 16], h].reshape(16, hd)[t % 16] for t in range(n_tot)])
        Vc = np.stack([raw[1, tbl[t // 16], h].reshape(hd, 16)[:, t % 16] for t in range(n_tot)])
        Ko = np.stack([si.round_to_bf16(orc.rope_apply(qkv[t, (Hq + h) * hd:(Hq + h + 1) * hd], t, base).astype(np.float32))
                       for t in range(n_tot)])
        Vo = si.round_to_bf16(np.ascontiguousarray(qkv[:, (Hq + Hkv + h) * hd:(Hq + Hkv + h + 1) * hd]))
        assert np.array_equal(Vc, Vo)
        _check_rotated_k_cache(Kc, Ko)
        K, V = si.bf16_to_f32(Kc), si.bf16_to_f32(Vc)
        for r in (0, 1, 31, 32, 63, 64, 127, 128, 129, 1000, 1023, 1024, M - 130, M - 2, M - 1):
            p_ = n_ctx + r
            q = orc.rope_apply(qkv[p_, h * hd:(h + 1) * hd], p_, base)
            ref = orc.attention_head(q, K[:p_ + 1], V[:p_ + 1])
            assert np.max(np.abs(out[r, h * hd:(h + 1) * hd] - ref)) <= 2e-5, (h, r)


def test_attention_row_result_does_not_depend_on_m(T):
    """The same position gives the same bits alone and inside a pass of 6 rows."""
    args = (8, 8, 128, True)
    _, out6 = _attention_case(T, *args, 250, 6, 1e4, True, seed=77)
    for r in (0, 3, 5):
        _, out1 = _attention_case(T, *args, 250 + r, 1, 1e4, True, seed=77)
        assert np.array_equal(out1[0], out6[r])
    # a pass whose rows straddle a chunk boundary (1024): the number of chunks a row sees is a
    # function of its own position, alone or beside rows that see one chunk less
    _, out6 = _attention_case(T, *args, 1021, 6, 1e4, True, seed=78)
    for r in (0, 2, 3, 5):
        _, out1 = _attention_case(T, *args, 1021 + r, 1, 1e4, True, seed=78)
        assert np.array_equal(out1[0], out6[r]), r
    # a pass of six rows with 32 kv heads x 25 chunks (more blocks than the chip holds at once) against
    # single rows with 24 and with 25 chunks
    args = (32, 32, 128, True)
    _, out6 = _attention_case(T, *args, 3070, 6, 1e4, True, seed=79, oracle=False)
    for r in (0, 1, 2, 5):
        _, out1 = _attention_case(T, *args, 3070 + r, 1, 1e4, True, seed=79, oracle=False)
        assert np.array_equal(out1[0], out6[r]), r

