// Host side of libspecbound: the C ABI, argument validation, and the state
// machine of Bounded Speculation with Cached States (Sec. 3.3, Appendix A) that
// decides which rows go through which layer and enqueues the kernels.  All
// arithmetic of the method runs in the kernels; the host only keeps integers
// (positions, reached layers, counters).  This file: configuration, model and session
// life cycle, the rounds of one sequence.  batch.cpp: several sequences side by side;
// ops.cpp: the single-kernel entry points; host.h: what the three share.
#include <chrono>
#include <cmath>
#include <cstdio>

#include "host.h"

using namespace sb;
using namespace sbhost;

namespace sbhost {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

double now_ms() {
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

}  // namespace sbhost

namespace {

int check_config(const sb_config* c) {
    if (!c) return fail(SB_EINVAL, "config is NULL");
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 1 || c->vocab < 1)
        return fail(SB_EINVAL, "config: non-positive dimension");
    if (c->n_heads % c->n_kv_heads) return fail(SB_EINVAL, "config: n_heads must be a multiple of n_kv_heads");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(SB_EINVAL, "config: head_dim must be 64 or 128");
    if (c->weight_dtype != SB_FP32 && c->weight_dtype != SB_BF16) return fail(SB_EINVAL, "config: weight_dtype");
    if (c->kv_dtype != SB_FP32 && c->kv_dtype != SB_BF16) return fail(SB_EINVAL, "config: kv_dtype");
    if (c->n_exit_heads < 0 || c->n_exit_heads > c->n_layers || c->n_exit_heads > SB_MAX_EXIT_LAYERS)
        return fail(SB_EINVAL, "config: n_exit_heads out of range");
    if (c->max_seq < SB_KV_BLOCK || c->max_seq % SB_KV_BLOCK)
        return fail(SB_EINVAL, "config: max_seq must be a positive multiple of %d", SB_KV_BLOCK);
    // the attention kernels merge at most 512 key chunks (of 128 keys, 64 where a key's row exceeds 256 bytes)
    if ((c->max_seq + attn_chunk_keys(c->head_dim, c->kv_dtype) - 1) / attn_chunk_keys(c->head_dim, c->kv_dtype) > 512)
        return fail(SB_EINVAL, "config: max_seq = %d exceeds the longest context the attention kernels take (%d tokens)", c->max_seq,
                    512 * attn_chunk_keys(c->head_dim, c->kv_dtype));
    if (c->d_model % 8 || c->d_ffn % 8 || (c->n_heads * c->head_dim) % 8)
        return fail(SB_EINVAL, "config: d_model, d_ffn and n_heads*head_dim must be multiples of 8");
    if (!(c->rms_eps >= 0.f) || !(c->rope_base > 0.f)) return fail(SB_EINVAL, "config: rms_eps / rope_base");
    if (c->proj_kernel < SB_PROJ_AUTO || c->proj_kernel > SB_PROJ_MFMA_PACKED) return fail(SB_EINVAL, "config: proj_kernel");
    if (c->kv_block != 0 && c->kv_block != SB_KV_BLOCK) return fail(SB_EINVAL, "config: kv_block must be %d (or 0)", SB_KV_BLOCK);
    if (c->max_w < 0 || c->max_w > SB_MAX_W) return fail(SB_EINVAL, "config: max_w must be in 1..%d (or 0)", SB_MAX_W);
    if (c->proj_kernel == SB_PROJ_MFMA || c->proj_kernel == SB_PROJ_MFMA_PACKED) {
        if (c->weight_dtype != SB_BF16) return fail(SB_EINVAL, "config: the MFMA projection path needs bf16 weights");
        if (c->d_model % 128 || c->d_ffn % 128 || (c->n_heads * c->head_dim) % 128 || c->vocab % 16 || c->d_ffn % 16)
            return fail(SB_EINVAL, "config: the MFMA path needs K %% 128 == 0 and N %% 16 == 0");
    }
    return SB_OK;
}

int resolve_proj(const sb_config* c) {
    if (c->proj_kernel != SB_PROJ_AUTO) return c->proj_kernel;
    bool ok = c->weight_dtype == SB_BF16 && c->d_model % 128 == 0 && c->d_ffn % 128 == 0 &&
              (c->n_heads * c->head_dim) % 128 == 0 && c->vocab % 16 == 0;
    return ok ? SB_PROJ_MFMA_PACKED : SB_PROJ_VALU;
}


WsLayout ws_layout(const sb_config* c) {
    WsLayout L{};
    const size_t d = c->d_model, f = c->d_ffn, V = c->vocab, hq = (size_t)c->n_heads * c->head_dim;
    const size_t qkv_rows = (size_t)(c->n_heads + 2 * c->n_kv_heads) * c->head_dim;
    L.n_pages = c->max_seq / SB_KV_BLOCK;
    const int ch = attn_chunk_keys(c->head_dim, c->kv_dtype);
    L.max_chunks = (c->max_seq + ch - 1) / ch;
    const int hb_v = head_blocks_valu(c->vocab), hb_m = head_blocks_mfma(c->vocab);
    L.head_blocks = hb_v > hb_m ? hb_v : hb_m;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.H = take(SB_MAX_W * d * 4);
    L.xn = take(SB_MAX_W * d * 4);
    // slot-indexed inputs of the MFMA projections: bf16 parts of gain * h, and the
    // partial sums of squares that give the RMSNorm scale
    L.ssq_ld = (int)((d + 15) / 16);
    L.xs_attn = take(16 * d * 2);
    L.xs_ffn = take(16 * d * 2);
    L.xs_exit = take(16 * d * 2);
    L.xs_exit2 = take(16 * d * 2);
    L.ssq_exit = take((size_t)2 * SB_MAX_W * L.ssq_ld * 4);
    L.ssq_attn = take((size_t)SB_MAX_W * L.ssq_ld * 4);
    L.ssq_ffn = take((size_t)SB_MAX_W * L.ssq_ld * 4);
    L.qkv = take(SB_MAX_W * qkv_rows * 4);
    L.att = take(SB_MAX_W * hq * 4);
    L.atts = take(16 * hq * 2);
    L.u = take(SB_MAX_W * f * 4);
    L.us = take(16 * f * 2);
    L.attn_part = take((size_t)SB_MAX_W * c->n_heads * L.max_chunks * (c->head_dim + 2) * 4);
    L.head_part = take((size_t)SB_MAX_W * L.head_blocks * 16);
    L.logits_exit = take((size_t)(c->n_exit_heads > 0 ? c->n_exit_heads : 1) * V * 4);
    L.logits_final = take((size_t)SB_MAX_W * V * 4);
    // the sampling-mode acceptance kernel keeps the soft-max weights of a large vocabulary here
    L.sample_w = take(V > 32 * 1024 ? (size_t)SB_MAX_W * (V - 32 * 1024) * 4 : 0);
    L.round = take(sizeof(DevRound));
    L.table = take((size_t)L.n_pages * 4);
    L.prefill_gemm = resolve_proj(c) == SB_PROJ_MFMA_PACKED;
    if (L.prefill_gemm) {
        // a super-pass: up to SB_PREFILL_PASSES passes of SB_PREFILL_ROWS rows per launch
        const size_t PM = SB_PREFILL_ROWS;
        size_t RS = (size_t)(c->max_seq + PM - 1) / PM * PM;
        if (RS > PM * SB_PREFILL_PASSES) RS = PM * SB_PREFILL_PASSES;
        L.p_rows = (int)RS;
        L.p_ssq_ld = (int)((d + 255) / 256);
        L.p_tok = take((size_t)c->max_seq * 4);
        L.p_H = take(RS * d * 4);
        L.p_xs = take(2 * RS * d * 2);
        L.p_ssq = take(RS * L.p_ssq_ld * 4);
        L.p_qkv = take(RS * qkv_rows * 4);
        L.p_atts = take(2 * RS * hq * 2);
        L.p_us = take(2 * RS * f * 2);
        size_t pe = 0;  // largest set of k-split partials: any projection, any number of passes
        const size_t shapes[4][2] = {{qkv_rows, d}, {d, hq}, {2 * f, d}, {d, f}};
        for (auto& sh : shapes)
            for (int np = 1; np <= (int)(RS / PM); ++np) {
                size_t e = (size_t)np * gemm_splits((int32_t)sh[0], (int32_t)sh[1], np) * PM * sh[0];
                if (e > pe) pe = e;
            }
        L.p_part = take(pe * 4);
        L.p_attn_part = take(PM * c->n_heads * L.max_chunks * (c->head_dim + 2) * 4);
    }
    L.total = off;
    return L;
}

// Bytes of the tile-packed copy of all projection matrices, each 256-byte aligned.
size_t packed_weight_bytes(const sb_config* c) {
    if (resolve_proj(c) != SB_PROJ_MFMA_PACKED) return 0;
    const size_t d = c->d_model, f = c->d_ffn, hq = (size_t)c->n_heads * c->head_dim, V = c->vocab;
    const size_t qkv_rows = (size_t)(c->n_heads + 2 * c->n_kv_heads) * c->head_dim;
    const size_t per_layer = align_up(qkv_rows * d * 2, 256) + align_up(d * hq * 2, 256) + align_up(2 * f * d * 2, 256) +
                             align_up(d * f * 2, 256);
    return per_layer * c->n_layers + align_up(V * d * 2, 256) * ((size_t)c->n_exit_heads + 1);
}

size_t kv_pool_bytes(const sb_config* c) {
    return (size_t)c->n_layers * 2 * (c->max_seq / SB_KV_BLOCK) * c->n_kv_heads * SB_KV_BLOCK * c->head_dim *
           esize(c->kv_dtype);
}

}  // namespace


namespace sbhost {

int check_params(const sb_session* s, const sb_params* p) {
    const sb_config& c = s->m->cfg;
    if (!p) return fail(SB_EINVAL, "params is NULL");
    const int wlim = c.max_w ? c.max_w : SB_MAX_W;
    if (p->w_max < 1 || p->w_max > wlim) return fail(SB_EINVAL, "w_max must be in 1..%d", wlim);
    int dlim = c.n_exit_heads < c.n_layers - 1 ? c.n_exit_heads : c.n_layers - 1;
    if (p->d_max < 0 || p->d_max > dlim) return fail(SB_EINVAL, "d_max must be in 0..%d", dlim);
    if (p->d_max > 0 && !p->T) return fail(SB_EINVAL, "T is NULL");
    for (int l = 0; l < p->d_max; ++l)
        if (!(p->T[l] > 0.f)) return fail(SB_EINVAL, "T[%d] must be positive", l);
    if (p->n_forced < 0) return fail(SB_EINVAL, "n_forced < 0");
    if (p->head_mask && p->d_max > 32) return fail(SB_EINVAL, "head_mask has 32 bits: d_max must be <= 32 with it");
    if (p->sample_temperature < 0.f) return fail(SB_EINVAL, "sample_temperature < 0");
    if (p->sample_temperature > 0.f) {
        if (!(p->top_p > 0.f) || p->top_p > 1.f) return fail(SB_EINVAL, "top_p must be in (0, 1]");
        if (!p->sample_u || p->n_sample_u < 0) return fail(SB_EINVAL, "sample_u is NULL");
    }
    return SB_OK;
}

int join_head(sb_session* s);

int readback(sb_session* s) {
    int jrc = join_head(s);
    if (jrc) return jrc;
    HIP_TRY(hipMemcpyAsync(s->h_round, s->d_round, sizeof(DevRound), hipMemcpyDeviceToHost, s->m->stream));
    HIP_TRY(hipStreamSynchronize(s->m->stream));
    return SB_OK;
}

// Waits until the head merge that carries sequence number `seq` has left its note, then takes the
// exit decision and what belongs to it into the host's copy of the round record.  The wait is a
// poll of host memory; if the note does not come (a failed launch), the stream's own error decides.
int wait_note(sb_session* s, int32_t seq, int idx) {
    volatile int32_t* n = s->note_h;
    const double t0 = now_ms();
    bool seen = false;
    for (int64_t spin = 0;; ++spin) {
        if (__atomic_load_n(&s->note_h[0], __ATOMIC_ACQUIRE) == seq) { seen = true; break; }
        if ((spin & 0x3ff) == 0x3ff) {
            const hipError_t q = hipStreamQuery(s->m->stream);
            if (q != hipErrorNotReady) {   // the stream is idle (or failed): the note is there now, or never comes
                HIP_TRY(q);
                seen = __atomic_load_n(&s->note_h[0], __ATOMIC_ACQUIRE) == seq;
                break;
            }
            if (now_ms() - t0 > 10000.0) break;
        }
    }
    s->st.host_wait_ms += now_ms() - t0;
    if (!seen) return fail(SB_EDEVICE, "draft_step: the exit decision did not arrive from the device");
    s->h_round->exit_flag = n[1];
    s->h_round->drafts[idx] = n[2];
    int32_t cb = n[3];
    memcpy(&s->h_round->conf[idx], &cb, 4);
    s->h_round->head_argmax[idx] = n[4];
    return SB_OK;
}


// Main stream waits for the exit head on the head stream that reads exit-operand buffer b.
int join_head_buf(sb_session* s, int b) {
    if (!s->head_pending[b]) return SB_OK;
    HIP_TRY(hipStreamWaitEvent(s->m->stream, s->ev_head[s->head_pending_ev[b]], 0));
    s->head_pending[b] = false;
    return SB_OK;
}
// Main stream waits for every exit head that is still running on the head stream.
int join_head(sb_session* s) {
    int rc = join_head_buf(s, 0);
    return rc ? rc : join_head_buf(s, 1);
}

int64_t gemv_bytes(const GemvArgs& a) {
    const int64_t rows = a.epi == EPI_SWIGLU ? 2 * (int64_t)a.N : a.N;
    const int64_t out = a.epi == EPI_HEAD ? 0 : (int64_t)a.M * a.N * 4;
    return rows * a.K * (int64_t)esize(a.w_dtype) + (int64_t)a.M * a.K * 4 + out;
}

int gemv(sb_session* s, GemvArgs& a, int cls, hipStream_t st) {
    a.packed = s->m->packed ? 1 : 0;
    if (s->fail_countdown > 0 && --s->fail_countdown == 0)   // test tap (sb_debug_fail_launch)
        return fail(SB_EDEVICE, "projection launch (N=%d K=%d M=%d epi=%d): injected failure", a.N, a.K, a.M, a.epi);
    ProfScope ps(s, cls, gemv_bytes(a), st);
    hipError_t e = s->m->proj == SB_PROJ_MFMA ? launch_gemv_mfma(a, st) : launch_gemv_valu(a, st);
    if (e != hipSuccess) return fail(SB_EDEVICE, "projection launch (N=%d K=%d M=%d epi=%d): %s", a.N, a.K, a.M, a.epi,
                                     hipGetErrorString(e));
    return SB_OK;
}

// One decoder layer (0-based l) on rows slot0..slot0+M-1, whose positions are
// c+slot0.. : RMSNorm -> QKV -> attention (with RoPE + KV append) -> W_o (+residual)
// -> RMSNorm -> gate/up + SwiGLU -> W_down (+residual).
// On the MFMA path the two RMSNorms are folded into the projections: whoever
// writes a hidden row (embedding, W_o, W_down) also leaves gain * h in bf16 parts
// and the partial sums of squares, per slot, for the projection that reads it
// next.  head_gain (nullable) asks W_down to do the same for the head that follows.
// exit_buf: which of the two exit-operand buffers W_down fills for the head (draft steps alternate
// them by layer, so that only the head of two layers ago has to be over); -1 = the first one, after
// every head still running has finished (alignment, verification).
int run_layer(sb_session* s, int l, int slot0, int M, const float* head_gain, int exit_buf = -1) {
    sb_model* m = s->m;
    const sb_config& c = m->cfg;
    const bool mf = m->proj == SB_PROJ_MFMA;
    hipStream_t st = m->stream;
    const int d = c.d_model, f = c.d_ffn, hq = c.n_heads * c.head_dim;
    const int qkv_rows = (c.n_heads + 2 * c.n_kv_heads) * c.head_dim;
    const int pos0 = s->c + slot0;
    if (pos0 + M > c.max_seq) return fail(SB_ECAPACITY, "KV capacity exceeded");
    float* H = wsp<float>(s, s->L.H) + (size_t)slot0 * d;
    float* xn = wsp<float>(s, s->L.xn);
    uint16_t* xs_attn = wsp<uint16_t>(s, s->L.xs_attn) + (size_t)slot0 * d;
    uint16_t* xs_ffn = wsp<uint16_t>(s, s->L.xs_ffn) + (size_t)slot0 * d;
    uint16_t* xs_exit = wsp<uint16_t>(s, exit_buf == 1 ? s->L.xs_exit2 : s->L.xs_exit) + (size_t)slot0 * d;
    float* ssq_attn = wsp<float>(s, s->L.ssq_attn) + (size_t)slot0 * s->L.ssq_ld;
    float* ssq_ffn = wsp<float>(s, s->L.ssq_ffn) + (size_t)slot0 * s->L.ssq_ld;
    float* qkv = wsp<float>(s, s->L.qkv);
    float* att = wsp<float>(s, s->L.att);
    uint16_t* atts = wsp<uint16_t>(s, s->L.atts);
    float* u = wsp<float>(s, s->L.u);
    uint16_t* us = wsp<uint16_t>(s, s->L.us);
    int rc;

    if (!mf) {
        ProfScope ps(s, SB_K_RMSNORM, (int64_t)M * d * 8, st);
        HIP_TRY(launch_rmsnorm(H, m->attn_norm[l], xn, nullptr, d, M, d, c.rms_eps, st));
    }
    GemvArgs g{};
    g.w_dtype = c.weight_dtype; g.M = M; g.eps = c.rms_eps; g.ssq_ld = s->L.ssq_ld;
    g.W = m->w_qkv[l]; g.N = qkv_rows; g.K = d; g.x = xn; g.xs = xs_attn; g.y = qkv; g.ldy = qkv_rows; g.epi = EPI_STORE;
    if (mf) { g.ssq_in = ssq_attn; g.ssq_nb = l == 0 ? 1 : d / 16; }  // layer 0 reads what the embedding left
    if ((rc = gemv(s, g, SB_K_QKV, st))) return rc;

    AttnArgs a{};
    a.q = qkv; a.rope_cos = m->rope_cos; a.rope_sin = m->rope_sin; a.qkv_rows = qkv_rows; a.n_heads = c.n_heads;
    a.kv = s->kv; a.layer = l; a.pos0 = pos0; a.M = M;
    a.partials = wsp<float>(s, s->L.attn_part); a.max_chunks = s->L.max_chunks;
    a.out = mf ? nullptr : att; a.out_split = mf ? atts : nullptr; a.split_rows = 8;
    const int64_t kv_read = (int64_t)(pos0 + M) * 2 * c.n_kv_heads * c.head_dim * (int64_t)esize(c.kv_dtype);
    {
        ProfScope ps(s, SB_K_ATTN, kv_read, st);
        HIP_TRY(launch_attention(a, st));
    }

    g.ssq_in = nullptr;
    g.W = m->w_o[l]; g.N = d; g.K = hq; g.x = att; g.xs = atts; g.y = H; g.ldy = d; g.epi = EPI_RESID;
    if (mf) { g.gainA = m->ffn_norm[l]; g.nxA = xs_ffn; g.ssq_out = ssq_ffn; }
    if ((rc = gemv(s, g, SB_K_WO, st))) return rc;
    g.gainA = nullptr; g.nxA = nullptr; g.ssq_out = nullptr;

    if (!mf) {
        ProfScope ps(s, SB_K_RMSNORM, (int64_t)M * d * 8, st);
        HIP_TRY(launch_rmsnorm(H, m->ffn_norm[l], xn, nullptr, d, M, d, c.rms_eps, st));
    }
    g.W = m->w_gate_up[l]; g.N = f; g.K = d; g.x = xn; g.xs = xs_ffn; g.y = mf ? nullptr : u; g.ys = mf ? us : nullptr;
    g.ldy = f; g.epi = EPI_SWIGLU;
    if (mf) { g.ssq_in = ssq_ffn; g.ssq_nb = d / 16; }
    if ((rc = gemv(s, g, SB_K_GATEUP, st))) return rc;
    g.ssq_in = nullptr;

    g.W = m->w_down[l]; g.N = d; g.K = f; g.x = u; g.xs = us; g.y = H; g.ys = nullptr; g.ldy = d; g.epi = EPI_RESID;
    if (mf) {
        if (l + 1 < c.n_layers) { g.gainA = m->attn_norm[l + 1]; g.nxA = xs_attn; }
        if (head_gain) { g.gainB = head_gain; g.nxB = xs_exit; }
        g.ssq_out = ssq_attn;
        if (head_gain && exit_buf >= 0)
            g.ssq_out2 = wsp<float>(s, s->L.ssq_exit) + ((size_t)exit_buf * SB_MAX_W + slot0) * s->L.ssq_ld;
    }
    // W_down overwrites what a still-running exit head reads (its slot's parts and sums of squares)
    if ((rc = exit_buf >= 0 ? join_head_buf(s, exit_buf) : join_head(s))) return rc;
    if ((rc = gemv(s, g, SB_K_DOWN, st))) return rc;

    s->st.layer_sweeps += 1;
    s->st.row_layers += M;
    s->st.weight_bytes += m->layer_bytes;
    s->st.kv_bytes += kv_read;
    if (s->phase_bytes) *s->phase_bytes += m->layer_bytes + kv_read;
    return SB_OK;
}

// Head projection + arg max / confidence for the M rows starting at slot `slot0`.
// VALU path: RMSNorm kernel first.  MFMA path: the last W_down already left
// gain * h and the sums of squares for these slots (run_layer's head_gain).
int run_head(sb_session* s, const void* W, const float* gain, int slot0, int M, HeadArgs h, hipStream_t st,
             bool prenormed = false, int exit_buf = -1) {
    sb_model* m = s->m;
    const sb_config& c = m->cfg;
    const bool mf = m->proj == SB_PROJ_MFMA;
    float* xn = wsp<float>(s, s->L.xn);
    const float* rows = wsp<float>(s, s->L.H) + (size_t)slot0 * c.d_model;
    if (!mf) {
        ProfScope ps(s, SB_K_RMSNORM, (int64_t)M * c.d_model * 8, st);
        HIP_TRY(launch_rmsnorm(rows, gain, xn, nullptr, c.d_model, M, c.d_model, c.rms_eps, st));
    }
    h.partials = wsp<float>(s, s->L.head_part);
    h.round = s->d_round;
    GemvArgs g{};
    g.W = W; g.w_dtype = c.weight_dtype; g.N = c.vocab; g.K = c.d_model; g.x = xn; g.M = M;
    g.xs = wsp<uint16_t>(s, exit_buf == 1 ? s->L.xs_exit2 : s->L.xs_exit) + (size_t)slot0 * c.d_model;
    if (mf && !prenormed) {  // (prenormed: xs already holds the normalised rows)
        g.ssq_in = exit_buf >= 0 ? wsp<float>(s, s->L.ssq_exit) + ((size_t)exit_buf * SB_MAX_W + slot0) * s->L.ssq_ld
                                 : wsp<float>(s, s->L.ssq_attn) + (size_t)slot0 * s->L.ssq_ld;
        g.ssq_nb = c.d_model / 16; g.ssq_ld = s->L.ssq_ld; g.eps = c.rms_eps;
    }
    g.epi = EPI_HEAD; g.head = h;
    int rc = gemv(s, g, h.post == POST_EXIT ? SB_K_EXIT_HEAD : SB_K_FINAL_HEAD, st);
    if (rc) return rc;
    s->st.weight_bytes += m->head_bytes;
    if (s->phase_bytes) *s->phase_bytes += m->head_bytes;
    return SB_OK;
}

// What the embedding kernel leaves for layer 0's QKV projection (MFMA path).
EmbedNorm embed_norm(sb_session* s, int slot0) {
    EmbedNorm en{nullptr, nullptr, nullptr, 0};
    if (s->m->proj == SB_PROJ_MFMA) {
        en.gain = s->m->attn_norm[0];
        en.nx = wsp<uint16_t>(s, s->L.xs_attn) + (size_t)slot0 * s->m->cfg.d_model;
        en.ssq_out = wsp<float>(s, s->L.ssq_attn) + (size_t)slot0 * s->L.ssq_ld;
        en.ssq_ld = s->L.ssq_ld;
    }
    return en;
}

void reset_session(sb_session* s) {
    s->c = 0; s->has_pending = false; s->n_slots = 0; s->n_drafts = 0; s->round_closed = false;
    s->next_embedded = false;
    s->phase_bytes = nullptr;   // (prefill: counted in the totals only)
    s->draft_counter = 0;
    memset(&s->st, 0, sizeof s->st);
}

// One projection of a super-pass (R rows = several prompt passes): k-split GEMM, then its epilogue.
int prefill_proj(sb_session* s, const void* Wp, int rows, int K, const uint16_t* xs, int R, GemmEpiArgs e, int cls) {
    hipStream_t st = s->m->stream;
    GemmArgs g{};
    g.Wp = Wp; g.rows = rows; g.K = K; g.xs = xs; g.plane_rows = s->L.p_rows; g.M = R;
    g.n_pass = (R + SB_PREFILL_ROWS - 1) / SB_PREFILL_ROWS;
    g.part = wsp<float>(s, s->L.p_part); g.S = gemm_splits(rows, K, g.n_pass);
    e.part = g.part; e.S = g.S; e.rows = rows; e.M = R; e.n_pass = g.n_pass; e.plane_rows = s->L.p_rows;
    e.K = K; e.eps = s->m->cfg.rms_eps; e.ssq_ld = s->L.p_ssq_ld;
    if (e.epi == EPI_SWIGLU || e.epi == EPI_STORE) {  // the GEMM finishes the row blocks it owns whole
        g.fused = e.fused = 1 + e.epi;
        g.N = e.N; g.ssq_in = e.ssq_in; g.ssq_nb = e.ssq_nb; g.ssq_ld = e.ssq_ld; g.eps = e.eps;
        g.ys = e.ys; g.y = e.y; g.ldy = e.ldy;
    }
    ProfScope ps(s, cls, (int64_t)rows * K * 2 + (int64_t)R * K * 4 + (int64_t)R * rows * 4, st);
    hipError_t err = launch_prefill_gemm(g, st);
    if (err == hipSuccess) err = launch_prefill_epilogue(e, st);
    if (err != hipSuccess) return fail(SB_EDEVICE, "prompt projection launch (rows=%d K=%d R=%d): %s", rows, K, R,
                                       hipGetErrorString(err));
    return SB_OK;
}

// The prompt through all layers, a super-pass (up to SB_PREFILL_PASSES passes of
// SB_PREFILL_ROWS rows) at a time: per layer one launch per projection over all its rows,
// and one attention launch per pass, in order (a pass attends to the keys of the passes
// before it).  Same layer as run_layer; hidden rows and bf16 planes live in the p_* buffers.
int prefill_gemm_impl(sb_session* s, const int32_t* prompt, int32_t n, int32_t* first_token) {
    sb_model* m = s->m;
    const sb_config& c = m->cfg;
    hipStream_t st = m->stream;
    const int d = c.d_model, f = c.d_ffn, hq = c.n_heads * c.head_dim;
    const int qkv_rows = (c.n_heads + 2 * c.n_kv_heads) * c.head_dim;
    const int nb_d = (d + 255) / 256, PM = SB_PREFILL_ROWS, RS = s->L.p_rows;
    int32_t* toks = wsp<int32_t>(s, s->L.p_tok);
    float* H = wsp<float>(s, s->L.p_H);
    uint16_t* xs = wsp<uint16_t>(s, s->L.p_xs);
    float* ssq = wsp<float>(s, s->L.p_ssq);
    float* qkv = wsp<float>(s, s->L.p_qkv);
    uint16_t* atts = wsp<uint16_t>(s, s->L.p_atts);
    uint16_t* us = wsp<uint16_t>(s, s->L.p_us);
    HIP_TRY(hipMemcpyAsync(toks, prompt, (size_t)n * 4, hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));  // the caller's buffer is pageable: do not return while it is being read
    int rc, R = 0;
    for (int r0 = 0; r0 < n; r0 += RS) {
        R = n - r0 < RS ? n - r0 : RS;
        HIP_TRY(launch_prefill_embed(m->embed, c.weight_dtype, c.vocab, d, toks + r0, R, H, m->attn_norm[0], xs, RS, ssq,
                                     s->L.p_ssq_ld, st));
        for (int l = 0; l < c.n_layers; ++l) {
            GemmEpiArgs e{};
            e.N = qkv_rows; e.epi = EPI_STORE; e.ssq_in = ssq; e.ssq_nb = nb_d; e.y = qkv; e.ldy = qkv_rows;
            if ((rc = prefill_proj(s, m->w_qkv[l], qkv_rows, d, xs, R, e, SB_K_QKV))) return rc;

            int64_t kv_read = 0;
            if (c.kv_dtype == SB_BF16) {  // all rows in one launch, running softmax per query
                AttnArgs a{};
                a.q = qkv; a.rope_cos = m->rope_cos; a.rope_sin = m->rope_sin;
                a.qkv_rows = qkv_rows; a.n_heads = c.n_heads;
                a.kv = s->kv; a.layer = l; a.pos0 = s->c; a.M = R;
                a.out = nullptr; a.out_split = atts; a.split_rows = RS;
                // a block of 64 queries reads the keys and values up to its last row once
                const int G = c.n_heads / c.n_kv_heads, rows_per_block = 64 / G > 0 ? 64 / G : 1;
                for (int q0 = 0; q0 < R; q0 += rows_per_block)
                    kv_read += (int64_t)(s->c + (q0 + rows_per_block < R ? q0 + rows_per_block : R)) * 2 * c.n_kv_heads *
                               c.head_dim * 2;
                ProfScope ps(s, SB_K_ATTN, kv_read, st);
                HIP_TRY(launch_prefill_attention(a, st));
            } else
            for (int p0 = 0; p0 < R; p0 += PM) {
                AttnArgs a{};
                a.q = qkv + (size_t)p0 * qkv_rows; a.rope_cos = m->rope_cos; a.rope_sin = m->rope_sin;
                a.qkv_rows = qkv_rows; a.n_heads = c.n_heads;
                a.kv = s->kv; a.layer = l; a.pos0 = s->c + p0; a.M = R - p0 < PM ? R - p0 : PM;
                a.partials = wsp<float>(s, s->L.p_attn_part); a.max_chunks = s->L.max_chunks;
                a.out = nullptr; a.out_split = atts + (size_t)p0 * hq; a.split_rows = RS;
                const int64_t kvb = (int64_t)(a.pos0 + a.M) * 2 * c.n_kv_heads * c.head_dim * (int64_t)esize(c.kv_dtype);
                kv_read += kvb;
                ProfScope ps(s, SB_K_ATTN, kvb, st);
                HIP_TRY(launch_attention(a, st));
            }

            e = GemmEpiArgs{};
            e.N = d; e.epi = EPI_RESID; e.y = H; e.ldy = d; e.gain = m->ffn_norm[l]; e.nx = xs; e.ssq_out = ssq;
            if ((rc = prefill_proj(s, m->w_o[l], d, hq, atts, R, e, SB_K_WO))) return rc;

            e = GemmEpiArgs{};
            e.N = f; e.epi = EPI_SWIGLU; e.ssq_in = ssq; e.ssq_nb = nb_d; e.ys = us;
            if ((rc = prefill_proj(s, m->w_gate_up[l], 2 * f, d, xs, R, e, SB_K_GATEUP))) return rc;

            e = GemmEpiArgs{};
            e.N = d; e.epi = EPI_RESID; e.y = H; e.ldy = d; e.ssq_out = ssq;
            if (l + 1 < c.n_layers) { e.gain = m->attn_norm[l + 1]; e.nx = xs; }
            if ((rc = prefill_proj(s, m->w_down[l], d, f, us, R, e, SB_K_DOWN))) return rc;

            s->st.layer_sweeps += 1;
            s->st.row_layers += R;
            s->st.weight_bytes += m->layer_bytes;
            s->st.kv_bytes += kv_read;
        }
        s->c += R;
    }
    // final head on the last prompt row: normalise it into slot 0's projection input
    {
        ProfScope ps(s, SB_K_RMSNORM, (int64_t)d * 8, st);
        HIP_TRY(launch_rmsnorm(H + (size_t)(R - 1) * d, m->final_norm, wsp<float>(s, s->L.xn),
                               wsp<uint16_t>(s, s->L.xs_exit), d, 1, d, c.rms_eps, st));
    }
    HeadArgs h{};
    h.T = 1.0f; h.post = POST_NONE;
    h.argmax_out = s->d_round->g; h.conf_out = s->d_round->gconf;
    h.logits = s->debug ? wsp<float>(s, s->L.logits_final) : nullptr;
    if ((rc = run_head(s, m->lm_head, m->final_norm, 0, 1, h, st, true))) return rc;
    s->st.final_head_sweeps++;
    if ((rc = readback(s))) return rc;
    s->pending = s->h_round->g[0];
    s->has_pending = true;
    *first_token = s->pending;
    return SB_OK;
}

int prefill_impl(sb_session* s, const int32_t* prompt, int32_t n, int32_t* first_token) {
    sb_model* m = s->m;
    const sb_config& c = m->cfg;
    if (!prompt || !first_token) return fail(SB_EINVAL, "prefill: NULL argument");
    if (n < 1) return fail(SB_EINVAL, "prefill: empty prompt");
    if (n > c.max_seq) return fail(SB_ECAPACITY, "prefill: prompt of %d tokens exceeds max_seq %d", n, c.max_seq);
    for (int i = 0; i < n; ++i)
        if (prompt[i] < 0 || prompt[i] >= c.vocab) return fail(SB_EINVAL, "prefill: token id %d out of range", prompt[i]);
    {
        int jrc = join_head(s);
        if (jrc) return jrc;
    }
    reset_session(s);
    if (s->L.prefill_gemm && m->packed) return prefill_gemm_impl(s, prompt, n, first_token);
    float* H = wsp<float>(s, s->L.H);
    int last_rows = 0;
    for (int i0 = 0; i0 < n; i0 += SB_MAX_W) {
        int M = n - i0 < SB_MAX_W ? n - i0 : SB_MAX_W;
        RowToks t;
        for (int r = 0; r < SB_MAX_W; ++r) t.tok[r] = r < M ? prompt[i0 + r] : 0;
        HIP_TRY(launch_embed(m->embed, c.weight_dtype, c.vocab, c.d_model, H, M, t, s->d_round->slot_tok, nullptr,
                             embed_norm(s, 0), m->stream));
        const bool last_chunk = i0 + M >= n;
        for (int l = 0; l < c.n_layers; ++l) {
            int rc = run_layer(s, l, 0, M, (last_chunk && l == c.n_layers - 1) ? m->final_norm : nullptr);
            if (rc) return rc;
        }
        s->c += M;
        last_rows = M;
    }
    HeadArgs h{};
    h.T = 1.0f; h.post = POST_NONE;
    h.argmax_out = s->d_round->g; h.conf_out = s->d_round->gconf;
    h.logits = s->debug ? wsp<float>(s, s->L.logits_final) : nullptr;
    int rc = run_head(s, m->lm_head, m->final_norm, last_rows - 1, 1, h, m->stream);
    if (rc) return rc;
    s->st.final_head_sweeps++;
    if ((rc = readback(s))) return rc;
    s->pending = s->h_round->g[0];
    s->has_pending = true;
    *first_token = s->pending;
    return SB_OK;
}

// sync: read the step's result back before returning (always done when the exit
// decision is computed on the device, since it gates the next layer's launch).
int draft_step_impl(sb_session* s, const sb_params* p, sb_draft_result* out, bool sync) {
    int rc = check_params(s, p);
    if (rc) return rc;
    sb_model* m = s->m;
    const sb_config& c = m->cfg;
    if (!s->has_pending) return fail(SB_ESTATE, "draft_step: no pending token (prefill first)");
    if (s->round_closed) return fail(SB_ESTATE, "draft_step: a bound was hit, call sb_verify");
    if (s->n_slots >= p->w_max) return fail(SB_ESTATE, "draft_step: w_max rows are open");
    if (s->c + s->n_slots >= c.max_seq) return fail(SB_ECAPACITY, "draft_step: KV capacity exceeded");
    const int64_t k = s->draft_counter;
    int forced = (p->forced_exit && k < p->n_forced) ? p->forced_exit[k] : -1;
    int over = (p->forced_draft && k < p->n_forced) ? p->forced_draft[k] : -1;
    if (forced > p->d_max) return fail(SB_EINVAL, "forced_exit[%lld] = %d exceeds d_max", (long long)k, forced);
    if (forced >= 1 && p->head_mask && !((p->head_mask >> (forced - 1)) & 1u))
        return fail(SB_EINVAL, "forced_exit[%lld] = %d names a layer outside head_mask", (long long)k, forced);
    if (over >= c.vocab) return fail(SB_EINVAL, "forced_draft[%lld] = %d out of range", (long long)k, over);
    if (forced < -1) forced = -1;
    if (over < -1) over = -1;
    const bool computed = forced < 0 || p->exit_readback != 0;   // the exit decision is read from the device after each head

    // the previous step's last exit head wrote the token this step embeds
    if ((rc = join_head(s))) return rc;
    const bool overlap = !computed && m->proj == SB_PROJ_MFMA && s->head_stream;
    const int idx = s->n_slots;
    RowToks t;
    for (int r = 0; r < SB_MAX_W; ++r) t.tok[r] = 0;
    t.tok[0] = idx == 0 ? s->pending : s->draft_host[idx - 1];  // -1: the id is on the device only
    float* Hrow = wsp<float>(s, s->L.H) + (size_t)idx * c.d_model;
    if (s->phase_timing && idx == 0) HIP_TRY(hipEventRecord(s->ev_ph[0], m->stream));   // the round begins
    if (!(idx > 0 && s->next_embedded))   // (else the head merge that drafted this row's token has embedded it)
        HIP_TRY(launch_embed(m->embed, c.weight_dtype, c.vocab, c.d_model, Hrow, 1, t, s->d_round->slot_tok + idx,
                             &s->d_round->exit_flag, embed_norm(s, idx), m->stream));
    s->next_embedded = false;
    s->phase_bytes = &s->st.draft_bytes;
    // a draft that exits is embedded as the next row by its own head merge, if a next step can follow
    const bool embed_next = s->n_drafts + 1 < p->w_max && idx + 1 < SB_MAX_W;
    s->draft_counter++;
    s->st.draft_steps++;
    s->n_slots++;
    s->reached[idx] = 0;
    s->exit_layer[idx] = 0;
    s->draft_host[idx] = -1;

    int exit_at = 0, n_heads_run = 0;
    for (int l = 1; l <= p->d_max; ++l) {
        int j0 = idx;
        while (j0 > 0 && s->reached[j0 - 1] == l - 1) --j0;
        const bool has_head = !p->head_mask || ((p->head_mask >> (l - 1)) & 1u);
        const int xb = overlap ? (l & 1) : -1;   // exit-operand buffer of this layer's head
        if ((rc = run_layer(s, l - 1, j0, idx - j0 + 1, has_head ? m->exit_norm[l - 1] : nullptr, xb))) return rc;
        for (int j = j0; j <= idx; ++j) s->reached[j] = l;
        if (!has_head) continue;  // (variant: no exit test at this layer)
        ++n_heads_run;
        HeadArgs h{};
        h.T = p->T[l - 1]; h.post = POST_EXIT; h.slot = idx; h.layer = l; h.forced_exit = forced; h.forced_draft = over;
        h.threshold = p->threshold;
        h.logits = s->debug ? wsp<float>(s, s->L.logits_exit) + (size_t)(l - 1) * c.vocab : nullptr;
        if (embed_next) {
            h.embed_E = m->embed; h.embed_dtype = c.weight_dtype; h.embed_vocab = c.vocab; h.embed_d = c.d_model;
            h.embed_H = Hrow + c.d_model;
            h.embed_en = embed_norm(s, idx + 1);
        }
        if (computed) { h.note = s->note_d; h.note_seq = ++s->note_seq; }   // the host's next launch waits for this decision
        // The head only reads what W_down left for it, so it can run beside the next layer on the
        // second stream -- except the head at which the row exits: the next step starts from its
        // result, so it stays on the main stream (no hop between streams on the critical path).
        if (overlap && l != forced) {
            // the head only reads what W_down left for it: let it run beside the next layer
            const unsigned e = s->ev_i++ & 3;
            HIP_TRY(hipEventRecord(s->ev_main[e], m->stream));
            HIP_TRY(hipStreamWaitEvent(s->head_stream, s->ev_main[e], 0));
            if ((rc = run_head(s, m->exit_head[l - 1], m->exit_norm[l - 1], idx, 1, h, s->head_stream, false, xb))) return rc;
            HIP_TRY(hipEventRecord(s->ev_head[e], s->head_stream));
            s->head_pending[xb] = true;
            s->head_pending_ev[xb] = (int)e;
        } else {
            // (the merges write one round record: this head's comes after those of the heads still running)
            if ((rc = join_head(s))) return rc;
            if ((rc = run_head(s, m->exit_head[l - 1], m->exit_norm[l - 1], idx, 1, h, m->stream, false, xb))) return rc;
        }
        s->st.head_evals++;
        if (computed) {
            if ((rc = wait_note(s, h.note_seq, idx))) return rc;
            if (s->h_round->exit_flag) { exit_at = l; break; }
        } else if (l == forced) {
            exit_at = l;
            break;
        }
    }
    if (!computed && sync && n_heads_run > 0)
        if ((rc = readback(s))) return rc;
    const bool have = (computed || sync) && n_heads_run > 0;

    sb_draft_result res{-1, 0, SB_DEPTH_BOUND, 0.f};
    if (have) res.confidence = s->h_round->conf[idx];
    if (exit_at) {
        s->exit_layer[idx] = exit_at;
        s->next_embedded = embed_next;
        s->draft_host[idx] = over >= 0 ? over : (have ? s->h_round->drafts[idx] : -1);
        s->n_drafts++;
        s->st.drafts++;
        s->st.exit_hist[exit_at]++;
        res.token = s->draft_host[idx];
        res.exit_layer = exit_at;
        res.status = s->n_drafts == p->w_max ? SB_WIDTH_BOUND : SB_EXITED;
    } else {
        s->st.exit_hist[0]++;
    }
    if (res.status != SB_EXITED) s->round_closed = true;
    if (out) *out = res;
    return SB_OK;
}

int verify_impl(sb_session* s, const sb_params* p, sb_verify_result* out) {
    int rc = check_params(s, p);
    if (rc) return rc;
    if (s->n_slots == 0) return fail(SB_ESTATE, "verify: no open row");
    sb_model* m = s->m;
    const sb_config& c = m->cfg;
    if ((rc = join_head(s))) return rc;
    const bool pt = s->phase_timing;
    if (pt) HIP_TRY(hipEventRecord(s->ev_ph[1], m->stream));   // drafting (with its last exit head) is over
    const int M = s->n_slots, D = s->reached[0];
    for (int j = 1; j < M; ++j)
        if (s->reached[j] > s->reached[j - 1]) return fail(SB_ESTATE, "verify: reached layers not monotone");
    // align: rows standing below the deepest layer reached catch up (Appendix A)
    s->phase_bytes = &s->st.align_bytes;
    for (int l = 2; l <= D; ++l) {
        int j0 = M;
        while (j0 > 0 && s->reached[j0 - 1] == l - 1) --j0;
        if (j0 == M) continue;
        if ((rc = run_layer(s, l - 1, j0, M - j0, nullptr))) return rc;
        for (int j = j0; j < M; ++j) s->reached[j] = l;
    }
    if (pt) HIP_TRY(hipEventRecord(s->ev_ph[2], m->stream));   // aligned
    s->phase_bytes = &s->st.verify_bytes;
    // one parallel pass of all rows through the remaining layers
    for (int l = D + 1; l <= c.n_layers; ++l) {
        if ((rc = run_layer(s, l - 1, 0, M, l == c.n_layers ? m->final_norm : nullptr))) return rc;
        for (int j = 0; j < M; ++j) s->reached[j] = l;
    }
    const bool sampling = p->sample_temperature > 0.f;
    if (sampling && p->n_sample_u < 2 * (int64_t)(s->c + M))
        return fail(SB_EINVAL, "verify: sample_u has %lld entries, the rows of this round need %lld", (long long)p->n_sample_u,
                    2 * (long long)(s->c + M));
    HeadArgs h{};
    h.T = 1.0f; h.post = sampling ? POST_NONE : POST_ACCEPT; h.n_drafts = s->n_drafts;
    h.logits = (s->debug || sampling) ? wsp<float>(s, s->L.logits_final) : nullptr;
    if (sampling) { h.argmax_out = s->d_round->g; h.conf_out = s->d_round->gconf; }   // (overwritten by the acceptance kernel)
    if ((rc = join_head(s))) return rc;
    if ((rc = run_head(s, m->lm_head, m->final_norm, 0, M, h, m->stream))) return rc;
    if (sampling) {
        SampleArgs sa{};
        sa.logits = wsp<float>(s, s->L.logits_final); sa.wts = wsp<float>(s, s->L.sample_w); sa.V = c.vocab; sa.M = M; sa.n_drafts = s->n_drafts;
        sa.temp = p->sample_temperature; sa.top_p = p->top_p; sa.round = s->d_round;
        for (int i = 0; i < M; ++i) {
            sa.ua[i] = p->sample_u[2 * (int64_t)(s->c + i)];
            sa.ur[i] = p->sample_u[2 * (int64_t)(s->c + i) + 1];
        }
        HIP_TRY(launch_sample_accept(sa, m->stream));
    }
    s->st.final_head_sweeps++;
    if (pt) HIP_TRY(hipEventRecord(s->ev_ph[3], m->stream));   // verified
    const double tw0 = now_ms();
    HIP_TRY(hipMemcpyAsync(s->h_round, s->d_round, sizeof(DevRound), hipMemcpyDeviceToHost, m->stream));
    if (pt) HIP_TRY(hipEventRecord(s->ev_ph[4], m->stream));
    HIP_TRY(hipStreamSynchronize(m->stream));
    s->st.host_wait_ms += now_ms() - tw0;
    if (pt) {
        double* acc[4] = {&s->st.gpu_draft_ms, &s->st.gpu_align_ms, &s->st.gpu_verify_ms, &s->st.gpu_readback_ms};
        for (int i = 0; i < 4; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, s->ev_ph[i], s->ev_ph[i + 1]) == hipSuccess) *acc[i] += ms;
        }
    }
    const DevRound& R = *s->h_round;
    if (R.n_emit < 1 || R.n_emit > M) return fail(SB_EDEVICE, "verify: device returned n_emit = %d", R.n_emit);
    sb_verify_result res{};
    res.n_rows = M; res.n_drafts = s->n_drafts; res.n_matched = R.n_matched; res.n_emit = R.n_emit; res.align_layer = D;
    for (int i = 0; i < SB_MAX_W; ++i) res.tokens[i] = i < M ? R.g[i] : -1;
    for (int i = 0; i < SB_MAX_W; ++i) res.accept_prob[i] = (sampling && i < M) ? R.gconf[i] : 0.f;
    // commit the emitted rows; KV entries of the other rows are simply left
    // beyond the committed length and overwritten by the next round
    s->c += R.n_emit;
    s->pending = R.g[R.n_emit - 1];
    s->n_slots = 0; s->n_drafts = 0; s->round_closed = false; s->next_embedded = false;
    s->st.rounds++; s->st.emitted += R.n_emit; s->st.accept_hist[R.n_emit]++;
    if (out) *out = res;
    return SB_OK;
}

hipError_t sync_all(sb_session* s);

// A launch or copy failed in the middle of a round: what the rows of the round hold on the
// device is no longer what the host's bookkeeping says, so the round is dropped as a whole.
// Committed positions (< c) were not touched by it: rows only write positions >= c.
int round_guard(sb_session* s, int rc) {
    if (rc != SB_EDEVICE) return rc;
    const std::string msg = g_err;
    (void)sync_all(s);
    s->draft_counter -= s->n_slots;   // the abandoned steps' entries of the forced schedule are taken again
    if (s->draft_counter < 0) s->draft_counter = 0;
    s->n_slots = 0; s->n_drafts = 0; s->round_closed = false; s->next_embedded = false;
    g_err = msg + " (the open round was abandoned)";
    return rc;
}

hipError_t sync_all(sb_session* s) {
    hipError_t e = hipStreamSynchronize(s->m->stream);
    if (e == hipSuccess && s->head_stream) e = hipStreamSynchronize(s->head_stream);
    s->head_pending[0] = s->head_pending[1] = false;
    return e;
}

void free_session_resources(sb_session* s) {
    if (s->h_round) (void)hipHostFree(s->h_round);
    if (s->note_h) (void)hipHostFree(s->note_h);
    for (int i = 0; i < 5; ++i)
        if (s->ev_ph[i]) { (void)hipEventDestroy(s->ev_ph[i]); s->ev_ph[i] = nullptr; }
    for (int i = 0; i < 4; ++i) {
        if (s->ev_main[i]) (void)hipEventDestroy(s->ev_main[i]);
        if (s->ev_head[i]) (void)hipEventDestroy(s->ev_head[i]);
    }
    if (s->head_stream) (void)hipStreamDestroy(s->head_stream);
    for (hipEvent_t x : s->prof_ev) (void)hipEventDestroy(x);
    s->prof_ev.clear();
    for (hipEvent_t x : s->prof_cal) (void)hipEventDestroy(x);
    s->prof_cal.clear();
}

// Rounds of draft steps + verification until *cnt == max_new or eos.  While the
// exit decisions are forced the host knows the round's shape in advance, so a
// whole round is enqueued without waiting and read back once, after verification.
int decode_impl(sb_session* s, const sb_params* p, int32_t* out_tokens, int* cnt_io, int max_new) {
    int cnt = *cnt_io, rc;
    double t1 = now_ms();
    while (cnt < max_new && !(p->eos_id >= 0 && cnt > 0 && out_tokens[cnt - 1] == p->eos_id)) {
        sb_draft_result dr;
        const double th0 = now_ms();
        do {
            if ((rc = draft_step_impl(s, p, &dr, false))) return round_guard(s, rc);
        } while (dr.status == SB_EXITED);
        const double th1 = now_ms(), w0 = s->st.host_wait_ms;
        sb_verify_result vr;
        if ((rc = verify_impl(s, p, &vr))) return round_guard(s, rc);
        s->st.host_draft_ms += th1 - th0;
        s->st.host_verify_ms += (now_ms() - th1) - (s->st.host_wait_ms - w0);
        int take = 0;
        while (take < vr.n_emit && cnt < max_new) {
            out_tokens[cnt++] = vr.tokens[take++];
            if (p->eos_id >= 0 && out_tokens[cnt - 1] == p->eos_id) break;
        }
        if (take < vr.n_emit) {  // emission cut short: give the uncommitted positions back
            s->c -= vr.n_emit - take;
            s->st.emitted -= vr.n_emit - take;
            s->pending = out_tokens[cnt - 1];
        }
    }
    s->st.decode_ms = now_ms() - t1;
    *cnt_io = cnt;
    return SB_OK;
}

}  // namespace sbhost

// ============================================================================ C ABI
extern "C" {

const char* sb_last_error(void) { return g_err.c_str(); }

int32_t sb_temperature_schedule(double alpha, int32_t L, int32_t n, float* T) {
    if (!T || L < 1 || n < 0) return fail(SB_EINVAL, "temperature_schedule: bad argument");
    for (int l = 1; l <= n; ++l) T[l - 1] = (float)(1.0 + alpha * (1.0 - (double)l / (double)L));
    return SB_OK;
}

int32_t sb_query_sizes(const sb_config* cfg, sb_sizes* out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!out) return fail(SB_EINVAL, "query_sizes: out is NULL");
    out->kv_pool_bytes = kv_pool_bytes(cfg);
    out->workspace_bytes = ws_layout(cfg).total;
    out->packed_weight_bytes = packed_weight_bytes(cfg);
    return SB_OK;
}

int32_t sb_load_model(const sb_config* cfg, const sb_weights* w, void* stream, sb_model** out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!w || !out) return fail(SB_EINVAL, "load_model: NULL argument");
    if (!w->embed || !w->final_norm || !w->lm_head || !w->attn_norm || !w->w_qkv || !w->w_o || !w->ffn_norm ||
        !w->w_gate_up || !w->w_down)
        return fail(SB_EINVAL, "load_model: NULL weight pointer");
    if (cfg->n_exit_heads > 0 && (!w->exit_norm || !w->exit_head)) return fail(SB_EINVAL, "load_model: NULL exit heads");
    const size_t pack_need = packed_weight_bytes(cfg);
    if (w->packed && pack_need) {
        if ((uintptr_t)w->packed & 255) return fail(SB_EINVAL, "load_model: the packed-weight buffer must be 256-byte aligned");
        if (w->packed_bytes < pack_need)
            return fail(SB_ENOMEM, "load_model: packed-weight buffer too small (%zu < %zu)", w->packed_bytes, pack_need);
    }
    sb_model* m = new sb_model();
    m->cfg = *cfg;
    m->embed = w->embed; m->lm_head = w->lm_head; m->final_norm = w->final_norm;
    for (int l = 0; l < cfg->n_layers; ++l) {
        if (!w->attn_norm[l] || !w->w_qkv[l] || !w->w_o[l] || !w->ffn_norm[l] || !w->w_gate_up[l] || !w->w_down[l]) {
            delete m;
            return fail(SB_EINVAL, "load_model: NULL weight pointer in layer %d", l);
        }
        m->attn_norm.push_back(w->attn_norm[l]); m->w_qkv.push_back(w->w_qkv[l]); m->w_o.push_back(w->w_o[l]);
        m->ffn_norm.push_back(w->ffn_norm[l]); m->w_gate_up.push_back(w->w_gate_up[l]);
        m->w_down.push_back(w->w_down[l]);
    }
    for (int l = 0; l < cfg->n_exit_heads; ++l) {
        if (!w->exit_norm[l] || !w->exit_head[l]) {
            delete m;
            return fail(SB_EINVAL, "load_model: NULL exit head %d", l);
        }
        m->exit_norm.push_back(w->exit_norm[l]); m->exit_head.push_back(w->exit_head[l]);
    }
    m->stream = (hipStream_t)stream;
    m->proj = resolve_proj(cfg);
    m->packed = m->proj == SB_PROJ_MFMA_PACKED;
    if (m->packed) m->proj = SB_PROJ_MFMA;
    const int64_t es = (int64_t)esize(cfg->weight_dtype), d = cfg->d_model, f = cfg->d_ffn;
    const int64_t qkv_rows = (int64_t)(cfg->n_heads + 2 * cfg->n_kv_heads) * cfg->head_dim;
    m->layer_bytes = es * (qkv_rows * d + d * (int64_t)cfg->n_heads * cfg->head_dim + 3 * f * d);
    m->head_bytes = es * (int64_t)cfg->vocab * d;
    // rotary table: angle = pos * base^(-2i/hd) in double, cos/sin rounded to float
    const int half = cfg->head_dim / 2;
    std::vector<float> hc((size_t)cfg->max_seq * half), hs((size_t)cfg->max_seq * half);
    for (int p = 0; p < cfg->max_seq; ++p)
        for (int i = 0; i < half; ++i) {
            double theta = std::pow((double)cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
            double a = (double)p * theta;
            hc[(size_t)p * half + i] = (float)std::cos(a);
            hs[(size_t)p * half + i] = (float)std::sin(a);
        }
    m->rope_cos = m->rope_sin = nullptr;
    hipError_t e = hipMalloc((void**)&m->rope_cos, hc.size() * 4);
    if (e == hipSuccess) e = hipMalloc((void**)&m->rope_sin, hs.size() * 4);
    if (e == hipSuccess) e = hipMemcpy(m->rope_cos, hc.data(), hc.size() * 4, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(m->rope_sin, hs.data(), hs.size() * 4, hipMemcpyHostToDevice);
    // tile-packed copies of the projection matrices
    if (e == hipSuccess && m->packed) {
        const int dm = cfg->d_model, ff = cfg->d_ffn, hq = cfg->n_heads * cfg->head_dim, V = cfg->vocab;
        // one buffer for all packed matrices: the caller's, or one the model owns
        char* pbase = (char*)w->packed;
        if (!pbase) {
            e = hipMalloc((void**)&pbase, pack_need);
            if (e == hipSuccess) m->owned.push_back(pbase);
        }
        size_t poff = 0;
        auto pack = [&](const void*& W, int N, int K) {
            if (e != hipSuccess) return;
            void* P = pbase + poff;
            poff += align_up((size_t)N * K * 2, 256);
            e = launch_repack(W, P, N, K, m->stream);
            W = P;
        };
        for (int l = 0; l < cfg->n_layers; ++l) {
            pack(m->w_qkv[l], (int)qkv_rows, dm);
            pack(m->w_o[l], dm, hq);
            pack(m->w_gate_up[l], 2 * ff, dm);
            pack(m->w_down[l], dm, ff);
        }
        for (int l = 0; l < cfg->n_exit_heads; ++l) pack(m->exit_head[l], V, dm);
        pack(m->lm_head, V, dm);
        if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    }
    if (e != hipSuccess) {
        if (m->rope_cos) (void)hipFree(m->rope_cos);
        if (m->rope_sin) (void)hipFree(m->rope_sin);
        for (void* p : m->owned) (void)hipFree(p);
        delete m;
        return fail(e == hipErrorOutOfMemory ? SB_ENOMEM : SB_EDEVICE, "load_model: %s", hipGetErrorString(e));
    }
    *out = m;
    return SB_OK;
}

void sb_free_model(sb_model* m) {
    if (!m) return;
    (void)hipFree(m->rope_cos);
    (void)hipFree(m->rope_sin);
    for (void* p : m->owned) (void)hipFree(p);
    delete m;
}

int32_t sb_new_session(sb_model* m, void* kv_pool, size_t kv_bytes, void* workspace, size_t ws_bytes,
                       const int32_t* page_order, sb_session** out) {
    if (!m || !out) return fail(SB_EINVAL, "new_session: NULL argument");
    if (!kv_pool || !workspace) return fail(SB_EINVAL, "new_session: NULL device buffer");
    if (((uintptr_t)kv_pool & 255) || ((uintptr_t)workspace & 255))
        return fail(SB_EINVAL, "new_session: buffers must be 256-byte aligned");
    WsLayout L = ws_layout(&m->cfg);
    if (kv_bytes < kv_pool_bytes(&m->cfg)) return fail(SB_ENOMEM, "new_session: kv_pool too small (%zu < %zu)", kv_bytes, kv_pool_bytes(&m->cfg));
    if (ws_bytes < L.total) return fail(SB_ENOMEM, "new_session: workspace too small (%zu < %zu)", ws_bytes, L.total);
    std::vector<int32_t> table(L.n_pages);
    if (page_order) {
        std::vector<char> seen(L.n_pages, 0);
        for (int i = 0; i < L.n_pages; ++i) {
            int32_t pg = page_order[i];
            if (pg < 0 || pg >= L.n_pages || seen[pg]) return fail(SB_EINVAL, "new_session: page_order is not a permutation");
            seen[pg] = 1;
            table[i] = pg;
        }
    } else {
        for (int i = 0; i < L.n_pages; ++i) table[i] = i;
    }
    sb_session* s = new sb_session();
    s->m = m; s->ws = (char*)workspace; s->L = L;
    s->d_round = wsp<DevRound>(s, L.round);
    s->kv.pool = kv_pool; s->kv.table = wsp<int32_t>(s, L.table); s->kv.n_pages = L.n_pages;
    s->kv.n_kv_heads = m->cfg.n_kv_heads; s->kv.head_dim = m->cfg.head_dim; s->kv.kv_dtype = m->cfg.kv_dtype;
    s->debug = false;
    s->prof_mask = 0;
    s->prof_used = 0;
    s->prof_every = 1;
    s->head_stream = nullptr;
    s->ev_i = 0;
    s->head_pending[0] = s->head_pending[1] = false;
    s->head_pending_ev[0] = s->head_pending_ev[1] = 0;
    for (int i = 0; i < 4; ++i) { s->ev_main[i] = nullptr; s->ev_head[i] = nullptr; }
    s->h_round = nullptr;
    s->note_h = nullptr; s->note_d = nullptr; s->note_seq = 0;
    s->phase_timing = false;
    s->fail_countdown = 0;
    for (int i = 0; i < 5; ++i) s->ev_ph[i] = nullptr;
    reset_session(s);
    hipError_t e = hipHostMalloc((void**)&s->h_round, sizeof(DevRound), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc((void**)&s->note_h, 64, hipHostMallocMapped | hipHostMallocCoherent);
    if (e == hipSuccess) { memset(s->note_h, 0, 64); e = hipHostGetDevicePointer((void**)&s->note_d, s->note_h, 0); }
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&s->head_stream, hipStreamNonBlocking);  // default priority
    for (int i = 0; i < 4 && e == hipSuccess; ++i) {
        e = hipEventCreateWithFlags(&s->ev_main[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&s->ev_head[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipMemcpyAsync(wsp<int32_t>(s, L.table), table.data(), (size_t)L.n_pages * 4, hipMemcpyHostToDevice, m->stream);
    if (e == hipSuccess) e = launch_fill_u32(reinterpret_cast<uint32_t*>(s->d_round), sizeof(DevRound) / 4, 0u, m->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
    if (e != hipSuccess) {
        free_session_resources(s);
        delete s;
        return fail(SB_EDEVICE, "new_session: %s", hipGetErrorString(e));
    }
    memset(s->h_round, 0, sizeof(DevRound));
    *out = s;
    return SB_OK;
}

void sb_free_session(sb_session* s) {
    if (!s) return;
    (void)sync_all(s);
    free_session_resources(s);
    delete s;
}

int32_t sb_prefill(sb_session* s, const int32_t* prompt, int32_t n, int32_t* first_token) {
    if (!s) return fail(SB_EINVAL, "prefill: session is NULL");
    return prefill_impl(s, prompt, n, first_token);
}

int32_t sb_draft_step(sb_session* s, const sb_params* p, sb_draft_result* out) {
    if (!s || !out) return fail(SB_EINVAL, "draft_step: NULL argument");
    return round_guard(s, draft_step_impl(s, p, out, true));
}

int32_t sb_verify(sb_session* s, const sb_params* p, sb_verify_result* out) {
    if (!s || !out) return fail(SB_EINVAL, "verify: NULL argument");
    return round_guard(s, verify_impl(s, p, out));
}

int32_t sb_generate(sb_session* s, const int32_t* prompt, int32_t n, int32_t max_new, const sb_params* p,
                    int32_t* out_tokens, int32_t out_cap, int32_t* n_out, sb_stats* stats) {
    if (!s) return fail(SB_EINVAL, "generate: session is NULL");
    int rc = check_params(s, p);
    if (rc) return rc;
    if (!out_tokens || !n_out || max_new < 1 || out_cap < max_new) return fail(SB_EINVAL, "generate: bad output buffer");
    if ((int64_t)n + max_new + p->w_max > s->m->cfg.max_seq)
        return fail(SB_ECAPACITY, "generate: n + max_new + w_max = %lld exceeds max_seq %d",
                    (long long)n + max_new + p->w_max, s->m->cfg.max_seq);
    double t0 = now_ms();
    int32_t tok;
    if ((rc = prefill_impl(s, prompt, n, &tok))) return rc;
    double t1 = now_ms();
    out_tokens[0] = tok;
    int cnt = 1;
    if ((rc = decode_impl(s, p, out_tokens, &cnt, max_new))) return rc;
    s->st.prefill_ms = t1 - t0;
    *n_out = cnt;
    if (stats) *stats = s->st;
    return SB_OK;
}

int32_t sb_decode(sb_session* s, int32_t max_new, const sb_params* p, int32_t* out_tokens, int32_t out_cap,
                  int32_t* n_out, sb_stats* stats) {
    if (!s) return fail(SB_EINVAL, "decode: session is NULL");
    int rc = check_params(s, p);
    if (rc) return rc;
    if (!out_tokens || !n_out || max_new < 1 || out_cap < max_new) return fail(SB_EINVAL, "decode: bad output buffer");
    if (!s->has_pending) return fail(SB_ESTATE, "decode: no pending token (prefill first)");
    if (s->n_slots) return fail(SB_ESTATE, "decode: a round is open, call sb_verify first");
    if ((int64_t)s->c + max_new + p->w_max > s->m->cfg.max_seq)
        return fail(SB_ECAPACITY, "decode: committed + max_new + w_max = %lld exceeds max_seq %d",
                    (long long)s->c + max_new + p->w_max, s->m->cfg.max_seq);
    int cnt = 0;
    if ((rc = decode_impl(s, p, out_tokens, &cnt, max_new))) return rc;
    *n_out = cnt;
    if (stats) *stats = s->st;
    return SB_OK;
}

int32_t sb_rewind(sb_session* s, int32_t n_keep, int32_t pending_token, int64_t draft_counter) {
    if (!s) return fail(SB_EINVAL, "rewind: session is NULL");
    if (n_keep < 1 || n_keep > s->c) return fail(SB_EINVAL, "rewind: n_keep must be in 1..%d", s->c);
    if (pending_token < 0 || pending_token >= s->m->cfg.vocab) return fail(SB_EINVAL, "rewind: token id out of range");
    if (draft_counter < 0) return fail(SB_EINVAL, "rewind: draft_counter < 0");
    HIP_TRY(sync_all(s));
    reset_session(s);
    s->c = n_keep;
    s->pending = pending_token;
    s->has_pending = true;
    s->draft_counter = draft_counter;
    return SB_OK;
}

int32_t sb_profile_begin(sb_session* s, uint32_t class_mask, int32_t max_launches, int32_t sample_every) {
    if (!s) return fail(SB_EINVAL, "profile_begin: session is NULL");
    if (max_launches < 1 || max_launches > (1 << 22)) return fail(SB_EINVAL, "profile_begin: max_launches out of range");
    if (sample_every < 1) return fail(SB_EINVAL, "profile_begin: sample_every must be >= 1");
    if (!s->prof_ev.empty()) return fail(SB_ESTATE, "profile_begin: timing already running");
    s->prof_ev.reserve((size_t)max_launches * 2);
    for (int i = 0; i < max_launches * 2; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) {
            for (hipEvent_t x : s->prof_ev) (void)hipEventDestroy(x);
            s->prof_ev.clear();
            return fail(SB_ENOMEM, "profile_begin: cannot create %d events", max_launches * 2);
        }
        s->prof_ev.push_back(e);
    }
    s->prof_cls.assign(max_launches, 0);
    s->prof_bytes.assign(max_launches, 0);
    s->prof_used = 0;
    s->prof_every = sample_every;
    for (int k = 0; k < SB_K_COUNT; ++k) s->prof_seen[k] = 0;
    // calibration: a few event pairs with nothing between them
    s->prof_cal.clear();
    for (int i = 0; i < 2 * 16; ++i) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) break;
        s->prof_cal.push_back(e);
    }
    for (size_t i = 0; i + 1 < s->prof_cal.size(); i += 2) {
        (void)hipEventRecord(s->prof_cal[i], s->m->stream);
        (void)hipEventRecord(s->prof_cal[i + 1], s->m->stream);
    }
    s->prof_mask = class_mask;
    return SB_OK;
}

int32_t sb_profile_end(sb_session* s, int64_t* launches, double* total_ms, int64_t* bytes, double* empty_pair_ms) {
    if (!s || !launches || !total_ms || !bytes) return fail(SB_EINVAL, "profile_end: NULL argument");
    if (s->prof_ev.empty()) return fail(SB_ESTATE, "profile_end: timing is not running");
    s->prof_mask = 0;
    hipError_t e = sync_all(s);
    for (int k = 0; k < SB_K_COUNT; ++k) { launches[k] = 0; total_ms[k] = 0.0; bytes[k] = 0; }
    for (size_t i = 0; i < s->prof_used && e == hipSuccess; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, s->prof_ev[2 * i], s->prof_ev[2 * i + 1]);
        launches[s->prof_cls[i]]++;
        total_ms[s->prof_cls[i]] += ms;
        bytes[s->prof_cls[i]] += s->prof_bytes[i];
    }
    double cal = 0.0;
    int ncal = 0;
    for (size_t i = 0; i + 1 < s->prof_cal.size() && e == hipSuccess; i += 2) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, s->prof_cal[i], s->prof_cal[i + 1]) == hipSuccess && i >= 4) { cal += ms; ++ncal; }
    }
    if (empty_pair_ms) *empty_pair_ms = ncal ? cal / ncal : 0.0;
    for (hipEvent_t x : s->prof_cal) (void)hipEventDestroy(x);
    s->prof_cal.clear();
    for (hipEvent_t x : s->prof_ev) (void)hipEventDestroy(x);
    s->prof_ev.clear();
    s->prof_used = 0;
    if (e != hipSuccess) return fail(SB_EDEVICE, "profile_end: %s", hipGetErrorString(e));
    return SB_OK;
}

int32_t sb_phase_timing(sb_session* s, int32_t on) {
    if (!s) return fail(SB_EINVAL, "phase_timing: session is NULL");
    if (on && !s->ev_ph[0])
        for (int i = 0; i < 5; ++i)
            if (hipEventCreate(&s->ev_ph[i]) != hipSuccess) {
                for (int j = 0; j < i; ++j) { (void)hipEventDestroy(s->ev_ph[j]); s->ev_ph[j] = nullptr; }
                s->ev_ph[i] = nullptr;
                return fail(SB_ENOMEM, "phase_timing: cannot create events");
            }
    s->phase_timing = on != 0;
    return SB_OK;
}

int32_t sb_debug_fail_launch(sb_session* s, int32_t n) {
    if (!s || n < 0) return fail(SB_EINVAL, "debug_fail_launch: bad argument");
    s->fail_countdown = n;
    return SB_OK;
}

int32_t sb_open_rows(const sb_session* s) { return s ? s->n_slots : SB_EINVAL; }

int32_t sb_get_stats(const sb_session* s, sb_stats* out) {
    if (!s || !out) return fail(SB_EINVAL, "get_stats: NULL argument");
    *out = s->st;
    return SB_OK;
}

int32_t sb_committed_len(const sb_session* s) { return s ? s->c : SB_EINVAL; }

int32_t sb_debug_enable(sb_session* s, int32_t on) {
    if (!s) return fail(SB_EINVAL, "debug_enable: session is NULL");
    s->debug = on != 0;
    return SB_OK;
}

int32_t sb_debug_logits(sb_session* s, int32_t layer, int32_t row, float* out, int32_t cap) {
    if (!s || !out) return fail(SB_EINVAL, "debug_logits: NULL argument");
    const sb_config& c = s->m->cfg;
    if (!s->debug) return fail(SB_ESTATE, "debug_logits: debug is off");
    if (cap < c.vocab) return fail(SB_EINVAL, "debug_logits: cap < vocab");
    const float* src;
    if (layer == 0) {
        if (row < 0 || row >= SB_MAX_W) return fail(SB_EINVAL, "debug_logits: row out of range");
        src = wsp<float>(s, s->L.logits_final) + (size_t)row * c.vocab;
    } else {
        if (layer < 1 || layer > c.n_exit_heads) return fail(SB_EINVAL, "debug_logits: layer out of range");
        src = wsp<float>(s, s->L.logits_exit) + (size_t)(layer - 1) * c.vocab;
    }
    HIP_TRY(sync_all(s));
    HIP_TRY(hipMemcpy(out, src, (size_t)c.vocab * 4, hipMemcpyDeviceToHost));
    return SB_OK;
}

int32_t sb_debug_hidden(sb_session* s, int32_t slot, float* out, int32_t cap) {
    if (!s || !out) return fail(SB_EINVAL, "debug_hidden: NULL argument");
    const sb_config& c = s->m->cfg;
    if (slot < 0 || slot >= SB_MAX_W || cap < c.d_model) return fail(SB_EINVAL, "debug_hidden: bad slot / cap");
    HIP_TRY(sync_all(s));
    HIP_TRY(hipMemcpy(out, wsp<float>(s, s->L.H) + (size_t)slot * c.d_model, (size_t)c.d_model * 4, hipMemcpyDeviceToHost));
    return SB_OK;
}

int32_t sb_debug_kv(sb_session* s, int32_t layer, int32_t pos, float* k_out, float* v_out, int32_t cap) {
    if (!s || !k_out || !v_out) return fail(SB_EINVAL, "debug_kv: NULL argument");
    const sb_config& c = s->m->cfg;
    const int w = c.n_kv_heads * c.head_dim;
    if (layer < 0 || layer >= c.n_layers || pos < 0 || pos >= c.max_seq || cap < w) return fail(SB_EINVAL, "debug_kv: out of range");
    HIP_TRY(sync_all(s));
    std::vector<int32_t> table(s->L.n_pages);
    HIP_TRY(hipMemcpy(table.data(), s->kv.table, table.size() * 4, hipMemcpyDeviceToHost));
    const size_t es = esize(c.kv_dtype);
    const int page = table[pos / SB_KV_BLOCK], t = pos % SB_KV_BLOCK;
    // one kv head's slab of a page: K [16 keys][head_dim]; V the same for an fp32 cache and
    // transposed, [head_dim][16 keys], for a bf16 cache
    std::vector<char> slab((size_t)SB_KV_BLOCK * c.head_dim * es);
    for (int which = 0; which < 2; ++which)
        for (int h = 0; h < c.n_kv_heads; ++h) {
            size_t off = (((size_t)(layer * 2 + which) * s->L.n_pages + page) * c.n_kv_heads + h) * SB_KV_BLOCK * c.head_dim;
            HIP_TRY(hipMemcpy(slab.data(), (const char*)s->kv.pool + off * es, slab.size(), hipMemcpyDeviceToHost));
            float* dst = (which == 0 ? k_out : v_out) + (size_t)h * c.head_dim;
            for (int i = 0; i < c.head_dim; ++i) {
                if (c.kv_dtype == SB_BF16) {
                    const size_t e = which == 0 ? (size_t)t * c.head_dim + i : (size_t)i * SB_KV_BLOCK + t;
                    uint32_t u = (uint32_t)((const uint16_t*)slab.data())[e] << 16;
                    memcpy(&dst[i], &u, 4);
                } else {
                    dst[i] = ((const float*)slab.data())[(size_t)t * c.head_dim + i];
                }
            }
        }
    return SB_OK;
}

}  // extern "C"
