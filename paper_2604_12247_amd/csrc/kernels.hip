// gfx950 kernels of the bounded self-speculative decode step: embedding, RMSNorm, operand split, the
// merge stage of a head evaluation, sampling-mode acceptance, bandwidth yardsticks.  The projections
// are in gemv.hip, attention in attention.hip, the prompt pass in prefill.hip.
//
// Every kernel here is written so that the value computed for one token row
// depends only on that row's inputs, its absolute position and the operand
// shapes -- never on how many other rows share the launch.  That is what makes a
// row verified in a pass of M rows bit-identical to the same row decoded alone,
// and hence speculative output identical to greedy decoding by the same library
// (the exactness property of Sec. 3.3).
#include "kernels.h"
#include "device_utils.h"

#include <math.h>
#include <mutex>

namespace sb {

// ---------------------------------------------------------------- embedding
// Row r of the hidden cache := embedding of token `tok` (+ what the first layer's projection
// needs: bf16 parts of gain * h and the row's sum of squares).  Executed by the first 256
// threads of a block, which all reach the barrier inside; the same code serves the embedding
// kernel and the head merge that embeds the token it has just drafted, so a row's values do
// not depend on which of the two wrote it.
template <typename WT>
__device__ __forceinline__ void embed_row(const WT* __restrict__ E, int vocab, int d, float* __restrict__ H, int tok, int r,
                                          EmbedNorm en, float* red /*[4] shared*/) {
    constexpr int VMAX = 4;  // 8-element groups a thread keeps in registers (covers d <= 8192)
    const int tid = threadIdx.x;
    const bool act = tid < 256;
    if (tok < 0 || tok >= vocab) tok = 0;  // never index outside the table
    const WT* e = E + (size_t)tok * d;
    const int ngrp = d >> 3;
    float ss = 0.f;
    if (act) {
        float v[VMAX][8], gn[VMAX][8];
#pragma unroll
        for (int j = 0; j < VMAX; ++j) {
            const int gi = tid + j * 256;
            if (gi < ngrp) {
                load8(e + gi * 8, v[j]);
                if (en.nx) load8(en.gain + gi * 8, gn[j]);
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) v[j][k] = 0.f;
            }
        }
#pragma unroll
        for (int j = 0; j < VMAX; ++j) {
            const int gi = tid + j * 256;
            if (gi < ngrp) {
#pragma unroll
                for (int k = 0; k < 8; ++k) {
                    H[(size_t)r * d + gi * 8 + k] = v[j][k];
                    ss += v[j][k] * v[j][k];
                    if (en.nx) split_store(en.nx, d, r, gi * 8 + k, v[j][k] * gn[j][k]);
                }
            }
        }
        for (int i = VMAX * 2048 + tid; i < d; i += 256) {  // d > 8192
            float x = ldf(e + i);
            H[(size_t)r * d + i] = x;
            ss += x * x;
            if (en.nx) split_store(en.nx, d, r, i, x * en.gain[i]);
        }
    }
    if (en.ssq_out) {  // the row's sum of squares, as a single partial
        ss = wave_sum(ss);
        if (act && (tid & 63) == 0) red[tid >> 6] = ss;
        __syncthreads();
        if (tid == 0) en.ssq_out[(size_t)r * en.ssq_ld] = ((red[0] + red[1]) + red[2]) + red[3];
    }
}

template <typename WT>
__global__ __launch_bounds__(256) void embed_kernel(const WT* __restrict__ E, int vocab, int d, float* __restrict__ H,
                                                    RowToks toks, const int32_t* __restrict__ slot_tok,
                                                    int32_t* clear_flag, EmbedNorm en) {
    __shared__ float red[4];
    int r = blockIdx.x, tid = threadIdx.x;
    int tok = toks.tok[r];
    if (tok < 0) tok = slot_tok[r];
    if (clear_flag && r == 0 && tid == 0) *clear_flag = 0;
    embed_row<WT>(E, vocab, d, H, tok, r, en, red);
}

hipError_t launch_embed(const void* E, int32_t w_dtype, int32_t vocab, int32_t d, float* H, int32_t M,
                        RowToks toks, const int32_t* slot_tok, int32_t* clear_flag, EmbedNorm en, hipStream_t st) {
    if (w_dtype == SB_BF16)
        embed_kernel<uint16_t><<<M, 256, 0, st>>>((const uint16_t*)E, vocab, d, H, toks, slot_tok, clear_flag, en);
    else
        embed_kernel<float><<<M, 256, 0, st>>>((const float*)E, vocab, d, H, toks, slot_tok, clear_flag, en);
    return hipGetLastError();
}

// ---------------------------------------------------------------- RMSNorm
// out = x / sqrt(mean(x^2) + eps) * gain, one block per row.
__global__ __launch_bounds__(256) void rmsnorm_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                      float* __restrict__ out, uint16_t* __restrict__ outs, int lds,
                                                      int d, float eps) {
    constexpr int VMAX = 8;  // float4 values a thread keeps in registers (covers d <= 8192)
    __shared__ float red[4];
    const int r = blockIdx.x, tid = threadIdx.x;
    const int nvec = d >> 2;
    const float4* xr = reinterpret_cast<const float4*>(x + (size_t)r * d);
    const float4* g4 = reinterpret_cast<const float4*>(gain);
    float4 v[VMAX], g[VMAX];
    // all loads are issued before the first use: one memory round trip, not d/256
#pragma unroll
    for (int j = 0; j < VMAX; ++j) {
        int idx = tid + j * 256;
        v[j] = idx < nvec ? xr[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
        g[j] = idx < nvec ? g4[idx] : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float ss = 0.f;
#pragma unroll
    for (int j = 0; j < VMAX; ++j) ss += (v[j].x * v[j].x + v[j].y * v[j].y) + (v[j].z * v[j].z + v[j].w * v[j].w);
    for (int idx = tid + VMAX * 256; idx < nvec; idx += 256) {
        float4 t = xr[idx];
        ss += (t.x * t.x + t.y * t.y) + (t.z * t.z + t.w * t.w);
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float tot = ((red[0] + red[1]) + red[2]) + red[3];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    auto emit = [&](int idx, float4 t, float4 gg) {
        float4 o = make_float4(t.x * inv * gg.x, t.y * inv * gg.y, t.z * inv * gg.z, t.w * inv * gg.w);
        if (out) reinterpret_cast<float4*>(out + (size_t)r * d)[idx] = o;
        if (outs) {
            uint16_t h0 = f2bf(o.x), h1 = f2bf(o.y), h2 = f2bf(o.z), h3 = f2bf(o.w);
            uint16_t l0 = f2bf(o.x - bf2f(h0)), l1 = f2bf(o.y - bf2f(h1)), l2 = f2bf(o.z - bf2f(h2)),
                     l3 = f2bf(o.w - bf2f(h3));
            uint2 hi = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
            uint2 lo = make_uint2((uint32_t)l0 | ((uint32_t)l1 << 16), (uint32_t)l2 | ((uint32_t)l3 << 16));
            *reinterpret_cast<uint2*>(outs + (size_t)r * lds + idx * 4) = hi;
            *reinterpret_cast<uint2*>(outs + (size_t)(8 + r) * lds + idx * 4) = lo;
        }
    };
#pragma unroll
    for (int j = 0; j < VMAX; ++j) {
        int idx = tid + j * 256;
        if (idx < nvec) emit(idx, v[j], g[j]);
    }
    for (int idx = tid + VMAX * 256; idx < nvec; idx += 256) emit(idx, xr[idx], g4[idx]);
}

hipError_t launch_rmsnorm(const float* x, const float* gain, float* out, uint16_t* out_split, int32_t ld_split,
                          int32_t M, int32_t d, float eps, hipStream_t st) {
    rmsnorm_kernel<<<M, 256, 0, st>>>(x, gain, out, out_split, ld_split, d, eps);
    return hipGetLastError();
}

__global__ void split_kernel(const float* __restrict__ x, uint16_t* __restrict__ xs, int K) {
    int m = blockIdx.y;
    int i = blockIdx.x * 256 + threadIdx.x;
    if (i < K) split_store(xs, K, m, i, x[(size_t)m * K + i]);
}
hipError_t launch_split(const float* x, uint16_t* xs, int32_t M, int32_t K, hipStream_t st) {
    split_kernel<<<dim3((K + 255) / 256, M), 256, 0, st>>>(x, xs, K);
    return hipGetLastError();
}

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) p[i] = v;
}
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t st) {
    if (n == 0) return hipSuccess;
    fill_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(p, n, v);
    return hipGetLastError();
}

// ---------------------------------------------------------------- bandwidth yardsticks
__global__ __launch_bounds__(256) void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    for (; i < n; i += stride) dst[i] = src[i];
}
hipError_t launch_copy(void* dst, const void* src, size_t nbytes, hipStream_t st) {
    size_t n = nbytes / 16;
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    copy_kernel<<<(unsigned)blocks, 256, 0, st>>>((uint4*)dst, (const uint4*)src, n);
    return hipGetLastError();
}
__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, size_t n, float* sink) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * 256;
    uint32_t acc = 0;
    for (; i + 3 * stride < n; i += 4 * stride) {
        uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n; i += stride) { uint4 a = src[i]; acc ^= a.x ^ a.y ^ a.z ^ a.w; }
    if (acc == 0x9e3779b9u) *sink = 1.0f;  // practically never: keeps the loads alive
}
hipError_t launch_read(const void* src, size_t nbytes, float* sink, hipStream_t st) {
    size_t n = nbytes / 16;
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 1023) / 1024;
    if (blocks > 256 * 16) blocks = 256 * 16;
    read_kernel<<<(unsigned)blocks, 256, 0, st>>>((const uint4*)src, n, sink);
    return hipGetLastError();
}

// ---------------------------------------------------------------- head reduction
// Second stage of a head evaluation: one block merges the per-block partials
// (max, arg max, sum of exp((z - max)/T)) of every row in a fixed order -- so the
// result does not depend on block scheduling -- and carries out the exit test
// (Eq. 2) or the acceptance rule.  Rows are merged side by side, 128 threads each (a
// row's order of additions does not depend on how many rows there are).  When a draft
// exits, the block also embeds the drafted token as the next row (the next draft step
// then starts at its first layer).  It is a kernel of its own: publishing the
// partials inside the projection kernel would need a device-wide fence per
// block, which on this chip writes back and invalidates a whole L2.
__device__ __forceinline__ void head_merge_body(const HeadArgs& h, const int M, const int nb) {
    __shared__ float r_max[SB_MAX_W][2], r_sum[SB_MAX_W][2];
    __shared__ int r_idx[SB_MAX_W][2];
    __shared__ int s_am[SB_MAX_W];
    __shared__ float s_cf[SB_MAX_W];
    __shared__ int s_embed_tok;
    __shared__ float e_red[4];
    const int tid = threadIdx.x, lane = tid & 63, m = tid >> 7, t = tid & 127, half = (tid >> 6) & 1;
    const float4* p = reinterpret_cast<const float4*>(h.partials) + (size_t)(h.row0 + (m < M ? m : 0)) * nb;
    float mx = -SB_INF;
    int idx = 0x7fffffff;
    if (m < M) {
        for (int b0 = t; b0 < nb; b0 += 512) {  // four independent loads per round
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = (b0 + 128 * u < nb) ? p[b0 + 128 * u] : make_float4(-SB_INF, __int_as_float(0x7fffffff), 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = __float_as_int(v[u].y);
                if (v[u].x > mx || (v[u].x == mx && i < idx)) { mx = v[u].x; idx = i; }
            }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ov = __shfl_xor(mx, o, 64);
            int oi = __shfl_xor(idx, o, 64);
            if (ov > mx || (ov == mx && oi < idx)) { mx = ov; idx = oi; }
        }
        if (lane == 0) { r_max[m][half] = mx; r_idx[m][half] = idx; }
    }
    __syncthreads();
    float gmax = 0.f;
    if (m < M) {
        gmax = r_max[m][0];
        int gi = r_idx[m][0];
        if (r_max[m][1] > gmax || (r_max[m][1] == gmax && r_idx[m][1] < gi)) { gmax = r_max[m][1]; gi = r_idx[m][1]; }
        if (t == 0) s_am[m] = gi == 0x7fffffff ? 0 : gi;
        float sum = 0.f;
        for (int b0 = t; b0 < nb; b0 += 512) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = (b0 + 128 * u < nb) ? p[b0 + 128 * u] : make_float4(-SB_INF, 0.f, 0.f, 0.f);
#pragma unroll
            for (int u = 0; u < 4; ++u) sum += v[u].z * expf((v[u].x - gmax) / h.T);
        }
        sum = wave_sum(sum);
        if (lane == 0) r_sum[m][half] = sum;
    }
    __syncthreads();
    if (tid < M) s_cf[tid] = 1.0f / (r_sum[tid][0] + r_sum[tid][1]);
    if (tid == 0) s_embed_tok = -1;
    __syncthreads();
    if (tid == 0) {
        for (int r = 0; r < M; ++r) {
            if (h.argmax_out) h.argmax_out[r] = s_am[r];
            if (h.conf_out) h.conf_out[r] = s_cf[r];
        }
        if (h.post == POST_EXIT) {
            // Early exit at the first layer whose confidence reaches the threshold
            // (Sec. 3.2), or exactly at the forced layer.
            DevRound* R = h.round;
            int s = h.slot;
            float cf = s_cf[0];
            int am = s_am[0];
            R->conf[s] = cf;
            R->head_argmax[s] = am;
            bool ex = h.forced_exit >= 0 ? (h.layer == h.forced_exit) : (cf >= h.threshold);
            R->exit_flag = ex ? 1 : 0;
            int tok = -1;
            if (ex) {
                tok = h.forced_draft >= 0 ? h.forced_draft : am;
                R->drafts[s] = tok;
                R->slot_tok[s + 1] = tok;
                R->exit_layer[s] = h.layer;
                if (h.embed_E) s_embed_tok = tok;
            }
            if (h.note) {   // the decision for the host, the sequence number last (system-scope release)
                h.note[1] = ex ? 1 : 0;
                h.note[2] = tok;
                h.note[3] = __float_as_int(cf);
                h.note[4] = am;
                __hip_atomic_store(&h.note[0], h.note_seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
            }
        } else if (h.post == POST_ACCEPT) {
            // Keep the longest prefix of drafts equal to the greedy tokens; the row
            // after it yields one more token: min(m + 1, M) >= 1 are emitted.
            DevRound* R = h.round;
            int mt = 0;
            for (int r = 0; r < M; ++r) { R->g[r] = s_am[r]; R->gconf[r] = s_cf[r]; }
            while (mt < h.n_drafts && mt < M && R->drafts[mt] == s_am[mt]) ++mt;
            R->n_matched = mt;
            R->n_emit = mt + 1 < M ? mt + 1 : M;
        }
    }
    if (h.post == POST_EXIT && h.embed_E) {   // (uniform for the block)
        __syncthreads();
        const int tok = s_embed_tok;
        if (tok >= 0) {   // the drafted token becomes the next row of the round
            if (h.embed_dtype == SB_BF16) embed_row<uint16_t>((const uint16_t*)h.embed_E, h.embed_vocab, h.embed_d, h.embed_H, tok, 0, h.embed_en, e_red);
            else embed_row<float>((const float*)h.embed_E, h.embed_vocab, h.embed_d, h.embed_H, tok, 0, h.embed_en, e_red);
        }
    }
}

__global__ __launch_bounds__(1024) void head_merge_kernel(HeadArgs h, int M, int nb) { head_merge_body(h, M, nb); }

// The merges of several sequences after one shared head sweep (batch > 1): block b is the
// single-sequence merge on sequence b's arguments.
__global__ __launch_bounds__(1024) void head_merge_batch_kernel(HeadMergeBatch hb, int nb) {
    const HeadArgs h = hb.h[blockIdx.x];
    head_merge_body(h, hb.M[blockIdx.x], nb);
}

hipError_t launch_head_merge(const HeadArgs& h, int32_t M, int32_t nb, hipStream_t st) {
    head_merge_kernel<<<1, 1024, 0, st>>>(h, M, nb);
    return hipGetLastError();
}

hipError_t launch_head_merge_batch(const HeadMergeBatch& hb, int32_t n, int32_t nb, hipStream_t st) {
    if (n < 1 || n > SB_MAX_W) return hipErrorInvalidValue;
    if (n == 1) return launch_head_merge(hb.h[0], hb.M[0], nb, st);
    head_merge_batch_kernel<<<n, 1024, 0, st>>>(hb, nb);
    return hipGetLastError();
}

// ---------------------------------------------------------------- sampling-mode acceptance
// Verification when the output is sampled (Sec. 4.3, "sampling strategies": temperature and
// top-p; the paper gives no rule, the one taken is that of speculative sampling for a draft
// proposed deterministically): with P the distribution the full model samples from after a row
// -- softmax(z / temp), cut to its nucleus of mass top_p and renormalised -- the row's draft x is
// accepted with probability P(x); at the first rejection the token is drawn from P without x;
// when every draft is accepted and one more row exists its token is drawn from P.  Each emitted
// token is then distributed exactly as the full model's own sample.  One block, rows in order;
// all sums are taken in a fixed order.  Works on unnormalised weights e_j = exp((z_j - max)/temp).
struct BlockRed {
    float* red;  // [16] shared
    __device__ __forceinline__ float sum(float v) {
        v = wave_sum(v);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        float t = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) t += red[w];
        return t;
    }
    __device__ __forceinline__ float max(float v) {
        v = wave_max(v);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
        __syncthreads();
        float t = red[0];
#pragma unroll
        for (int w = 1; w < 16; ++w) t = fmaxf(t, red[w]);
        return t;
    }
};

// A thread's share (tokens tid, tid + 1024, ... of the V in w) of the sum of the weights >= t, added to f
// in index order; sixteen loads are in flight at a time.
__device__ __forceinline__ float add_at_least(const float* w, int V, float t, float f) {
    int j = threadIdx.x;
    for (; j + 15 * 1024 < V; j += 16 * 1024) {
        float e[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) e[i] = w[j + 1024 * i];
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (e[i] >= t) f += e[i];
    }
    for (; j < V; j += 1024) { const float e = w[j]; if (e >= t) f += e; }
    return f;
}

// Thread tid owns the weights of tokens tid, tid + 1024, ...: the first 32 of them stay in registers
// through the passes of the nucleus search, the rest (vocabularies above 32768) in a.wts, where a
// thread re-reads only what it wrote itself.
__global__ __launch_bounds__(1024) void sample_accept_kernel(SampleArgs a) {
    constexpr int NR = 32, VR = NR * 1024;
    __shared__ float red[16];
    __shared__ float seg[1024];
    __shared__ float s_base;
    __shared__ int s_seg, s_tok;
    BlockRed br{red};
    const int tid = threadIdx.x, V = a.V;
    const int Vw = V > VR ? V - VR : 0;   // weights kept in a.wts
    DevRound* R = a.round;
    int m = 0;       // accepted drafts so far (uniform)
    int drawn = -1;  // row at which a token was drawn
    for (int row = 0; row < a.M; ++row) {
        const float* z = a.logits + (size_t)row * V;
        float* w = a.wts + (size_t)row * Vw;
        float mx = -SB_INF;
        for (int j = tid; j < V; j += 1024) mx = fmaxf(mx, z[j]);
        mx = br.max(mx);
        float sm = 0.f;
        float ev[NR];   // weight of token tid + 1024 i
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const int j = tid + 1024 * i;
            ev[i] = j < V ? expf((z[j] - mx) / a.temp) : 0.f;
            if (j < V) sm += ev[i];
        }
        for (int j = tid; j < Vw; j += 1024) { const float e = expf((z[VR + j] - mx) / a.temp); w[j] = e; sm += e; }
        const float S = br.sum(sm);
        auto mass_at_least = [&](float t) {   // sum of the weights >= t, in a fixed order
            float f = 0.f;
#pragma unroll
            for (int i = 0; i < NR; ++i)
                if (tid + 1024 * i < V && ev[i] >= t) f += ev[i];
            if (Vw > 0) f = add_at_least(w, Vw, t, f);
            return br.sum(f);
        };
        // nucleus: the largest weight value `cut` such that the weights >= cut hold a share top_p
        // of S (so equal weights at its edge stay together); found by bisection on the bit
        // pattern of a positive float, which is monotone in its value
        float cut = 0.f, keep = S;
        if (a.top_p < 1.0f) {
            const float need = a.top_p * S;
            uint32_t lo = 0u, hi = __float_as_uint(1.0f) + 1u;  // the largest weight is exp(0) = 1
            while (hi - lo > 1u) {
                const uint32_t mid = lo + (hi - lo) / 2u;
                if (mass_at_least(__uint_as_float(mid)) >= need) lo = mid; else hi = mid;
            }
            cut = __uint_as_float(lo);
            keep = mass_at_least(cut);
        }
        const bool has_draft = row < a.n_drafts;
        const int x = has_draft ? R->drafts[row] : -1;
        float ex = 0.f;
        if (x >= 0 && x < V) {
            ex = expf((z[x] - mx) / a.temp);
            if (ex < cut) ex = 0.f;
        }
        if (tid == 0) R->gconf[row] = ex / keep;   // P(x): the row's acceptance probability
        if (has_draft && a.ua[row] * keep < ex) {  // accepted
            if (tid == 0) R->g[row] = x;
            ++m;
            continue;
        }
        // draw from P without x: inverse CDF over the tokens in index order
        const float total = keep - ex, target = a.ur[row] * total;
        const int per = (V + 1023) / 1024, j0 = tid * per, j1 = (j0 + per < V) ? j0 + per : V;
        float ssum = 0.f;
        int last_mass = -1;
        for (int j = j0; j < j1; ++j) {
            const float e = expf((z[j] - mx) / a.temp);
            if (e >= cut && j != x) { ssum += e; last_mass = j; }
        }
        seg[tid] = ssum;
        __syncthreads();
        if (tid == 0) {
            float c = 0.f;
            int chosen = -1;
            for (int t = 0; t < 1024; ++t) {
                if (c + seg[t] > target) { chosen = t; break; }
                c += seg[t];
            }
            s_seg = chosen;
            s_base = c;
            s_tok = -1;
        }
        __syncthreads();
        const int chosen = s_seg;
        if (chosen >= 0) {
            if (tid == chosen) {
                float c = s_base;
                int tok = last_mass;
                for (int j = j0; j < j1; ++j) {
                    const float e = expf((z[j] - mx) / a.temp);
                    if (e >= cut && j != x) {
                        c += e;
                        if (c > target) { tok = j; break; }
                    }
                }
                s_tok = tok;
            }
            __syncthreads();
        } else {  // rounding at the upper end: the last token that has mass
            int lm = last_mass;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) { int v = __shfl_xor(lm, o, 64); lm = v > lm ? v : lm; }
            const float best = br.max((float)lm);   // token ids are exact in a float up to 2^24
            if (tid == 0) s_tok = (int)best;
            __syncthreads();
        }
        if (tid == 0) R->g[row] = s_tok;
        drawn = row;
        break;
    }
    if (tid == 0) {
        for (int row = (drawn >= 0 ? drawn : a.M - 1) + 1; row < a.M; ++row) { R->g[row] = -1; R->gconf[row] = 0.f; }
        R->n_matched = m;
        R->n_emit = m + 1 < a.M ? m + 1 : a.M;
    }
}

hipError_t launch_sample_accept(const SampleArgs& a, hipStream_t st) {
    if (!a.logits || !a.round || a.V < 1 || a.V > (1 << 24) || a.M < 1 || a.M > SB_MAX_W || !(a.temp > 0.f) || !(a.top_p > 0.f))
        return hipErrorInvalidValue;
    if (a.V > 32 * 1024 && !a.wts) return hipErrorInvalidValue;
    sample_accept_kernel<<<1, 1024, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace sb
