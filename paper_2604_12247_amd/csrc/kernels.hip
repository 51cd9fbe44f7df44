// gfx950 kernels of the bounded self-speculative decode step.
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

__global__ __launch_bounds__(1024) void sample_accept_kernel(SampleArgs a) {
    __shared__ float red[16];
    __shared__ float seg[1024];
    __shared__ float s_base;
    __shared__ int s_seg, s_tok;
    BlockRed br{red};
    const int tid = threadIdx.x, V = a.V;
    DevRound* R = a.round;
    int m = 0;       // accepted drafts so far (uniform)
    int drawn = -1;  // row at which a token was drawn
    for (int row = 0; row < a.M; ++row) {
        const float* z = a.logits + (size_t)row * V;
        float mx = -SB_INF;
        for (int j = tid; j < V; j += 1024) mx = fmaxf(mx, z[j]);
        mx = br.max(mx);
        float sm = 0.f;
        for (int j = tid; j < V; j += 1024) sm += expf((z[j] - mx) / a.temp);
        const float S = br.sum(sm);
        // nucleus: the largest weight value `cut` such that the weights >= cut hold a share top_p
        // of S (so equal weights at its edge stay together); found by bisection on the bit
        // pattern of a positive float, which is monotone in its value
        float cut = 0.f, keep = S;
        if (a.top_p < 1.0f) {
            const float need = a.top_p * S;
            uint32_t lo = 0u, hi = __float_as_uint(1.0f) + 1u;  // the largest weight is exp(0) = 1
            while (hi - lo > 1u) {
                const uint32_t mid = lo + (hi - lo) / 2u;
                const float t = __uint_as_float(mid);
                float f = 0.f;
                for (int j = tid; j < V; j += 1024) {
                    const float e = expf((z[j] - mx) / a.temp);
                    if (e >= t) f += e;
                }
                f = br.sum(f);
                if (f >= need) lo = mid; else hi = mid;
            }
            cut = __uint_as_float(lo);
            float f = 0.f;
            for (int j = tid; j < V; j += 1024) {
                const float e = expf((z[j] - mx) / a.temp);
                if (e >= cut) f += e;
            }
            keep = br.sum(f);
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
    sample_accept_kernel<<<1, 1024, 0, st>>>(a);
    return hipGetLastError();
}

// Partial (max, arg max, sum exp) of the block's logits zs[i][m], i < ROWS: thread (m, i) holds one
// logit, the ROWS lanes of a row are reduced with a fixed shuffle tree (ties: the lower index).
// Every thread of the block calls it (blocks have at least 8 * ROWS threads).
template <int ROWS>
__device__ __forceinline__ void head_partial(const HeadArgs& h, float (*zs)[SB_MAX_W], uint32_t rows, int n0, int N, int nb) {
    static_assert(ROWS == 16 || ROWS == 32, "a row's lanes lie in one wave");
    const int tid = threadIdx.x;
    if (tid >= SB_MAX_W * ROWS) return;   // (whole waves: 8 * ROWS is a multiple of 64)
    const int m = tid / ROWS, i = tid % ROWS, n = n0 + i;
    const bool live = n < N;
    const float z = live ? zs[i][m] : -SB_INF;
    const bool row_on = (rows >> m) & 1u;
    if (h.logits && live && row_on) h.logits[(size_t)m * N + n] = z;
    float mx = z;
    int idx = live ? n : 0x7fffffff;
#pragma unroll
    for (int o = ROWS / 2; o > 0; o >>= 1) {
        const float ov = __shfl_xor(mx, o, 64);
        const int oi = __shfl_xor(idx, o, 64);
        if (ov > mx || (ov == mx && oi < idx)) { mx = ov; idx = oi; }
    }
    float sum = live ? expf((z - mx) / h.T) : 0.f;
#pragma unroll
    for (int o = ROWS / 2; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
    if (i == 0 && row_on) {
        float* p = h.partials + ((size_t)m * nb + blockIdx.x) * 4;
        p[0] = mx;
        p[1] = __int_as_float(idx);
        p[2] = sum;
    }
}

// ---------------------------------------------------------------- GEMV, vector ALU
// y[m][n] = sum_k W[n][k] x[m][k] for M rows sharing one sweep over W.  One wave
// owns 4 weight rows; lanes stride the K dimension in 16-byte pieces (128-bit
// loads), partial sums are combined with a fixed shuffle tree.  x is staged in
// LDS in chunks.  The order in which a row's products are added is a function of
// K alone.

template <typename WT, int M, int EPI>
__global__ __launch_bounds__(256) void gemv_valu_kernel(GemvArgs a) {
    constexpr int R = 4;
    constexpr int KC = (M <= 4) ? 2048 : 1024;
    constexpr int OUT_PER_BLOCK = (EPI == EPI_SWIGLU) ? 8 : 16;
    __shared__ __attribute__((aligned(16))) float xs[M][KC];
    __shared__ float zs[16][SB_MAX_W];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const WT* __restrict__ W = reinterpret_cast<const WT*>(a.W);
    const int N = a.N, K = a.K;
    const int n0 = blockIdx.x * OUT_PER_BLOCK;
    const int total_rows = (EPI == EPI_SWIGLU) ? 2 * N : N;

    int outn[R];
    const WT* wrow[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        int n, row;
        if (EPI == EPI_SWIGLU) {
            n = n0 + wave * 2 + (r & 1);
            row = (r < 2) ? n : N + n;
        } else {
            n = n0 + wave * 4 + r;
            row = n;
        }
        outn[r] = n;
        if (row > total_rows - 1) row = total_rows - 1;  // loads stay inside W; the result is dropped
        wrow[r] = W + (size_t)row * K;
    }

    float acc[R][M];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < M; ++m) acc[r][m] = 0.f;

    for (int k0 = 0; k0 < K; k0 += KC) {
        const int kc = (K - k0 < KC) ? (K - k0) : KC;
        __syncthreads();
        for (int i = tid * 4; i < M * KC; i += 1024) {
            int m = i / KC, kk = i - m * KC;
            if (kk < kc)
                *reinterpret_cast<float4*>(&xs[m][kk]) =
                    *reinterpret_cast<const float4*>(a.x + (size_t)m * K + k0 + kk);
        }
        __syncthreads();
#pragma unroll 2
        for (int kk = lane * 8; kk < kc; kk += 512) {
            float w[R][8];
#pragma unroll
            for (int r = 0; r < R; ++r) load8(wrow[r] + k0 + kk, w[r]);
#pragma unroll
            for (int m = 0; m < M; ++m) {
                float4 xa = *reinterpret_cast<const float4*>(&xs[m][kk]);
                float4 xb = *reinterpret_cast<const float4*>(&xs[m][kk + 4]);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float s = acc[r][m];
                    s = fmaf(w[r][0], xa.x, s); s = fmaf(w[r][1], xa.y, s);
                    s = fmaf(w[r][2], xa.z, s); s = fmaf(w[r][3], xa.w, s);
                    s = fmaf(w[r][4], xb.x, s); s = fmaf(w[r][5], xb.y, s);
                    s = fmaf(w[r][6], xb.z, s); s = fmaf(w[r][7], xb.w, s);
                    acc[r][m] = s;
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int m = 0; m < M; ++m) acc[r][m] = wave_sum(acc[r][m]);

    if (EPI == EPI_STORE || EPI == EPI_RESID) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int m = 0; m < M; ++m)
                if (lane == r * M + m && outn[r] < N) {
                    float* yp = a.y + (size_t)m * a.ldy + outn[r];
                    *yp = (EPI == EPI_RESID) ? (*yp + acc[r][m]) : acc[r][m];
                }
    } else if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int m = 0; m < M; ++m)
                if (lane == j * M + m && outn[j] < N)
                    a.y[(size_t)m * a.ldy + outn[j]] = silu_mul(acc[j][m], acc[2 + j][m]);
    } else {  // EPI_HEAD
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int m = 0; m < M; ++m)
                if (lane == r * M + m) zs[wave * 4 + r][m] = acc[r][m];
        __syncthreads();
        head_partial<16>(a.head, zs, (1u << M) - 1u, n0, N, gridDim.x);
    }
}

int head_blocks_valu(int32_t N) { return (N + 15) / 16; }

template <typename WT, int M>
static hipError_t launch_gemv_valu_m(const GemvArgs& a, hipStream_t st) {
    switch (a.epi) {
        case EPI_STORE: gemv_valu_kernel<WT, M, EPI_STORE><<<(a.N + 15) / 16, 256, 0, st>>>(a); break;
        case EPI_RESID: gemv_valu_kernel<WT, M, EPI_RESID><<<(a.N + 15) / 16, 256, 0, st>>>(a); break;
        case EPI_SWIGLU: gemv_valu_kernel<WT, M, EPI_SWIGLU><<<(a.N + 7) / 8, 256, 0, st>>>(a); break;
        case EPI_HEAD: {
            gemv_valu_kernel<WT, M, EPI_HEAD><<<(a.N + 15) / 16, 256, 0, st>>>(a);
            hipError_t e = hipGetLastError();
            return e != hipSuccess ? e : launch_head_merge(a.head, M, (a.N + 15) / 16, st);
        }
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
template <typename WT>
static hipError_t launch_gemv_valu_t(const GemvArgs& a, hipStream_t st) {
    switch (a.M) {
        case 1: return launch_gemv_valu_m<WT, 1>(a, st);
        case 2: return launch_gemv_valu_m<WT, 2>(a, st);
        case 3: return launch_gemv_valu_m<WT, 3>(a, st);
        case 4: return launch_gemv_valu_m<WT, 4>(a, st);
        case 5: return launch_gemv_valu_m<WT, 5>(a, st);
        case 6: return launch_gemv_valu_m<WT, 6>(a, st);
        case 7: return launch_gemv_valu_m<WT, 7>(a, st);
        case 8: return launch_gemv_valu_m<WT, 8>(a, st);
        default: return hipErrorInvalidValue;
    }
}
hipError_t launch_gemv_valu(const GemvArgs& a, hipStream_t st) {
    if (a.K % 8 != 0 || a.N < 1) return hipErrorInvalidValue;
    return a.w_dtype == SB_BF16 ? launch_gemv_valu_t<uint16_t>(a, st) : launch_gemv_valu_t<float>(a, st);
}

// ---------------------------------------------------------------- GEMV, MFMA tiles
// bf16 weights only.  The M <= 8 activation rows are given as two bf16 parts each
// (x ~= hi + lo, 16 bits of mantissa), laid out as the 16 columns of one
// 16x16x32 MFMA B operand: columns 0-7 high parts, 8-15 low parts.  A 16-row
// tile of W is the A operand, read straight from HBM with 128-bit loads: the four
// lanes (i, q = 0..3) of row i read 64 contiguous bytes per instruction, 256 bytes
// per 128-wide k block.
// The four waves of a block take k blocks round-robin and are summed through LDS
// in wave order.  Products of bf16 values are exact in fp32, so the only rounding
// is fp32 accumulation.  Columns never mix, hence row results do not depend on M.
//
// PACKED: the weights were re-laid out once (repack_kernel) so that what a wave
// loads is contiguous: per 16-row tile and 128-wide k block one 4 KB unit, in it
// 1 KB per MFMA step holding lane l's 16 bytes at l * 16.  Every load instruction
// then reads 1 KB of consecutive memory (whole cache lines, so a streaming hint is
// safe) and a block walks one contiguous slab.  Same values in the same MFMA slots
// as the row-major path: results are bit-identical.
// Element offset of lane group lq's share of MFMA step u inside a 128-wide k block:
// one load instruction then covers 64 contiguous bytes of each of the 16 rows (the
// k order inside a block is free as long as A and B use the same one).
#define SB_KOFF(lq, u) ((u) * 32 + (lq) * 8)
// W [N][K] row-major -> packed tiles (N % 16 == 0, K % 128 == 0); one thread moves 16 bytes.
__global__ __launch_bounds__(256) void repack_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ P, int N,
                                                     int K) {
    const int KB = K >> 7;
    const size_t unit = (size_t)blockIdx.x * 256 + threadIdx.x;  // 16-byte unit of the packed array
    const size_t n_units = (size_t)N * K / 8;
    if (unit >= n_units) return;
    const int l = (int)(unit & 63), u = (int)((unit >> 6) & 3);
    const size_t blk = unit >> 8;  // (tile, k block)
    const int kb = (int)(blk % KB);
    const size_t tile = blk / KB;
    const int i = l & 15, q = l >> 4;
    const uint4 v = *reinterpret_cast<const uint4*>(W + (tile * 16 + i) * (size_t)K + (size_t)kb * 128 + SB_KOFF(q, u));
    *reinterpret_cast<uint4*>(P + unit * 8) = v;
}
hipError_t launch_repack(const void* W, void* P, int32_t N, int32_t K, hipStream_t st) {
    if (N % 16 || K % 128 || N < 16 || K < 128) return hipErrorInvalidValue;
    const size_t n_units = (size_t)N * K / 8;
    repack_kernel<<<(unsigned)((n_units + 255) / 256), 256, 0, st>>>((const uint16_t*)W, (uint16_t*)P, N, K);
    return hipGetLastError();
}

template <int RT, int EPI, int WPB, bool PACKED>
__global__ __launch_bounds__(64 * WPB) void gemv_mfma_kernel(GemvArgs a) {
    constexpr int NT = 64 * WPB;
    static_assert(NT >= RT * 128, "the tails take one element per thread");
    __shared__ __attribute__((aligned(16))) float red[WPB][RT][64][4];
    __shared__ float cs[RT][16][17];
    __shared__ float zs[16 * RT][SB_MAX_W];
    __shared__ float s_inv[SB_MAX_W];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const uint16_t* __restrict__ W = reinterpret_cast<const uint16_t*>(a.W);
    const int N = a.N, K = a.K, M = a.M;
    const int KB = K >> 7;  // k blocks of 128
    const int n0 = blockIdx.x * ((EPI == EPI_SWIGLU) ? 16 : 16 * RT);

    const uint16_t* wp[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        int row0 = (EPI == EPI_SWIGLU) ? (t == 0 ? n0 : N + n0) : (n0 + t * 16);  // first row of the tile
        int total = (EPI == EPI_SWIGLU) ? 2 * N : N;
        if (PACKED) {
            if (row0 > total - 16) row0 = total - 16;
            wp[t] = W + (size_t)(row0 >> 4) * KB * 2048 + lane * 8;
        } else {
            int row = row0 + li;
            if (row > total - 1) row = total - 1;
            wp[t] = W + (size_t)row * K;
        }
    }
    // Rows of this launch: the first M slots, or (passes that gather the rows of several
    // sequences) the slots of a bit mask.  Lanes whose column is a row that is not there load nothing.
    const uint32_t rows = a.row_mask ? a.row_mask : ((1u << M) - 1u);
    const bool bact = (rows >> (li & 7)) & 1u;
    const uint16_t* bp = a.xs + (size_t)li * K;

    f32x4 acc[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};

    // Ring of DEPTH register buffers, DEPTH - 1 k blocks in flight per wave.  The
    // stage loop is fully unrolled, so every buffer index is a compile-time constant.
    // chosen by measurement: three buffers, but two for the eight-wave blocks of the
    // narrow projections (a deeper ring there only costs occupancy)
    constexpr int DEPTH = (RT == 1 && WPB == 8) ? 2 : 3;
    uint4 wbuf[DEPTH][RT][4], bbuf[DEPTH][4];
    // k block index is clamped instead of tested: loads past the end re-read the last
    // block (unused), which keeps the steady-state loop free of bounds tests.
    auto load_block = [&](uint4 (&wr)[RT][4], uint4 (&br)[4], int kb) {
        const int kc = kb < KB ? kb : KB - 1;
        const size_t off = (size_t)kc * 128;
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                wr[t][u] = PACKED ? ld_weights_packed(wp[t] + (size_t)kc * 2048 + u * 512)
                                  : *reinterpret_cast<const uint4*>(wp[t] + off + SB_KOFF(lq, u));
#pragma unroll
        for (int u = 0; u < 4; ++u)
            br[u] = bact ? *reinterpret_cast<const uint4*>(bp + off + SB_KOFF(lq, u)) : make_uint4(0, 0, 0, 0);
    };
    auto mma_block = [&](const uint4 (&wr)[RT][4], const uint4 (&br)[4]) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            bf16x8 bv = __builtin_bit_cast(bf16x8, br[u]);
#pragma unroll
            for (int t = 0; t < RT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wr[t][u]), bv, acc[t],
                                                                 0, 0, 0);
        }
    };
    const int kb0 = wave;
    const int nkb = KB > wave ? (KB - wave + WPB - 1) / WPB : 0;  // k blocks of this wave
#pragma unroll
    for (int s = 0; s < DEPTH - 1; ++s) load_block(wbuf[s], bbuf[s], kb0 + s * WPB);
    // What the residual tail needs from memory (the element this thread finishes, its norm gains)
    // is requested now, behind the first weight loads, instead of at the end of the k loop.
    float pre_y = 0.f, pre_gA = 0.f, pre_gB = 0.f;
    if (EPI == EPI_RESID && tid < RT * 16 * 8) {
        const int t = tid >> 7, m = (tid >> 4) & 7, i = tid & 15, n = n0 + t * 16 + i;
        if (((rows >> m) & 1u) && n < N) {
            pre_y = a.y[(size_t)m * a.ldy + n];
            if (a.nxA) pre_gA = a.gainA[n];
            if (a.nxB) pre_gB = a.gainB[n];
        }
    }
    // RMSNorm scale of each row from the partial sums of squares its producer left
    // (added in index order; the first weight loads are already in flight)
    if (a.ssq_in) {
        for (int m = wave; m < SB_MAX_W; m += WPB) {
            if (!((rows >> m) & 1u)) continue;   // (wave-uniform)
            float t = 0.f;
            for (int b = lane; b < a.ssq_nb; b += 64) t += a.ssq_in[(size_t)m * a.ssq_ld + b];
            t = wave_sum(t);
            if (lane == 0) s_inv[m] = 1.0f / sqrtf(t / (float)K + a.eps);
        }
    } else if (tid < SB_MAX_W) {
        s_inv[tid] = 1.0f;
    }
    int it = 0;
    for (; it + DEPTH <= nkb; it += DEPTH) {  // steady state: before it, buf[s] holds block it + s (s < DEPTH-1)
#pragma unroll
        for (int s = 0; s < DEPTH; ++s) {
            load_block(wbuf[(s + DEPTH - 1) % DEPTH], bbuf[(s + DEPTH - 1) % DEPTH], kb0 + (it + s + DEPTH - 1) * WPB);
            mma_block(wbuf[s], bbuf[s]);
        }
    }
#pragma unroll
    for (int s = 0; s < DEPTH - 1; ++s)  // the last nkb - it < DEPTH blocks are already in the ring
        if (it + s < nkb) mma_block(wbuf[s], bbuf[s]);
#pragma unroll
    for (int t = 0; t < RT; ++t) *reinterpret_cast<f32x4*>(&red[wave][t][lane][0]) = acc[t];
    __syncthreads();
    // C layout of the 16x16 tile: lane (j = l%16, g = l/16), register r -> row 4g + r, column j.
    for (int e = tid; e < RT * 256; e += NT) {
        int t = e >> 8, l = (e >> 2) & 63, r = e & 3;
        float v = red[0][t][l][r];
#pragma unroll
        for (int w = 1; w < WPB; ++w) v += red[w][t][l][r];
        cs[t][4 * (l >> 4) + r][l & 15] = v;
    }
    __syncthreads();

    if (EPI == EPI_STORE || EPI == EPI_RESID) {
        for (int e = tid; e < RT * 16 * 8; e += NT) {
            int t = e >> 7, m = (e >> 4) & 7, i = e & 15;
            int n = n0 + t * 16 + i;
            float sq = 0.f;
            if (((rows >> m) & 1u) && n < N) {
                float v = (cs[t][i][m] + cs[t][i][m + 8]) * s_inv[m];
                float* yp = a.y + (size_t)m * a.ldy + n;
                if (EPI == EPI_RESID) v += pre_y;   // (e == tid: a block has at least RT * 128 threads)
                *yp = v;
                if (EPI == EPI_RESID) {
                    if (a.nxA) split_store(a.nxA, a.ldy, m, n, v * pre_gA);
                    if (a.nxB) split_store(a.nxB, a.ldy, m, n, v * pre_gB);
                    sq = v * v;
                }
            }
            if (EPI == EPI_RESID) zs[t * 16 + i][m] = sq;
        }
        if (EPI == EPI_RESID && a.ssq_out) {  // sum of squares of each 16-row tile, rows in index order
            __syncthreads();
            if (tid < RT * 8) {
                int t = tid >> 3, m = tid & 7;
                if (((rows >> m) & 1u) && n0 + t * 16 < N) {
                    float sum = 0.f;
                    for (int i = 0; i < 16; ++i) sum += zs[t * 16 + i][m];
                    a.ssq_out[(size_t)m * a.ssq_ld + blockIdx.x * RT + t] = sum;
                }
            }
        }
    } else if (EPI == EPI_SWIGLU) {
        if (tid < 128) {
            int m = tid >> 4, i = tid & 15;
            int n = n0 + i;
            if (((rows >> m) & 1u) && n < N) {
                float g = (cs[0][i][m] + cs[0][i][m + 8]) * s_inv[m];
                float u = (cs[1][i][m] + cs[1][i][m + 8]) * s_inv[m];
                float v = silu_mul(g, u);
                if (a.y) a.y[(size_t)m * a.ldy + n] = v;
                if (a.ys) split_store(a.ys, a.ldy, m, n, v);
            }
        }
    } else {  // EPI_HEAD
        for (int e = tid; e < RT * 16 * 8; e += NT) {
            int t = e >> 7, m = (e >> 4) & 7, i = e & 15;
            zs[t * 16 + i][m] = (cs[t][i][m] + cs[t][i][m + 8]) * (((rows >> m) & 1u) ? s_inv[m] : 0.f);
        }
        __syncthreads();
        head_partial<16 * RT>(a.head, zs, rows, n0, N, gridDim.x);
    }
}

// Row tiles and waves per block: fixed by the operand shape alone (never by M).
// Few output rows -> one tile per block and eight waves splitting K, so that
// enough loads are in flight; many rows -> two tiles sharing one B operand.
static int mfma_row_tiles(int32_t N) { return N >= 15000 ? 2 : 1; }  // (measured: [15360 x 5120] gains 13 % at six rows with two, [12288 x 4096] loses 5 %)
static int mfma_waves(int32_t N) { return N <= 8192 ? 8 : 4; }
int head_blocks_mfma(int32_t N) { return (N + 16 * mfma_row_tiles(N) - 1) / (16 * mfma_row_tiles(N)); }

template <int EPI, bool PACKED>
static void launch_gemv_mfma_e(const GemvArgs& a, hipStream_t st) {
    if constexpr (EPI == EPI_SWIGLU) {
        gemv_mfma_kernel<2, EPI, 4, PACKED><<<a.N / 16, 256, 0, st>>>(a);
    } else {
        const int rt = mfma_row_tiles(a.N), wpb = mfma_waves(a.N);
        if (rt == 2) gemv_mfma_kernel<2, EPI, 4, PACKED><<<(a.N + 31) / 32, 256, 0, st>>>(a);
        else if (wpb == 8) gemv_mfma_kernel<1, EPI, 8, PACKED><<<a.N / 16, 512, 0, st>>>(a);
        else gemv_mfma_kernel<1, EPI, 4, PACKED><<<a.N / 16, 256, 0, st>>>(a);
    }
}

hipError_t launch_gemv_mfma(const GemvArgs& a, hipStream_t st) {
    if (a.w_dtype != SB_BF16 || a.K % 128 != 0 || a.N % 16 != 0 || a.M < 1 || a.M > 8 || !a.xs)
        return hipErrorInvalidValue;
    switch (a.epi) {
        case EPI_STORE: a.packed ? launch_gemv_mfma_e<EPI_STORE, true>(a, st) : launch_gemv_mfma_e<EPI_STORE, false>(a, st); break;
        case EPI_RESID: a.packed ? launch_gemv_mfma_e<EPI_RESID, true>(a, st) : launch_gemv_mfma_e<EPI_RESID, false>(a, st); break;
        case EPI_SWIGLU: a.packed ? launch_gemv_mfma_e<EPI_SWIGLU, true>(a, st) : launch_gemv_mfma_e<EPI_SWIGLU, false>(a, st); break;
        case EPI_HEAD: {
            a.packed ? launch_gemv_mfma_e<EPI_HEAD, true>(a, st) : launch_gemv_mfma_e<EPI_HEAD, false>(a, st);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess || a.head.skip_merge) return e;
            return launch_head_merge(a.head, a.M, head_blocks_mfma(a.N), st);
        }
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- head evaluation without a workspace
// For callers that cannot allocate device memory (code under graph capture, tight serving
// loops): the head partials and the split-bf16 operand of a single head evaluation live in a
// file-scope device array instead of a caller's scratch buffer.  Each GPU holds its own copy
// of the array at its own address, looked up once per device; every call on a GPU shares it,
// so calls that overlap on one GPU race.  Nothing in it has to start at zero: every element a
// launch reads was written by that launch sequence (partials of all blocks of rows < M, the
// operand rows of rows < M).
static __device__ __align__(256) unsigned char scratch[SB_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, once looked up
std::mutex g_scratch_mu;
}  // namespace

hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));   // the array's address on the current device
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

// ---------------------------------------------------------------- RoPE + KV append + attention
// M causal query rows at positions pos0..pos0+M-1 against keys 0..pos of the
// paged cache.  qkv holds the rows' raw projections (q heads, k heads, v heads).
// The key range is cut into fixed chunks of absolute positions; one block handles
// one (kv head, chunk, group of <= 16 queries) and writes a partial (max, sum,
// weighted V) per query; a second kernel merges the chunks in ascending order.
//
// The work inside a block is latency, not bandwidth, so everything is laid out for
// few dependent steps: K and V go from the cache straight into registers (no LDS
// tile), each in the mapping its consumer needs, all loads issued up front.
//   scores   thread = (key, slice of head_dim): partial dot products, slices added in order
//   softmax  wave per query over the chunk's keys
//   values   thread = (16-byte group of dims, key slot): a few keys each, then a fixed
//            shuffle tree over the key slots of a wave and the four waves in order
// Keys that belong to the new rows are not read from the cache: the block rotates
// (half-split pairing, table built on the host in double and held in float) and
// rounds them from qkv exactly as they are stored, and the block of query group 0
// also writes them into the cache (KV append).  A row's result depends on its own
// position and keys only.
template <typename KVT> struct KvVec;
template <> struct KvVec<uint16_t> {
    static constexpr int EPV = 8;
    static __device__ __forceinline__ void unpack(uint4 v, float* f) {
        f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
        f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
        f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
        f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4((uint32_t)f2bf(f[0]) | ((uint32_t)f2bf(f[1]) << 16), (uint32_t)f2bf(f[2]) | ((uint32_t)f2bf(f[3]) << 16),
                          (uint32_t)f2bf(f[4]) | ((uint32_t)f2bf(f[5]) << 16), (uint32_t)f2bf(f[6]) | ((uint32_t)f2bf(f[7]) << 16));
    }
};
template <> struct KvVec<float> {
    static constexpr int EPV = 4;
    static __device__ __forceinline__ void unpack(uint4 v, float* f) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y); f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};

template <typename KVT, int HD>
__global__ __launch_bounds__(256) void attn_kernel(AttnArgs a) {
    constexpr int CH = (HD * sizeof(KVT) <= 256) ? 128 : 64;  // keys per chunk
    constexpr int EPV = KvVec<KVT>::EPV;                      // elements per 16 bytes
    constexpr int QG = 16;                                    // queries per block
    constexpr int HALF = HD / 2;
    constexpr int DSPLIT = 256 / CH;                          // score threads per key
    constexpr int DPT = HD / DSPLIT;                          // dims per score thread
    constexpr int NKV = DPT / EPV;                            // 16-byte loads per score thread
    // values mapping: each wave owns HD/4 dims and sees every key of the chunk, so the
    // sum over keys ends inside the wave (no cross-wave stage, no LDS buffer for it)
    constexpr int DGW = HD / 4 / EPV;                         // 16-byte dim groups per wave
    constexpr int KS = 64 / DGW;                              // key slots (lanes per dim group)
    constexpr int KPT = CH / KS;                              // keys per value thread
    static_assert(DPT <= HALF && HALF % DPT == 0, "a score thread's dims lie in one rotary half");
    static_assert(DGW >= 1 && KS * KPT == CH, "value mapping");
    __shared__ __attribute__((aligned(16))) float qs[QG * HD];
    __shared__ __attribute__((aligned(16))) float sp[DSPLIT * QG * CH];  // partial scores, then probabilities
    __shared__ float s_m[QG], s_l[QG];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.x, chunk = blockIdx.y, qg = blockIdx.z;
    const int Hq = a.n_heads, Hkv = a.kv.n_kv_heads, G = Hq / Hkv;
    const int nq_total = a.M * G, q0 = qg * QG;
    const int nq = (nq_total - q0 < QG) ? (nq_total - q0) : QG;
    const int key0 = chunk * CH, n_total = a.pos0 + a.M;
    const float scale = 1.0f / sqrtf((float)HD);
    const size_t page_elems = (size_t)Hkv * SB_KV_BLOCK * HD;
    KVT* const kbase = reinterpret_cast<KVT*>(a.kv.pool) + (size_t)(a.layer * 2 + 0) * a.kv.n_pages * page_elems;
    KVT* const vbase = reinterpret_cast<KVT*>(a.kv.pool) + (size_t)(a.layer * 2 + 1) * a.kv.n_pages * page_elems;

    // ---- issue every global load first: q (+ its rotary factors), K, V
    constexpr int QIT = QG * HALF / 256;
    float qx[QIT], qy[QIT], qc[QIT], qsn[QIT];
#pragma unroll
    for (int it = 0; it < QIT; ++it) {
        const int i = tid + it * 256;
        const int qi = i / HALF, j = i - qi * HALF;
        qx[it] = qy[it] = qsn[it] = 0.f;
        qc[it] = 1.f;
        if (qi < nq) {
            int qq = q0 + qi, r = qq / G, gi = qq - r * G;
            const float* qp = a.q + (size_t)r * a.qkv_rows + (size_t)(g * G + gi) * HD;
            qx[it] = qp[j];
            qy[it] = qp[j + HALF];
            qc[it] = a.rope_cos[(size_t)(a.pos0 + r) * HALF + j];
            qsn[it] = a.rope_sin[(size_t)(a.pos0 + r) * HALF + j];
        }
    }
    // scores mapping: key kt, dims [kd0, kd0 + DPT)
    const int kt = tid % CH, kd0 = (tid / CH) * DPT;
    const int kkey = key0 + kt;
    uint4 kreg[NKV];
    size_t kaddr = 0;  // element offset of this thread's K slice inside the K pool of the layer
    if (kkey < n_total) kaddr = (size_t)a.kv.table[kkey / SB_KV_BLOCK] * page_elems + ((size_t)g * SB_KV_BLOCK + (kkey % SB_KV_BLOCK)) * HD + kd0;
#pragma unroll
    for (int i = 0; i < NKV; ++i) {
        kreg[i] = make_uint4(0, 0, 0, 0);
        if (kkey < a.pos0) kreg[i] = *reinterpret_cast<const uint4*>(kbase + kaddr + i * EPV);
    }
    // values mapping: dims [vd0, vd0 + EPV), keys vks + KS * i
    const int vd0 = wave * (HD / 4) + (lane % DGW) * EPV, vks = lane / DGW;
    uint4 vreg[KPT];
    size_t vaddr[KPT];
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int key = key0 + vks + KS * i;
        vreg[i] = make_uint4(0, 0, 0, 0);
        vaddr[i] = 0;
        if (key < n_total) vaddr[i] = (size_t)a.kv.table[key / SB_KV_BLOCK] * page_elems + ((size_t)g * SB_KV_BLOCK + (key % SB_KV_BLOCK)) * HD + vd0;
        if (key < a.pos0) vreg[i] = *reinterpret_cast<const uint4*>(vbase + vaddr[i]);
    }

    // ---- rotated queries -> LDS
#pragma unroll
    for (int it = 0; it < QIT; ++it) {
        const int i = tid + it * 256;
        const int qi = i / HALF, j = i - qi * HALF;
        qs[qi * HD + j] = qx[it] * qc[it] - qy[it] * qsn[it];
        qs[qi * HD + j + HALF] = qy[it] * qc[it] + qx[it] * qsn[it];
    }
    // ---- keys and values of the new rows: built from qkv, appended by query group 0
    if (kkey >= a.pos0 && kkey < n_total) {
        const int r = kkey - a.pos0;
        const float* kp = a.q + (size_t)r * a.qkv_rows + (size_t)(Hq + g) * HD;
        const bool lo = kd0 < HALF;
        const int dj = lo ? kd0 : kd0 - HALF;
#pragma unroll
        for (int i = 0; i < NKV; ++i) {
            float f[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) {
                const int j = dj + i * EPV + e;
                float c = a.rope_cos[(size_t)kkey * HALF + j], sn = a.rope_sin[(size_t)kkey * HALF + j];
                float x = kp[j], y = kp[j + HALF];
                f[e] = lo ? (x * c - y * sn) : (y * c + x * sn);
            }
            kreg[i] = KvVec<KVT>::pack(f);
            if (qg == 0) *reinterpret_cast<uint4*>(kbase + kaddr + i * EPV) = kreg[i];
        }
    }
#pragma unroll
    for (int i = 0; i < KPT; ++i) {
        const int key = key0 + vks + KS * i;
        if (key >= a.pos0 && key < n_total) {
            const float* vp = a.q + (size_t)(key - a.pos0) * a.qkv_rows + (size_t)(Hq + Hkv + g) * HD + vd0;
            float f[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) f[e] = vp[e];
            vreg[i] = KvVec<KVT>::pack(f);
            if (qg == 0) *reinterpret_cast<uint4*>(vbase + vaddr[i]) = vreg[i];
        }
    }
    __syncthreads();

    // ---- partial scores: this thread's DPT dims of key kt against every live query
    {
        float kf[NKV][EPV];
#pragma unroll
        for (int i = 0; i < NKV; ++i) KvVec<KVT>::unpack(kreg[i], kf[i]);
        for (int qi = 0; qi < nq; ++qi) {
            const float* qp = &qs[qi * HD + kd0];
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < NKV; ++i)
#pragma unroll
                for (int e = 0; e < EPV; e += 4) {
                    float4 qv = *reinterpret_cast<const float4*>(qp + i * EPV + e);
                    s = fmaf(qv.x, kf[i][e], s); s = fmaf(qv.y, kf[i][e + 1], s);
                    s = fmaf(qv.z, kf[i][e + 2], s); s = fmaf(qv.w, kf[i][e + 3], s);
                }
            sp[((tid / CH) * QG + qi) * CH + kt] = s;
        }
    }
    __syncthreads();
    // ---- softmax partial of each live query over the chunk (one wave per query)
    for (int qi = wave; qi < nq; qi += 4) {
        const int r = (q0 + qi) / G;
        float sc[CH / 64];
        float mx = -SB_INF;
#pragma unroll
        for (int h = 0; h < CH / 64; ++h) {
            const int t = lane + 64 * h;
            float s = sp[qi * CH + t];
#pragma unroll
            for (int ds = 1; ds < DSPLIT; ++ds) s += sp[(ds * QG + qi) * CH + t];
            sc[h] = (key0 + t <= a.pos0 + r) ? s * scale : -SB_INF;
            mx = fmaxf(mx, sc[h]);
        }
        mx = wave_max(mx);
        float l = 0.f;
#pragma unroll
        for (int h = 0; h < CH / 64; ++h) {
            float p = (mx == -SB_INF) ? 0.f : expf(sc[h] - mx);
            sc[h] = p;
            l += p;
        }
        l = wave_sum(l);
#pragma unroll
        for (int h = 0; h < CH / 64; ++h) sp[qi * CH + lane + 64 * h] = sc[h];
        if (lane == 0) { s_m[qi] = mx; s_l[qi] = l; }
    }
    __syncthreads();
    // ---- weighted values
    {
        float vf[KPT][EPV];
#pragma unroll
        for (int i = 0; i < KPT; ++i) KvVec<KVT>::unpack(vreg[i], vf[i]);
        for (int qi = 0; qi < nq; ++qi) {
            float o[EPV];
#pragma unroll
            for (int e = 0; e < EPV; ++e) o[e] = 0.f;
#pragma unroll
            for (int i = 0; i < KPT; ++i) {
                const float p = sp[qi * CH + vks + KS * i];
#pragma unroll
                for (int e = 0; e < EPV; ++e) o[e] = fmaf(p, vf[i][e], o[e]);
            }
            // sum over the key slots: fixed shuffle tree inside the wave
#pragma unroll
            for (int off = DGW; off < 64; off <<= 1)
#pragma unroll
                for (int e = 0; e < EPV; ++e) o[e] += __shfl_xor(o[e], off, 64);
            const int qq = q0 + qi, r = qq / G, gi = qq - r * G;
            if (lane < DGW && key0 <= a.pos0 + r) {  // (a chunk with no visible key leaves no partial)
                float* p = a.partials + ((size_t)(r * Hq + g * G + gi) * a.max_chunks + chunk) * (HD + 2);
#pragma unroll
                for (int e = 0; e < EPV; ++e) p[2 + vd0 + e] = o[e];
                if (tid == 0) { p[0] = s_m[qi]; p[1] = s_l[qi]; }
            }
        }
    }
}

// The same step for a bf16 cache, with both contractions on the matrix cores.
//   scores   S = Q K^T: A operand = rotated queries (16 rows; fp32 carried as a bf16
//            hi + lo pair, two MFMAs), B operand = keys straight from the cache (a lane's
//            8 consecutive dims of one key are one 16-byte load); a wave takes 32 keys
//   softmax  wave per query over the chunk's keys, probabilities left in LDS as hi + lo
//   values   O = P V: A operand = probabilities, B operand = values.  A lane needs 8
//            consecutive keys of one dim, so the V pages of a bf16 cache are stored
//            transposed, [kv head][dim][16 keys]: the operand is again one 16-byte load
//            and a wave's loads cover whole pages.  A wave owns HD/4 output dims.
// Every output row of an MFMA depends on its own operand row only, so a query's
// partial does not depend on which other queries share the block.
template <int HD>
__device__ __forceinline__ void attn_mfma_body(const AttnArgs& a, const int g, const int chunk, const int zb) {
    constexpr int CH = 128, QG = 16, HALF = HD / 2;
    constexpr int KSQ = HD / 32;      // k steps (of 32 dims) of the score product
    constexpr int KSV = CH / 32;      // k steps (of 32 keys) of the value product
    constexpr int DT = HD / 64;       // 16-dim output tiles per wave
    constexpr int QS = HD + 8;        // padded LDS row strides (bf16 elements / floats)
    constexpr int PS = CH + 8;
    constexpr int SS = CH + 4;
    __shared__ __attribute__((aligned(16))) uint16_t q_hi[QG * QS], q_lo[QG * QS];
    __shared__ __attribute__((aligned(16))) uint16_t p_hi[QG * PS], p_lo[QG * PS];
    __shared__ __attribute__((aligned(16))) float s_s[QG * SS];
    __shared__ float s_m[QG], s_l[QG];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int Hq = a.n_heads, Hkv = a.kv.n_kv_heads, G = Hq / Hkv;
    const int nq_total = a.M * G;
    // this block's query groups (16 queries each), handled one after the other with the
    // chunk's K and V held in registers
    const int n_qg = (nq_total + QG - 1) / QG;
    const int qg_first = zb * a.qg_per_block;
    const int qg_last = (qg_first + a.qg_per_block < n_qg) ? qg_first + a.qg_per_block : n_qg;
    const int key0 = chunk * CH, n_total = a.pos0 + a.M;
    const float scale = 1.0f / sqrtf((float)HD);
    const size_t page_elems = (size_t)Hkv * SB_KV_BLOCK * HD;
    uint16_t* const kbase = reinterpret_cast<uint16_t*>(a.kv.pool) + (size_t)(a.layer * 2 + 0) * a.kv.n_pages * page_elems;
    uint16_t* const vbase = reinterpret_cast<uint16_t*>(a.kv.pool) + (size_t)(a.layer * 2 + 1) * a.kv.n_pages * page_elems;
    const bool has_new = key0 + CH > a.pos0;  // the chunk holds keys of the new rows

    // ---- issue every global load first: q (+ its rotary factors) of the first group, K, V
    constexpr int QIT = QG * HALF / 256;
    float qx[QIT], qy[QIT], qc[QIT], qsn[QIT];
    auto load_q = [&](int qg) {
        const int q0 = qg * QG;
        const int nq = (nq_total - q0 < QG) ? (nq_total - q0) : QG;
#pragma unroll
        for (int it = 0; it < QIT; ++it) {
            const int i = tid + it * 256;
            const int qi = i / HALF, j = i - qi * HALF;
            qx[it] = qy[it] = qsn[it] = 0.f;
            qc[it] = 1.f;
            if (qi < nq) {
                int qq = q0 + qi, r = qq / G, gi = qq - r * G;
                const float* qp = a.q + (size_t)r * a.qkv_rows + (size_t)(g * G + gi) * HD;
                qx[it] = qp[j];
                qy[it] = qp[j + HALF];
                qc[it] = a.rope_cos[(size_t)(a.pos0 + r) * HALF + j];
                qsn[it] = a.rope_sin[(size_t)(a.pos0 + r) * HALF + j];
            }
        }
    };
    load_q(qg_first);
    // K operands: tile t of this wave = keys key0 + wave*32 + t*16 + li (one page), dims ks*32 + lq*8 ..
    uint4 kreg[2][KSQ];
    size_t kaddr[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int key = key0 + wave * 32 + t * 16 + li;
        // a tile is one page: its table entry is wave-uniform, read through the scalar cache
        const int kpage = __builtin_amdgcn_readfirstlane((key0 + wave * 32 + t * 16) / SB_KV_BLOCK);
        kaddr[t] = 0;
        if (kpage * SB_KV_BLOCK < n_total)
            kaddr[t] = (size_t)a.kv.table[kpage] * page_elems + ((size_t)g * SB_KV_BLOCK + li) * HD + lq * 8;
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            kreg[t][ks] = make_uint4(0, 0, 0, 0);
            if (key < a.pos0) kreg[t][ks] = *reinterpret_cast<const uint4*>(kbase + kaddr[t] + ks * 32);
        }
    }
    // V operands: dim (wave*DT + dt)*16 + li, keys key0 + ks*32 + lq*8 .. +8 (half a page row)
    uint4 vreg[DT][KSV];
    size_t vaddr[KSV];
#pragma unroll
    for (int ks = 0; ks < KSV; ++ks) {
        const int kf = key0 + ks * 32 + lq * 8;  // first key of this lane's 8
        // the 32 keys of a step lie in two pages (lq 0-1, lq 2-3): two wave-uniform table entries
        const int vpage = (key0 + ks * 32) / SB_KV_BLOCK;
        const int pg0 = vpage * SB_KV_BLOCK < n_total ? a.kv.table[vpage] : 0;
        const int pg1 = (vpage + 1) * SB_KV_BLOCK < n_total ? a.kv.table[vpage + 1] : 0;
        vaddr[ks] = 0;
        if (kf < n_total) vaddr[ks] = (size_t)(lq < 2 ? pg0 : pg1) * page_elems + ((size_t)g * HD + wave * DT * 16 + li) * SB_KV_BLOCK + (lq & 1) * 8;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            vreg[dt][ks] = make_uint4(0, 0, 0, 0);
            if (kf < a.pos0) vreg[dt][ks] = *reinterpret_cast<const uint4*>(vbase + vaddr[ks] + dt * 16 * SB_KV_BLOCK);
        }
    }

    // ---- keys and values of the new rows: built from qkv, appended by query group 0
    if (has_new) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int key = key0 + wave * 32 + t * 16 + li;
            if (key >= a.pos0 && key < n_total) {
                const float* kp = a.q + (size_t)(key - a.pos0) * a.qkv_rows + (size_t)(Hq + g) * HD;
#pragma unroll
                for (int ks = 0; ks < KSQ; ++ks) {
                    const int d0 = ks * 32 + lq * 8;
                    const bool lo = d0 < HALF;
                    const int dj = lo ? d0 : d0 - HALF;
                    float f[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int j = dj + e;
                        float c = a.rope_cos[(size_t)key * HALF + j], sn = a.rope_sin[(size_t)key * HALF + j];
                        float x = kp[j], y = kp[j + HALF];
                        f[e] = lo ? (x * c - y * sn) : (y * c + x * sn);
                    }
                    kreg[t][ks] = KvVec<uint16_t>::pack(f);
                    if (zb == 0) *reinterpret_cast<uint4*>(kbase + kaddr[t] + ks * 32) = kreg[t][ks];
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < KSV; ++ks) {
            const int kf = key0 + ks * 32 + lq * 8;
            if (kf + 8 > a.pos0 && kf < n_total) {  // some of the 8 keys are new
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const int d = (wave * DT + dt) * 16 + li;
                    uint32_t w[4] = {vreg[dt][ks].x, vreg[dt][ks].y, vreg[dt][ks].z, vreg[dt][ks].w};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int key = kf + e;
                        if (key >= a.pos0) {  // new row, or past the end: zero
                            uint32_t h = 0;
                            if (key < n_total) h = f2bf(a.q[(size_t)(key - a.pos0) * a.qkv_rows + (size_t)(Hq + Hkv + g) * HD + d]);
                            w[e >> 1] = (e & 1) ? ((w[e >> 1] & 0x0000ffffu) | (h << 16)) : ((w[e >> 1] & 0xffff0000u) | h);
                        }
                    }
                    vreg[dt][ks] = make_uint4(w[0], w[1], w[2], w[3]);
                    if (zb == 0) *reinterpret_cast<uint4*>(vbase + vaddr[ks] + dt * 16 * SB_KV_BLOCK) = vreg[dt][ks];
                }
            }
        }
    }
    for (int qg = qg_first; qg < qg_last; ++qg) {
    const int q0 = qg * QG;
    const int nq = (nq_total - q0 < QG) ? (nq_total - q0) : QG;
    // ---- rotated queries -> LDS as hi + lo
#pragma unroll
    for (int it = 0; it < QIT; ++it) {
        const int i = tid + it * 256;
        const int qi = i / HALF, j = i - qi * HALF;
        const float u = qx[it] * qc[it] - qy[it] * qsn[it], v = qy[it] * qc[it] + qx[it] * qsn[it];
        const uint16_t uh = f2bf(u), vh = f2bf(v);
        q_hi[qi * QS + j] = uh;
        q_lo[qi * QS + j] = f2bf(u - bf2f(uh));
        q_hi[qi * QS + j + HALF] = vh;
        q_lo[qi * QS + j + HALF] = f2bf(v - bf2f(vh));
    }
    if (qg + 1 < qg_last) load_q(qg + 1);  // (in flight during this group's products)
    __syncthreads();

    // ---- scores of this wave's 32 keys against the 16 query rows
    {
        f32x4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&q_hi[li * QS + ks * 32 + lq * 8]));
            const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&q_lo[li * QS + ks * 32 + lq * 8]));
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const bf16x8 kb = __builtin_bit_cast(bf16x8, kreg[t][ks]);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, kb, acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, kb, acc[t], 0, 0, 0);
            }
        }
        // result register r of lane (li, lq): query 4*lq + r, key li of the tile
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) s_s[(4 * lq + r) * SS + wave * 32 + t * 16 + li] = acc[t][r];
    }
    __syncthreads();
    // ---- softmax partial of each query over the chunk (one wave per query)
    for (int qi = wave; qi < QG; qi += 4) {
        if (qi >= nq) {  // unused operand rows: defined values
            p_hi[qi * PS + lane] = p_hi[qi * PS + lane + 64] = 0;
            p_lo[qi * PS + lane] = p_lo[qi * PS + lane + 64] = 0;
            continue;
        }
        const int r = (q0 + qi) / G;
        float sc[2];
        float mx = -SB_INF;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int t = lane + 64 * h;
            sc[h] = (key0 + t <= a.pos0 + r) ? s_s[qi * SS + t] * scale : -SB_INF;
            mx = fmaxf(mx, sc[h]);
        }
        mx = wave_max(mx);
        float l = 0.f;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float p = (mx == -SB_INF) ? 0.f : expf(sc[h] - mx);
            const uint16_t ph = f2bf(p);
            p_hi[qi * PS + lane + 64 * h] = ph;
            p_lo[qi * PS + lane + 64 * h] = f2bf(p - bf2f(ph));
            l += p;
        }
        l = wave_sum(l);
        if (lane == 0) { s_m[qi] = mx; s_l[qi] = l; }
    }
    __syncthreads();
    // ---- weighted values: this wave's DT tiles of 16 dims, all keys of the chunk
    {
        f32x4 o[DT];
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KSV; ++ks) {
            const bf16x8 ah = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&p_hi[li * PS + ks * 32 + lq * 8]));
            const bf16x8 al = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&p_lo[li * PS + ks * 32 + lq * 8]));
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) {
                const bf16x8 vb = __builtin_bit_cast(bf16x8, vreg[dt][ks]);
                o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, vb, o[dt], 0, 0, 0);
                o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, vb, o[dt], 0, 0, 0);
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int qi = 4 * lq + r;
            if (qi >= nq) continue;
            const int qq = q0 + qi, rr = qq / G, gi = qq - rr * G;
            if (key0 > a.pos0 + rr) continue;  // (a chunk with no visible key leaves no partial)
            float* p = a.partials + ((size_t)(rr * Hq + g * G + gi) * a.max_chunks + chunk) * (HD + 2);
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) p[2 + (wave * DT + dt) * 16 + li] = o[dt][r];
            if (wave == 0 && li == 0) { p[0] = s_m[qi]; p[1] = s_l[qi]; }
        }
    }
    __syncthreads();  // the next group overwrites the LDS arrays
    }
}

template <int HD>
__global__ __launch_bounds__(256, 3) void attn_mfma_kernel(AttnArgs a) {
    attn_mfma_body<HD>(a, blockIdx.x, blockIdx.y, blockIdx.z);
}

// Several sequences' passes in one launch (batch > 1): grid.z = sequence x query-group slice, grid.y
// = the longest sequence's chunks; a block outside its sequence's range leaves at once.  A block
// inside runs the code above on its sequence's arguments, so every value is the one the
// sequence's own launch computes.
template <int HD>
__global__ __launch_bounds__(256, 3) void attn_mfma_batch_kernel(AttnBatchArgs ab) {
    const int sq = blockIdx.z / ab.zdim, zb = blockIdx.z - sq * ab.zdim;
    const AttnArgs a = ab.seq[sq];
    const int n_chunks = (a.pos0 + a.M + 127) / 128;
    const int n_qg = (a.M * (a.n_heads / a.kv.n_kv_heads) + 15) / 16;
    if ((int)blockIdx.y >= n_chunks || zb * a.qg_per_block >= n_qg) return;
    attn_mfma_body<HD>(a, blockIdx.x, blockIdx.y, zb);
}

// Second stage: one block per (row, query head) merges that row's chunk partials
// (online-softmax rule against the row's overall maximum).  A thread owns two dims;
// the chunks are dealt round-robin to the block's thread groups so that all loads
// of a short context are in flight at once, each group adds its chunks in ascending
// order and the groups are added in index order.  The order depends on the row's
// position only.
template <int HD, int CH>
__device__ __forceinline__ void attn_merge_body(const AttnArgs& a, const int hq, const int r) {
    constexpr int MAXC = 512;
    constexpr int TPG = HD / 2;       // threads per group
    constexpr int NG = 256 / TPG;     // chunk groups
    constexpr int U = 8;              // loads in flight per thread
    __shared__ float sm[MAXC], sl[MAXC];
    __shared__ float red[4];
    __shared__ __attribute__((aligned(8))) float go[NG][HD];
    __shared__ float gl[NG];
    const int tid = threadIdx.x;
    const int grp = tid / TPG, dp = tid % TPG;
    const int Hq = a.n_heads, stride = HD + 2;
    const int nc = (a.pos0 + r) / CH + 1;
    const float* p = a.partials + (size_t)(r * Hq + hq) * a.max_chunks * stride;
    // this thread's first U chunks' values are requested before anything else
    float2 av[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = grp + NG * u;
        av[u] = make_float2(0.f, 0.f);
        if (c < nc) av[u] = *reinterpret_cast<const float2*>(p + (size_t)c * stride + 2 + 2 * dp);
    }
    float mx = -SB_INF;
    for (int c = tid; c < nc; c += 256) {
        const float2 ml = *reinterpret_cast<const float2*>(p + (size_t)c * stride);
        sm[c] = ml.x;
        sl[c] = ml.y;
        mx = fmaxf(mx, ml.x);
    }
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float L = 0.f, O0 = 0.f, O1 = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int c = grp + NG * u;
        if (c < nc) {
            const float w = expf(sm[c] - mx);
            L += sl[c] * w; O0 += av[u].x * w; O1 += av[u].y * w;
        }
    }
    for (int c0 = grp + NG * U; c0 < nc; c0 += NG * U) {  // long contexts: further rounds of U loads
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + NG * u;
            av[u] = make_float2(0.f, 0.f);
            if (c < nc) av[u] = *reinterpret_cast<const float2*>(p + (size_t)c * stride + 2 + 2 * dp);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + NG * u;
            if (c < nc) {
                const float w = expf(sm[c] - mx);
                L += sl[c] * w; O0 += av[u].x * w; O1 += av[u].y * w;
            }
        }
    }
    go[grp][2 * dp] = O0;
    go[grp][2 * dp + 1] = O1;
    if (dp == 0) gl[grp] = L;
    __syncthreads();
    if (tid < HD) {
        float Ls = 0.f, Os = 0.f;
#pragma unroll
        for (int gi = 0; gi < NG; ++gi) { Ls += gl[gi]; Os += go[gi][tid]; }
        const float v = Os / Ls;
        const size_t col = (size_t)hq * HD + tid;
        if (a.out) a.out[(size_t)r * Hq * HD + col] = v;
        if (a.out_split) split_store_rows(a.out_split, Hq * HD, a.split_rows, r, (int)col, v);
    }
}

template <int HD, int CH>
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a) {
    attn_merge_body<HD, CH>(a, blockIdx.x, blockIdx.y);
}

template <int HD, int CH>
__global__ __launch_bounds__(256) void attn_merge_batch_kernel(AttnBatchArgs ab) {
    const AttnArgs a = ab.seq[blockIdx.z];
    if ((int)blockIdx.y >= a.M) return;
    attn_merge_body<HD, CH>(a, blockIdx.x, blockIdx.y);
}

int attn_chunk_keys(int32_t head_dim, int32_t kv_dtype) {
    return (head_dim * (kv_dtype == SB_BF16 ? 2 : 4) <= 256) ? 128 : 64;
}

// Checks one pass's arguments and gives its launch shape: chunks, query groups, groups per block.
static bool attn_shape(const AttnArgs& a, int* n_chunks, int* n_qg, int* qpb) {
    const int hd = a.kv.head_dim;
    if ((hd != 64 && hd != 128) || a.M < 1 || a.M > SB_PREFILL_ROWS || a.n_heads % a.kv.n_kv_heads) return false;
    if (a.out_split && a.split_rows < a.M) return false;
    if (!a.rope_cos || !a.rope_sin) return false;
    const int ch = attn_chunk_keys(hd, a.kv.kv_dtype);
    *n_chunks = (a.pos0 + a.M + ch - 1) / ch;
    if (*n_chunks > a.max_chunks || *n_chunks > 512) return false;
    const int G = a.n_heads / a.kv.n_kv_heads;
    // Query groups of 16: one block each while the launch is small; in a large launch (a prompt
    // pass over a long context) a block takes several groups in turn on one load of its K/V
    // chunk.  A query's result does not depend on the grouping.
    *n_qg = (a.M * G + 15) / 16;
    *qpb = (int)(((long)a.kv.n_kv_heads * *n_chunks * *n_qg + 1023) / 1024);
    if (*qpb > *n_qg) *qpb = *n_qg;
    return true;
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
    const int hd = a.kv.head_dim;
    int n_chunks, n_qg, qpb;
    if (!attn_shape(a, &n_chunks, &n_qg, &qpb)) return hipErrorInvalidValue;
    AttnArgs b = a;
    b.qg_per_block = qpb;
    dim3 grid(a.kv.n_kv_heads, n_chunks, (n_qg + qpb - 1) / qpb);
    dim3 grid1(a.kv.n_kv_heads, n_chunks, n_qg);
    dim3 mgrid(a.n_heads, a.M);
    if (a.kv.kv_dtype == SB_BF16) {
        if (hd == 128) { attn_mfma_kernel<128><<<grid, 256, 0, st>>>(b); attn_merge_kernel<128, 128><<<mgrid, 256, 0, st>>>(a); }
        else { attn_mfma_kernel<64><<<grid, 256, 0, st>>>(b); attn_merge_kernel<64, 128><<<mgrid, 256, 0, st>>>(a); }
    } else {
        if (hd == 128) { attn_kernel<float, 128><<<grid1, 256, 0, st>>>(a); attn_merge_kernel<128, 64><<<mgrid, 256, 0, st>>>(a); }
        else { attn_kernel<float, 64><<<grid1, 256, 0, st>>>(a); attn_merge_kernel<64, 128><<<mgrid, 256, 0, st>>>(a); }
    }
    return hipGetLastError();
}

hipError_t launch_attention_batch(const AttnArgs* seqs, int n, hipStream_t st) {
    if (n < 1 || n > SB_MAX_W) return hipErrorInvalidValue;
    bool one_shape = seqs[0].kv.kv_dtype == SB_BF16;
    for (int i = 1; i < n; ++i)
        one_shape = one_shape && seqs[i].kv.kv_dtype == SB_BF16 && seqs[i].kv.head_dim == seqs[0].kv.head_dim &&
                    seqs[i].kv.n_kv_heads == seqs[0].kv.n_kv_heads && seqs[i].n_heads == seqs[0].n_heads;
    if (n == 1 || !one_shape) {  // (an fp32 cache takes the vector-ALU kernel, a launch per sequence)
        for (int i = 0; i < n; ++i) {
            hipError_t e = launch_attention(seqs[i], st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    AttnBatchArgs ab{};
    int max_chunks = 0, max_m = 0;
    ab.zdim = 1;
    for (int i = 0; i < n; ++i) {
        int n_chunks, n_qg, qpb;
        if (!attn_shape(seqs[i], &n_chunks, &n_qg, &qpb) || seqs[i].M > SB_MAX_W) return hipErrorInvalidValue;
        ab.seq[i] = seqs[i];
        ab.seq[i].qg_per_block = qpb;
        const int z = (n_qg + qpb - 1) / qpb;
        if (z > ab.zdim) ab.zdim = z;
        if (n_chunks > max_chunks) max_chunks = n_chunks;
        if (seqs[i].M > max_m) max_m = seqs[i].M;
    }
    dim3 grid(seqs[0].kv.n_kv_heads, max_chunks, n * ab.zdim);
    dim3 mgrid(seqs[0].n_heads, max_m, n);
    if (seqs[0].kv.head_dim == 128) {
        attn_mfma_batch_kernel<128><<<grid, 256, 0, st>>>(ab);
        attn_merge_batch_kernel<128, 128><<<mgrid, 256, 0, st>>>(ab);
    } else {
        attn_mfma_batch_kernel<64><<<grid, 256, 0, st>>>(ab);
        attn_merge_batch_kernel<64, 128><<<mgrid, 256, 0, st>>>(ab);
    }
    return hipGetLastError();
}

}  // namespace sb
