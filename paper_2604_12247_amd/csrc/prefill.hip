// gfx950 kernels of the prompt passes: the same decoder layer as a decode pass, for
// up to SB_PREFILL_ROWS rows at once, so that the weights are streamed once per 64
// prompt tokens instead of once per 8 (prefill is the base model's own, Sec. 3.1;
// only its cost matters, not its schedule).
//
// A projection is two kernels.  prefill_gemm_kernel streams the tile-packed bf16
// weights (A operand, straight from HBM into registers, as in the decode path) against
// the rows' activations, which every wave of the block needs and which are therefore
// staged through LDS (B operand; bf16 high and low parts, two MFMAs per weight tile,
// so a product keeps about 16 bits of the activation's mantissa as in the decode
// path).  The k range is split across blocks to fill the chip; each split leaves a
// partial sum.  prefill_epilogue_kernel adds the splits in index order, applies the
// RMSNorm scale and the projection's tail (store, residual + next input, SwiGLU).
#include "kernels.h"
#include "device_utils.h"

namespace sb {

namespace {
constexpr int PM = SB_PREFILL_ROWS;
constexpr int ROWB = 272;                  // LDS bytes per staged row: 128 bf16 + 16 bytes of padding
constexpr int STAGE = 2 * PM * ROWB;       // one k block of both planes
}  // namespace

// grid (ceil(rows / (64 RT)), S); 256 threads = 4 waves, each RT 16-row weight tiles
template <int RT>
__global__ __launch_bounds__(256) void prefill_gemm_kernel(GemmArgs a) {
    constexpr int CT = PM / 16;  // 16-row column tiles of the activations
    extern __shared__ __attribute__((aligned(16))) unsigned char bt[];  // [2][STAGE]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int K = a.K, KB = K >> 7;
    const int KBS = (KB + a.S - 1) / a.S;
    const int kb0 = blockIdx.y * KBS, kb1 = (kb0 + KBS < KB) ? kb0 + KBS : KB;
    if (kb0 >= kb1) return;
    const int n_tiles = a.rows >> 4;
    const int ctl = (a.M + 15) >> 4;  // live column tiles

    const uint16_t* wp[RT];
    int rt[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        rt[t] = (blockIdx.x * 4 + wave) * RT + t;
        const int c = rt[t] < n_tiles ? rt[t] : n_tiles - 1;  // a tile past the end re-reads the last one (not stored)
        wp[t] = reinterpret_cast<const uint16_t*>(a.Wp) + (size_t)c * KB * 2048 + lane * 8;
    }
    // staging map: 2 planes x 64 rows x 16 segments of 16 bytes, 8 per thread
    const uint16_t* bsrc[8];
    int bdst[8];
    bool bact[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int unit = tid + 256 * i;
        const int plane = unit >> 10, row = (unit >> 4) & 63, seg = unit & 15;
        bact[i] = row < a.M;
        bsrc[i] = a.xs + (size_t)(plane * PM + row) * K + seg * 8;
        bdst[i] = (plane * PM + row) * ROWB + seg * 16;
    }

    f32x4 acc[RT][CT];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int c = 0; c < CT; ++c) acc[t][c] = f32x4{0.f, 0.f, 0.f, 0.f};

    uint4 abuf[2][RT][4], breg[8];
    auto load_a = [&](uint4 (&ar)[RT][4], int kb) {
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int u = 0; u < 4; ++u) ar[t][u] = ld_weights_packed(wp[t] + (size_t)kb * 2048 + u * 512);
    };
    auto load_b = [&](int kb) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            breg[i] = bact[i] ? *reinterpret_cast<const uint4*>(bsrc[i] + (size_t)kb * 128) : make_uint4(0, 0, 0, 0);
    };
    auto store_b = [&](unsigned char* dst) {
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<uint4*>(dst + bdst[i]) = breg[i];
    };
    auto mma = [&](const uint4 (&ar)[RT][4], const unsigned char* src) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int c = 0; c < CT; ++c) {
                if (c < ctl) {
                    const unsigned char* rp = src + (c * 16 + li) * ROWB + u * 64 + lq * 16;
                    const bf16x8 bh = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(rp));
                    const bf16x8 bl = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(rp + PM * ROWB));
#pragma unroll
                    for (int t = 0; t < RT; ++t) {
                        const bf16x8 av = __builtin_bit_cast(bf16x8, ar[t][u]);
                        acc[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bh, acc[t][c], 0, 0, 0);
                        acc[t][c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, bl, acc[t][c], 0, 0, 0);
                    }
                }
            }
        }
    };
    // one k block: request the next block's operands, multiply the current one, then
    // publish the next activations (the buffer they go to was last read before the
    // barrier that ended the previous block)
    auto step = [&](const uint4 (&acur)[RT][4], uint4 (&anxt)[RT][4], unsigned char* bcur, unsigned char* bnxt, int kb) {
        const bool more = kb + 1 < kb1;
        if (more) { load_a(anxt, kb + 1); load_b(kb + 1); }
        mma(acur, bcur);
        if (more) store_b(bnxt);
        __syncthreads();
    };

    load_a(abuf[0], kb0);
    load_b(kb0);
    store_b(bt);
    __syncthreads();
    for (int kb = kb0; kb < kb1; kb += 2) {
        step(abuf[0], abuf[1], bt, bt + STAGE, kb);
        if (kb + 1 < kb1) step(abuf[1], abuf[0], bt + STAGE, bt, kb + 1);
    }

    // C layout: lane (j = li, g = lq), register r -> weight row 4g + r of the tile, activation row j
    float* part = a.part + (size_t)blockIdx.y * PM * a.rows;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        if (rt[t] >= n_tiles) continue;
#pragma unroll
        for (int c = 0; c < CT; ++c) {
            const int m = c * 16 + li;
            if (m < a.M) *reinterpret_cast<f32x4*>(part + (size_t)m * a.rows + rt[t] * 16 + 4 * lq) = acc[t][c];
        }
    }
}

static int gemm_row_tiles(int32_t rows) { return rows >= 8192 ? 2 : 1; }

// k splits: enough blocks for the chip, never an empty split
int gemm_splits(int32_t rows, int32_t K) {
    const int KB = K >> 7;
    const int nb = (rows + 64 * gemm_row_tiles(rows) - 1) / (64 * gemm_row_tiles(rows));
    int S = (640 + nb - 1) / nb;
    if (S > 16) S = 16;
    if (S > KB) S = KB;
    if (S < 1) S = 1;
    const int KBS = (KB + S - 1) / S;
    return (KB + KBS - 1) / KBS;
}

hipError_t launch_prefill_gemm(const GemmArgs& a, hipStream_t st) {
    if (a.rows < 16 || a.rows % 16 || a.K < 128 || a.K % 128 || a.M < 1 || a.M > PM || a.S < 1 || a.S > (a.K >> 7))
        return hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_gemm_kernel<1>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_gemm_kernel<2>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int rtl = gemm_row_tiles(a.rows);
    dim3 grid((a.rows + 64 * rtl - 1) / (64 * rtl), a.S);
    if (rtl == 2) prefill_gemm_kernel<2><<<grid, 256, 2 * STAGE, st>>>(a);
    else prefill_gemm_kernel<1><<<grid, 256, 2 * STAGE, st>>>(a);
    return hipGetLastError();
}

// grid (ceil(N / 256), M): thread = one output element
template <int EPI>
__global__ __launch_bounds__(256) void prefill_epilogue_kernel(GemmEpiArgs a) {
    __shared__ float red[4];
    const int tid = threadIdx.x, m = blockIdx.y, n = blockIdx.x * 256 + tid;
    float inv = 1.0f;
    if (a.ssq_in) {
        float t = 0.f;
        for (int b = 0; b < a.ssq_nb; ++b) t += a.ssq_in[(size_t)m * a.ssq_ld + b];
        inv = 1.0f / sqrtf(t / (float)a.K + a.eps);
    }
    const size_t plane = (size_t)PM * a.rows;
    const float* p = a.part + (size_t)m * a.rows;
    float sq = 0.f;
    if (n < a.N) {
        if (EPI == EPI_SWIGLU) {
            float g = 0.f, u = 0.f;
            for (int s = 0; s < a.S; ++s) { g += p[s * plane + n]; u += p[s * plane + a.N + n]; }
            split_store_rows(a.ys, a.N, PM, m, n, silu_mul(g * inv, u * inv));
        } else {
            float v = 0.f;
            for (int s = 0; s < a.S; ++s) v += p[s * plane + n];
            v *= inv;
            float* yp = a.y + (size_t)m * a.ldy + n;
            if (EPI == EPI_RESID) {
                v += *yp;
                if (a.nx) split_store_rows(a.nx, a.N, PM, m, n, v * a.gain[n]);
                sq = v * v;
            }
            *yp = v;
        }
    }
    if (EPI == EPI_RESID && a.ssq_out) {
        sq = wave_sum(sq);
        if ((tid & 63) == 0) red[tid >> 6] = sq;
        __syncthreads();
        if (tid == 0) a.ssq_out[(size_t)m * a.ssq_ld + blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
    }
}

hipError_t launch_prefill_epilogue(const GemmEpiArgs& a, hipStream_t st) {
    if (a.M < 1 || a.M > PM || a.N < 1 || a.S < 1) return hipErrorInvalidValue;
    if (a.epi == EPI_SWIGLU ? (!a.ys || a.rows != 2 * a.N) : (!a.y || a.rows != a.N)) return hipErrorInvalidValue;
    if (a.ssq_out && (a.N + 255) / 256 > a.ssq_ld) return hipErrorInvalidValue;
    dim3 grid((a.N + 255) / 256, a.M);
    switch (a.epi) {
        case EPI_STORE: prefill_epilogue_kernel<EPI_STORE><<<grid, 256, 0, st>>>(a); break;
        case EPI_RESID: prefill_epilogue_kernel<EPI_RESID><<<grid, 256, 0, st>>>(a); break;
        case EPI_SWIGLU: prefill_epilogue_kernel<EPI_SWIGLU><<<grid, 256, 0, st>>>(a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// grid (ceil(d / 256), M)
template <typename WT>
__global__ __launch_bounds__(256) void prefill_embed_kernel(const WT* __restrict__ E, int vocab, int d,
                                                            const int32_t* __restrict__ tokens, float* __restrict__ H,
                                                            const float* __restrict__ gain, uint16_t* __restrict__ nx,
                                                            float* __restrict__ ssq_out, int ssq_ld) {
    __shared__ float red[4];
    const int tid = threadIdx.x, m = blockIdx.y, n = blockIdx.x * 256 + tid;
    int tok = tokens[m];
    if (tok < 0 || tok >= vocab) tok = 0;  // never index outside the table
    float sq = 0.f;
    if (n < d) {
        const float x = ldf(E + (size_t)tok * d + n);
        H[(size_t)m * d + n] = x;
        if (nx) split_store_rows(nx, d, PM, m, n, x * gain[n]);
        sq = x * x;
    }
    if (ssq_out) {
        sq = wave_sum(sq);
        if ((tid & 63) == 0) red[tid >> 6] = sq;
        __syncthreads();
        if (tid == 0) ssq_out[(size_t)m * ssq_ld + blockIdx.x] = ((red[0] + red[1]) + red[2]) + red[3];
    }
}

hipError_t launch_prefill_embed(const void* E, int32_t w_dtype, int32_t vocab, int32_t d, const int32_t* tokens,
                                int32_t M, float* H, const float* gain, uint16_t* nx, float* ssq_out, int32_t ssq_ld,
                                hipStream_t st) {
    if (M < 1 || M > PM || (ssq_out && (d + 255) / 256 > ssq_ld)) return hipErrorInvalidValue;
    dim3 grid((d + 255) / 256, M);
    if (w_dtype == SB_BF16)
        prefill_embed_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)E, vocab, d, tokens, H, gain, nx, ssq_out, ssq_ld);
    else
        prefill_embed_kernel<float><<<grid, 256, 0, st>>>((const float*)E, vocab, d, tokens, H, gain, nx, ssq_out, ssq_ld);
    return hipGetLastError();
}

__global__ void prefill_split_kernel(const float* __restrict__ x, uint16_t* __restrict__ xs, int K) {
    const int m = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i < K) split_store_rows(xs, K, PM, m, i, x[(size_t)m * K + i]);
}
hipError_t launch_prefill_split(const float* x, uint16_t* xs, int32_t M, int32_t K, hipStream_t st) {
    if (M < 1 || M > PM) return hipErrorInvalidValue;
    prefill_split_kernel<<<dim3((K + 255) / 256, M), 256, 0, st>>>(x, xs, K);
    return hipGetLastError();
}

}  // namespace sb
