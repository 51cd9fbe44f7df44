// Projection kernels of the decode path: y = W x for up to 8 rows sharing one sweep over W, with the
// epilogues of the layer (store, residual + next RMSNorm inputs, SwiGLU, exit / final head partials of
// Eq. 2), on the vector ALUs and on the matrix cores; the tile packing of the weights; the head
// evaluation whose scratch area is a static device array.  As everywhere in this library, a row's
// value never depends on how many rows share the launch.
#include "kernels.h"
#include "device_utils.h"

#include <math.h>
#include <mutex>

namespace sb {

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
                    if (a.ssq_out2) a.ssq_out2[(size_t)m * a.ssq_ld + blockIdx.x * RT + t] = sum;
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
static int mfma_waves(int32_t N) { return N <= 4096 ? 8 : 4; }  // (measured: [6144 x 4096] is 9-12 % faster with four waves and the deeper ring, [5120 x K] the same with either)
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

}  // namespace sb
