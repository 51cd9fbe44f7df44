// gfx950 kernels of the prompt passes: the same decoder layer as a decode pass, for
// up to SB_PREFILL_ROWS rows at once, so that the weights are streamed once per 128
// prompt tokens instead of once per 8 (prefill is the base model's own, Sec. 3.1;
// only its cost matters, not its schedule).
//
// A projection is two kernels.  prefill_gemm_kernel streams the tile-packed bf16
// weights (A operand, straight from HBM into registers, as in the decode path) against
// the rows' activations, which every wave of the block needs and which are therefore
// staged through LDS (B operand; bf16 high and low parts, two MFMAs per weight tile,
// so a product keeps about 16 bits of the activation's mantissa as in the decode
// path).  The work is cut evenly across thread blocks, also along k, so a row of the
// result is left as a few partial sums.  prefill_epilogue_kernel adds them in index
// order, applies the RMSNorm scale and the projection's tail (store, residual + next
// input, SwiGLU).
#include "kernels.h"
#include "device_utils.h"

namespace sb {

namespace {
constexpr int PM = SB_PREFILL_ROWS;
constexpr int ROWB = 272;                  // LDS bytes per staged row: 128 bf16 + 16 bytes of padding
constexpr int STAGE = 2 * PM * ROWB;       // one k block of both planes
constexpr int WPB = 8;                     // waves per thread block (one block per CU: two LDS stages take 136 KB)
}  // namespace

// Work decomposition: the (row block, k block) pairs are numbered row block first and
// cut into equal contiguous ranges, one per thread block, so that every block streams
// the same number of weight bytes whatever the shape (a plain k split leaves a ragged
// last round of blocks on 256 CUs).  A range may end in the middle of a row block: each
// thread block that touches a row block leaves one partial sum for it, in slot
// (range index - first range of that row block).
struct GemmPlan {
    int rt;      // row block = 128 rt weight rows (2 rt tiles per wave)
    int nb;      // row blocks
    int q;       // (row block, k block) pairs per thread block
    int grid;    // thread blocks
    int smax;    // most partial sums a row block can get
};
static GemmPlan gemm_plan(int32_t rows, int32_t K, int32_t n_pass) {
    GemmPlan p;
    const int KB = K >> 7;
    p.rt = rows >= 8192 ? 2 : 1;
    p.nb = (rows + 16 * WPB * p.rt - 1) / (16 * WPB * p.rt);
    const long total = (long)p.nb * KB;
    // resident thread blocks: one per CU (LDS), shared out among the passes of the launch --
    // every pass gets the same cut, so the blocks of different passes that work on the same
    // weights are neighbours in the grid and run at the same time
    int slots = 256 / n_pass;
    if (slots < 1) slots = 1;
    p.q = (int)((total + slots - 1) / slots);
    if (p.q < 2 && KB >= 2) p.q = 2;          // (never one partial per k block)
    p.grid = (int)((total + p.q - 1) / p.q);  // per pass
    p.smax = (KB + p.q - 1) / p.q + 1;
    if (p.smax > KB) p.smax = KB;
    return p;
}
int gemm_splits(int32_t rows, int32_t K, int32_t n_pass) { return gemm_plan(rows, K, n_pass).smax; }

// ---- pieces of the GEMM kernel (all inlined; register arrays are passed by reference) ----
struct GemmCtx {
    const uint16_t* W;      // packed weights + this lane's 16 bytes
    const uint16_t* bsrc0;  // this thread's first staging unit in the activation planes
    int bdst0;              // ... and in an LDS stage
    int K, KB, n_tiles, it1, wr, wt, li, lq;  // wr: the wave's row group (0-3), wt: its token half (0-1)
    int lo_off;             // rows from a high-plane row to its low-plane row
    int Mp, cid, pass;      // live rows of this pass, range index, pass
};

// Weights of half a pair: half-step h = 2 * pair + (0 | 1) covers MFMA steps 2 (h & 1) and
// 2 (h & 1) + 1 of the pair's k block.  (Clamped to the block's range: a re-read of the last
// half keeps the steady-state loop free of conditional loads, whose completion could only be
// waited for conservatively.)  STREAM: the weights are read once by this launch (a single
// pass), so the loads carry the streaming hint; with several passes the other passes' blocks
// read the same lines and they are left to the caches.
template <int RT, bool STREAM>
__device__ __forceinline__ void gemm_load_a(uint4 (&ar)[RT][2], const GemmCtx& c, int h_) {
    const int h = h_ < 2 * c.it1 ? h_ : 2 * c.it1 - 1;
    const int it = h >> 1, b = it / c.KB, kb = it - b * c.KB;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        int tile = (b * 4 + c.wr) * RT + t;
        if (tile > c.n_tiles - 1) tile = c.n_tiles - 1;  // a tile past the end re-reads the last one (not stored)
        const uint16_t* wp = c.W + ((size_t)tile * c.KB + kb) * 2048 + (h & 1) * 1024;
#pragma unroll
        for (int u = 0; u < 2; ++u)
            ar[t][u] = STREAM ? ld_weights_packed(wp + u * 512) : *reinterpret_cast<const uint4*>(wp + u * 512);
    }
}
// Staging map: 2 planes x PM rows x 16 segments of 16 bytes, NBU per thread; unit i of a
// thread lies RPI rows below unit i - 1 (same segment), first in the high plane, then in
// the low plane.  Rows past the live ones are read too, from the planes' unused rows:
// whatever they hold only reaches result columns that are never stored.
constexpr int NBU = 2 * PM * 16 / (64 * WPB);
constexpr int RPI = 4 * WPB;
__device__ __forceinline__ void gemm_load_b(u32x4 (&br)[NBU], const GemmCtx& c, int it_) {
    const int it = it_ < c.it1 ? it_ : c.it1 - 1;
    const int kb = it % c.KB;
#pragma unroll
    for (int i = 0; i < NBU; ++i) {
        const int row = i * RPI < PM ? i * RPI : c.lo_off + i * RPI - PM;  // high plane, then low plane
        br[i] = *reinterpret_cast<const u32x4*>(c.bsrc0 + (size_t)row * c.K + (size_t)kb * 128);
    }
}
__device__ __forceinline__ void gemm_store_b(unsigned char* dst, const u32x4 (&br)[NBU], const GemmCtx& c) {
#pragma unroll
    for (int i = 0; i < NBU; ++i) *reinterpret_cast<u32x4*>(dst + c.bdst0 + i * RPI * ROWB) = br[i];
}
// A wave multiplies its RT weight tiles with the four column tiles (64 rows) of its token
// half: one LDS operand read serves RT MFMAs.  All column tiles are always multiplied, so
// the block of LDS reads and MFMAs stays free of branches.
constexpr int CTW = PM / 32;  // column tiles per wave
template <int RT>
__device__ __forceinline__ void gemm_mma(f32x4 (&acc)[RT][CTW], const uint4 (&ar)[RT][2], const unsigned char* src,
                                         const GemmCtx& c, int uhalf) {
#pragma unroll
    for (int uu = 0; uu < 2; ++uu) {
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) {
            const unsigned char* rp = src + ((c.wt * CTW + ct) * 16 + c.li) * ROWB + (uhalf * 2 + uu) * 64 + c.lq * 16;
            const bf16x8 bh = *reinterpret_cast<const bf16x8*>(rp);
            const bf16x8 bl = *reinterpret_cast<const bf16x8*>(rp + PM * ROWB);
#pragma unroll
            for (int t = 0; t < RT; ++t)
                acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ar[t][uu]), bh, acc[t][ct],
                                                                     0, 0, 0);
#pragma unroll
            for (int t = 0; t < RT; ++t)
                acc[t][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ar[t][uu]), bl, acc[t][ct],
                                                                     0, 0, 0);
        }
    }
}
// Partial sum of row block b (C layout: lane (j = li, g = lq), register r -> weight row 4g + r
// of the tile, activation row j), then zero for the next row block.
template <int RT>
__device__ __forceinline__ void gemm_flush(f32x4 (&acc)[RT][CTW], const GemmArgs& a, const GemmCtx& c, int b, int q) {
    const int slot = c.cid - (b * c.KB) / q;
    float* part = a.part + (size_t)(c.pass * a.S + slot) * PM * a.rows;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int tile = (b * 4 + c.wr) * RT + t;
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) {
            const int m = (c.wt * CTW + ct) * 16 + c.li;
            if (tile < c.n_tiles && m < c.Mp)
                *reinterpret_cast<f32x4*>(part + (size_t)m * a.rows + tile * 16 + 4 * c.lq) = acc[t][ct];
            acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
}

// Half a pair.  First half (P = 0): request the next pair's activations; both halves: request
// the weights two half-steps ahead, multiply the current half; second half (P = 1): leave the
// row block's partial sum if it ends here and publish the next activations (the stage they go
// to was last read before the barrier that ended the previous pair).  Loads complete in issue
// order and the activations are requested before the weights of the same half-step, so
// waiting for them leaves the newest weight loads in flight.
template <int RT, bool STREAM, int P>
__device__ __forceinline__ void gemm_half(f32x4 (&acc)[RT][CTW], const uint4 (&acur)[RT][2], uint4 (&afar)[RT][2],
                                          u32x4 (&breg)[NBU], unsigned char* bt, int& buf, const GemmArgs& a,
                                          const GemmCtx& c, int h, int q) {
    const int cur = h >> 1;
    if (P == 0) gemm_load_b(breg, c, cur + 1);
    gemm_load_a<RT, STREAM>(afar, c, h + 2);
    gemm_mma<RT>(acc, acur, bt + buf * STAGE, c, P);
    if (P == 1) {
        const int b = cur / c.KB;
        if (cur + 1 >= c.it1 || (cur + 1) / c.KB != b) gemm_flush<RT>(acc, a, c, b, q);
        buf ^= 1;
        gemm_store_b(bt + buf * STAGE, breg, c);
        __syncthreads();
    }
}

// 512 threads: four row groups x two token halves; a wave has RT 16-row weight tiles (of the
// block's 64 RT rows) and 64 of the pass's 128 rows, i.e. up to a 64 x 64 tile of the result.
// Weights: a ring of three register half-stages, requested two half-steps (one pair) ahead;
// activations: one pair ahead through LDS.
template <int RT, bool STREAM>
__global__ __launch_bounds__(64 * WPB) void prefill_gemm_kernel(GemmArgs a, int q) {
    static_assert(WPB == 8, "four row groups x two token halves");
    extern __shared__ __attribute__((aligned(16))) unsigned char bt[];  // [2][STAGE]
    const int tid = threadIdx.x, lane = tid & 63;
    GemmCtx c;
    c.wr = (tid >> 6) & 3; c.wt = tid >> 8; c.li = lane & 15; c.lq = lane >> 4;
    c.K = a.K; c.KB = a.K >> 7; c.n_tiles = a.rows >> 4;
    const int nb = (c.n_tiles + 4 * RT - 1) / (4 * RT);
    const int total = nb * c.KB;  // (checked on the host to fit an int)
    c.pass = blockIdx.x % a.n_pass;  // neighbours in the grid: same weights, different passes
    c.cid = blockIdx.x / a.n_pass;
    c.Mp = a.M - c.pass * PM < PM ? a.M - c.pass * PM : PM;
    c.lo_off = a.plane_rows;
    const int it0 = c.cid * q;
    c.it1 = it0 + q < total ? it0 + q : total;
    if (it0 >= c.it1) return;
    c.W = reinterpret_cast<const uint16_t*>(a.Wp) + lane * 8;
    c.bsrc0 = a.xs + (size_t)(c.pass * PM + (tid >> 4)) * a.K + (tid & 15) * 8;
    c.bdst0 = (tid >> 4) * ROWB + (tid & 15) * 16;

    f32x4 acc[RT][CTW];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
    uint4 ah[3][RT][2];  // ring of weight half-stages
    u32x4 breg[NBU];     // (a native vector type: the compiler keeps such an array in registers)

    gemm_load_b(breg, c, it0);
    gemm_load_a<RT, STREAM>(ah[0], c, 2 * it0);
    gemm_load_a<RT, STREAM>(ah[1], c, 2 * it0 + 1);
    gemm_store_b(bt, breg, c);
    __syncthreads();
    int buf = 0;  // LDS stage that holds the current pair's activations
    int it = it0;
    // steady state: three pairs = six half-steps, every ring index a constant
    for (; it + 3 <= c.it1; it += 3) {
        gemm_half<RT, STREAM, 0>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it, q);
        gemm_half<RT, STREAM, 1>(acc, ah[1], ah[0], breg, bt, buf, a, c, 2 * it + 1, q);
        gemm_half<RT, STREAM, 0>(acc, ah[2], ah[1], breg, bt, buf, a, c, 2 * it + 2, q);
        gemm_half<RT, STREAM, 1>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it + 3, q);
        gemm_half<RT, STREAM, 0>(acc, ah[1], ah[0], breg, bt, buf, a, c, 2 * it + 4, q);
        gemm_half<RT, STREAM, 1>(acc, ah[2], ah[1], breg, bt, buf, a, c, 2 * it + 5, q);
    }
    if (it < c.it1) {
        gemm_half<RT, STREAM, 0>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it, q);
        gemm_half<RT, STREAM, 1>(acc, ah[1], ah[0], breg, bt, buf, a, c, 2 * it + 1, q);
    }
    if (it + 1 < c.it1) {
        gemm_half<RT, STREAM, 0>(acc, ah[2], ah[1], breg, bt, buf, a, c, 2 * it + 2, q);
        gemm_half<RT, STREAM, 1>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it + 3, q);
    }
}

hipError_t launch_prefill_gemm(const GemmArgs& a, hipStream_t st) {
    if (a.rows < 16 || a.rows % 16 || a.K < 128 || a.K % 128 || a.M < 1 || a.n_pass < 1 || a.n_pass > SB_PREFILL_PASSES ||
        a.n_pass != (a.M + PM - 1) / PM || a.plane_rows < a.n_pass * PM)
        return hipErrorInvalidValue;
    const GemmPlan p = gemm_plan(a.rows, a.K, a.n_pass);
    if (a.S != p.smax || (long)p.nb * (a.K >> 7) > 0x3fffffffL) return hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        const void* fns[4] = {reinterpret_cast<const void*>(&prefill_gemm_kernel<2, false>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<2, true>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<4, false>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<4, true>)};
        for (const void* fn : fns) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    const int grid = p.grid * a.n_pass;
    const bool stream = a.n_pass == 1;
    if (p.rt == 2) {
        if (stream) prefill_gemm_kernel<4, true><<<grid, 64 * WPB, 2 * STAGE, st>>>(a, p.q);
        else prefill_gemm_kernel<4, false><<<grid, 64 * WPB, 2 * STAGE, st>>>(a, p.q);
    } else {
        if (stream) prefill_gemm_kernel<2, true><<<grid, 64 * WPB, 2 * STAGE, st>>>(a, p.q);
        else prefill_gemm_kernel<2, false><<<grid, 64 * WPB, 2 * STAGE, st>>>(a, p.q);
    }
    return hipGetLastError();
}

// Partial sums that row block b received: thread blocks first..last of the plan.
struct GemmSplitMap { int rows_per_block, KB, q; };
__device__ __forceinline__ int splits_of(const GemmSplitMap& mp, int n) {
    const int b = n / mp.rows_per_block;
    const int first = (int)(((long)b * mp.KB) / mp.q), last = (int)(((long)(b + 1) * mp.KB - 1) / mp.q);
    return last - first + 1;
}

// Partial sums of four neighbouring elements, added in slot order; eight loads in flight at a time.
__device__ __forceinline__ float4 sum_splits4(const float* p, size_t plane, int n_splits) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < n_splits; s0 += 8) {
        float4 t[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            t[i] = s0 + i < n_splits ? *reinterpret_cast<const float4*>(p + (size_t)(s0 + i) * plane) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int i = 0; i < 8; ++i) { v.x += t[i].x; v.y += t[i].y; v.z += t[i].z; v.w += t[i].w; }
    }
    return v;
}
// four values of row m, columns n..n+3 -> the two bf16 planes (8-byte stores)
__device__ __forceinline__ void split_store4(uint16_t* xs, int ld, int lo_rows, int m, int n, float4 v) {
    const uint16_t h0 = f2bf(v.x), h1 = f2bf(v.y), h2 = f2bf(v.z), h3 = f2bf(v.w);
    const uint16_t l0 = f2bf(v.x - bf2f(h0)), l1 = f2bf(v.y - bf2f(h1)), l2 = f2bf(v.z - bf2f(h2)), l3 = f2bf(v.w - bf2f(h3));
    *reinterpret_cast<uint2*>(xs + (size_t)m * ld + n) = make_uint2((uint32_t)h0 | ((uint32_t)h1 << 16), (uint32_t)h2 | ((uint32_t)h3 << 16));
    *reinterpret_cast<uint2*>(xs + (size_t)(lo_rows + m) * ld + n) =
        make_uint2((uint32_t)l0 | ((uint32_t)l1 << 16), (uint32_t)l2 | ((uint32_t)l3 << 16));
}

// grid (ceil(N / 256), ceil(M / 4)), 256 threads: a wave takes one row and 256 columns, a
// lane four neighbouring columns (all in one row block, hence with the same partial sums)
template <int EPI>
__global__ __launch_bounds__(256) void prefill_epilogue_kernel(GemmEpiArgs a, GemmSplitMap mp) {
    const int lane = threadIdx.x & 63;
    const int m = blockIdx.y * 4 + (threadIdx.x >> 6);  // row of the super-pass
    const int n = blockIdx.x * 256 + lane * 4;
    if (m >= a.M) return;
    float inv = 1.0f;
    if (a.ssq_in) {  // (added in index order; sixteen loads in flight at a time)
        float t = 0.f;
        for (int b0 = 0; b0 < a.ssq_nb; b0 += 16) {
            float q[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) q[i] = b0 + i < a.ssq_nb ? a.ssq_in[(size_t)m * a.ssq_ld + b0 + i] : 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) t += q[i];
        }
        inv = 1.0f / sqrtf(t / (float)a.K + a.eps);
    }
    const size_t plane = (size_t)PM * a.rows;
    const float* p = a.part + ((size_t)(m / PM) * a.S * PM + m % PM) * a.rows;
    float sq = 0.f;
    if (n < a.N) {
        if (EPI == EPI_SWIGLU) {
            const float4 g = sum_splits4(p + n, plane, splits_of(mp, n));
            const float4 u = sum_splits4(p + a.N + n, plane, splits_of(mp, a.N + n));
            const float4 v = make_float4(silu_mul(g.x * inv, u.x * inv), silu_mul(g.y * inv, u.y * inv),
                                         silu_mul(g.z * inv, u.z * inv), silu_mul(g.w * inv, u.w * inv));
            split_store4(a.ys, a.N, a.plane_rows, m, n, v);
        } else {
            float4 v = sum_splits4(p + n, plane, splits_of(mp, n));
            v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
            float4* yp = reinterpret_cast<float4*>(a.y + (size_t)m * a.ldy + n);
            if (EPI == EPI_RESID) {
                const float4 y0 = *yp;
                v.x += y0.x; v.y += y0.y; v.z += y0.z; v.w += y0.w;
                if (a.nx) {
                    const float4 gn = *reinterpret_cast<const float4*>(a.gain + n);
                    split_store4(a.nx, a.N, a.plane_rows, m, n, make_float4(v.x * gn.x, v.y * gn.y, v.z * gn.z, v.w * gn.w));
                }
                sq = (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
            }
            *yp = v;
        }
    }
    if (EPI == EPI_RESID && a.ssq_out) {
        sq = wave_sum(sq);
        if (lane == 0) a.ssq_out[(size_t)m * a.ssq_ld + blockIdx.x] = sq;
    }
}

hipError_t launch_prefill_epilogue(const GemmEpiArgs& a, hipStream_t st) {
    if (a.M < 1 || a.N < 1 || a.S < 1 || a.n_pass != (a.M + PM - 1) / PM || a.plane_rows < a.M) return hipErrorInvalidValue;
    if (a.epi == EPI_SWIGLU ? (!a.ys || a.rows != 2 * a.N) : (!a.y || a.rows != a.N)) return hipErrorInvalidValue;
    if (a.ssq_out && (a.N + 255) / 256 > a.ssq_ld) return hipErrorInvalidValue;
    if (a.N % 4 || a.ldy % 4) return hipErrorInvalidValue;
    dim3 grid((a.N + 255) / 256, (a.M + 3) / 4);
    const GemmPlan pl = gemm_plan(a.rows, a.K, a.n_pass);
    if (a.S != pl.smax) return hipErrorInvalidValue;
    const GemmSplitMap mp{16 * WPB * pl.rt, a.K >> 7, pl.q};
    switch (a.epi) {
        case EPI_STORE: prefill_epilogue_kernel<EPI_STORE><<<grid, 256, 0, st>>>(a, mp); break;
        case EPI_RESID: prefill_epilogue_kernel<EPI_RESID><<<grid, 256, 0, st>>>(a, mp); break;
        case EPI_SWIGLU: prefill_epilogue_kernel<EPI_SWIGLU><<<grid, 256, 0, st>>>(a, mp); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// grid (ceil(d / 256), M)
template <typename WT>
__global__ __launch_bounds__(256) void prefill_embed_kernel(const WT* __restrict__ E, int vocab, int d,
                                                            const int32_t* __restrict__ tokens, float* __restrict__ H,
                                                            const float* __restrict__ gain, uint16_t* __restrict__ nx,
                                                            int plane_rows, float* __restrict__ ssq_out, int ssq_ld) {
    __shared__ float red[4];
    const int tid = threadIdx.x, m = blockIdx.y, n = blockIdx.x * 256 + tid;
    int tok = tokens[m];
    if (tok < 0 || tok >= vocab) tok = 0;  // never index outside the table
    float sq = 0.f;
    if (n < d) {
        const float x = ldf(E + (size_t)tok * d + n);
        H[(size_t)m * d + n] = x;
        if (nx) split_store_rows(nx, d, plane_rows, m, n, x * gain[n]);
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
                                int32_t M, float* H, const float* gain, uint16_t* nx, int32_t plane_rows,
                                float* ssq_out, int32_t ssq_ld, hipStream_t st) {
    if (M < 1 || plane_rows < M || (ssq_out && (d + 255) / 256 > ssq_ld)) return hipErrorInvalidValue;
    dim3 grid((d + 255) / 256, M);
    if (w_dtype == SB_BF16)
        prefill_embed_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)E, vocab, d, tokens, H, gain, nx, plane_rows,
                                                              ssq_out, ssq_ld);
    else
        prefill_embed_kernel<float><<<grid, 256, 0, st>>>((const float*)E, vocab, d, tokens, H, gain, nx, plane_rows,
                                                           ssq_out, ssq_ld);
    return hipGetLastError();
}

__global__ void prefill_split_kernel(const float* __restrict__ x, uint16_t* __restrict__ xs, int plane_rows, int K) {
    const int m = blockIdx.y, i = blockIdx.x * 256 + threadIdx.x;
    if (i < K) split_store_rows(xs, K, plane_rows, m, i, x[(size_t)m * K + i]);
}
hipError_t launch_prefill_split(const float* x, uint16_t* xs, int32_t plane_rows, int32_t M, int32_t K, hipStream_t st) {
    if (M < 1 || plane_rows < M) return hipErrorInvalidValue;
    prefill_split_kernel<<<dim3((K + 255) / 256, M), 256, 0, st>>>(x, xs, plane_rows, K);
    return hipGetLastError();
}

}  // namespace sb
