// gfx950 kernels of the prompt passes: the same decoder layer as a decode pass, for
// up to SB_PREFILL_ROWS rows at once, so that the weights are streamed once per 128
// prompt tokens instead of once per 8 (prefill is the base model's own, Sec. 4.3;
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
#include <type_traits>
#include "kernels.h"
#include "device_utils.h"

namespace sb {

namespace {
constexpr int PM = SB_PREFILL_ROWS;
constexpr int ROWB = 288;                  // LDS bytes per staged row: 128 bf16 + 32 bytes of padding (16-byte operand
                                           // reads at rows 272 bytes apart measure as 2-way bank conflicts, at 288 as none)
constexpr int STAGE = 2 * PM * ROWB;       // one k block of both planes
constexpr int WPB = 8;                     // waves per thread block (one block per CU: two LDS stages take 144 KB)
constexpr int LDS_BYTES = 2 * STAGE + PM * 4;  // two stages + the rows' scales
constexpr int BLOCK_ROWS = 256;            // weight rows of a row block: 8 row groups x 2 tiles of 16
}  // namespace

// Work decomposition: the (row block, k block) pairs are numbered row block first and
// cut into equal contiguous ranges, one per thread block, so that every block streams
// the same number of weight bytes whatever the shape (a plain k split leaves a ragged
// last round of blocks on 256 CUs).  A range may end in the middle of a row block: each
// thread block that touches a row block leaves one partial sum for it, in slot
// (range index - first range of that row block).
struct GemmPlan {
    int nb;      // row blocks
    int q;       // (row block, k block) pairs per thread block
    int grid;    // thread blocks
    int smax;    // most partial sums a row block can get
};
static GemmPlan gemm_plan(int32_t rows, int32_t K, int32_t n_pass) {
    GemmPlan p;
    const int KB = K >> 7;
    p.nb = (rows + BLOCK_ROWS - 1) / BLOCK_ROWS;
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
    int K, KB, n_tiles, it1, wr, wt, li, lq;  // wr: the wave's row group, wt: its share of the pass's rows
    int lo_off;             // rows from a high-plane row to its low-plane row
    int Mp, cid, pass;      // live rows of this pass, range index, pass
    int n_out_tiles;        // fused gate/up: 16-column groups of the output (gate tile j pairs with up tile n_out_tiles + j)
};

// Weights of half a pair: half-step h = 2 * pair + (0 | 1) covers MFMA steps 2 (h & 1) and
// 2 (h & 1) + 1 of the pair's k block.  (Clamped to the block's range: a re-read of the last
// half keeps the steady-state loop free of conditional loads, whose completion could only be
// waited for conservatively.)  STREAM: the weights are read once by this launch (a single
// pass), so the loads carry the streaming hint; with several passes the other passes' blocks
// read the same lines and they are left to the caches.
// Weight tile t of this wave in row block b; -1 past the end.  Gate/up with the fused tail: the
// wave's two tiles are the gate and the up tile of one group of 16 outputs.
template <int RT, int RG, int FE>
__device__ __forceinline__ int gemm_tile(const GemmCtx& c, int b, int t) {
    if (FE == 1 + EPI_SWIGLU) {
        const int j = b * RG + c.wr;
        return j < c.n_out_tiles ? (t == 0 ? j : c.n_out_tiles + j) : -1;
    }
    const int tile = (b * RG + c.wr) * RT + t;
    return tile < c.n_tiles ? tile : -1;
}
template <int RT, bool STREAM, int RG, int FE>
__device__ __forceinline__ void gemm_load_a(uint4 (&ar)[RT][2], const GemmCtx& c, int h_) {
    const int h = h_ < 2 * c.it1 ? h_ : 2 * c.it1 - 1;
    const int it = h >> 1, b = it / c.KB, kb = it - b * c.KB;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        int tile = gemm_tile<RT, RG, FE>(c, b, t);
        if (tile < 0) tile = c.n_tiles - 1;  // a tile past the end re-reads the last one (not stored)
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
// A wave multiplies its RT weight tiles with the CTW column tiles (16 rows each) of its share of
// the pass: one LDS operand read serves RT MFMAs.  All column tiles are always multiplied, so
// the block of LDS reads and MFMAs stays free of branches.
template <int RT, int CTW>
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
    // issue order for the compiler's scheduler: two operand reads, 2 RT MFMAs, and so on (1 % faster
    // than its own choice)
#pragma unroll
    for (int i = 0; i < 2 * CTW; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * RT, 0);
    }
}
// Partial sum of row block b (C layout: lane (j = li, g = lq), register r -> weight row 4g + r
// of the tile, activation row j), then zero for the next row block.
template <int RT, int RG, int CTW, int FE>
__device__ __forceinline__ void gemm_flush(f32x4 (&acc)[RT][CTW], const GemmArgs& a, const GemmCtx& c, int b, int q,
                                           const float* s_inv) {
    const int first = (b * c.KB) / q;
    const bool whole = first == ((b + 1) * c.KB - 1) / q;  // the row block's whole k range was this thread block's
    if (FE == 1 + EPI_STORE && whole) {
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            const int tile = gemm_tile<RT, RG, FE>(c, b, t);
#pragma unroll
            for (int ct = 0; ct < CTW; ++ct) {
                const int m = (c.wt * CTW + ct) * 16 + c.li;
                if (tile >= 0 && m < c.Mp) {
                    const float inv = s_inv[m];
                    *reinterpret_cast<float4*>(a.y + (size_t)(c.pass * PM + m) * a.ldy + tile * 16 + 4 * c.lq) =
                        make_float4(acc[t][ct][0] * inv, acc[t][ct][1] * inv, acc[t][ct][2] * inv, acc[t][ct][3] * inv);
                }
                acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
        return;
    }
    if (FE == 1 + EPI_SWIGLU && whole) {
        // register r of lane (li, lq): output 16 j + 4 lq + r of row li of the column tile, gate in tile 0, up in tile 1
        const int j = b * RG + c.wr;
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) {
            const int m = (c.wt * CTW + ct) * 16 + c.li;
            if (j < c.n_out_tiles && m < c.Mp) {
                const float inv = s_inv[m];
                const float4 v = make_float4(silu_mul(acc[0][ct][0] * inv, acc[RT - 1][ct][0] * inv), silu_mul(acc[0][ct][1] * inv, acc[RT - 1][ct][1] * inv),
                                             silu_mul(acc[0][ct][2] * inv, acc[RT - 1][ct][2] * inv), silu_mul(acc[0][ct][3] * inv, acc[RT - 1][ct][3] * inv));
                split_store4(a.ys, a.N, a.plane_rows, c.pass * PM + m, j * 16 + 4 * c.lq, v);
            }
#pragma unroll
            for (int t = 0; t < RT; ++t) acc[t][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        return;
    }
    const int slot = c.cid - first;
    float* part = a.part + (size_t)(c.pass * a.S + slot) * PM * a.rows;
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int tile = gemm_tile<RT, RG, FE>(c, b, t);
#pragma unroll
        for (int ct = 0; ct < CTW; ++ct) {
            const int m = (c.wt * CTW + ct) * 16 + c.li;
            if (tile >= 0 && m < c.Mp)
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
template <int RT, bool STREAM, int P, int RG, int CTW, int FE>
__device__ __forceinline__ void gemm_half(f32x4 (&acc)[RT][CTW], const uint4 (&acur)[RT][2], uint4 (&afar)[RT][2],
                                          u32x4 (&breg)[NBU], unsigned char* bt, int& buf, const GemmArgs& a,
                                          const GemmCtx& c, int h, int q) {
    const int cur = h >> 1;
    if (P == 0) gemm_load_b(breg, c, cur + 1);
    gemm_load_a<RT, STREAM, RG, FE>(afar, c, h + 2);
    gemm_mma<RT, CTW>(acc, acur, bt + buf * STAGE, c, P);
    if (P == 1) {
        const int b = cur / c.KB;
        if (cur + 1 >= c.it1 || (cur + 1) / c.KB != b) gemm_flush<RT, RG, CTW, FE>(acc, a, c, b, q, reinterpret_cast<const float*>(bt + 2 * STAGE));
        buf ^= 1;
        gemm_store_b(bt + buf * STAGE, breg, c);
        __syncthreads();
    }
}

// 512 threads = RG row groups x (8 / RG) splits of the pass's 128 rows; a wave has RT 16-row weight
// tiles (of the block's 16 RG RT weight rows) and 16 RG of the pass's rows.  Used with RG = 8, RT = 2:
// 256 weight rows per block, a 32 x 128 tile of the result per wave, every wave loading weights of
// its own.  (Four row groups x two halves of the pass, a 64 x 64 tile per wave, read every weight
// tile in two waves: the vector memory path was busy 64 % of the time instead of 46 %, the launches
// took 4-5 % longer on the wide projections and 20 % longer on the narrow ones at 16 passes.)
// Weights: a ring of three register half-stages, requested two half-steps (one pair) ahead;
// activations: one pair ahead through LDS.
template <int RT, bool STREAM, int RG, int FE>
__global__ __launch_bounds__(64 * WPB) void prefill_gemm_kernel(GemmArgs a, int q, int xa) {
    static_assert(WPB == 8 && (RG == 4 || RG == 8), "row groups x splits of the pass's rows");
    constexpr int CTW = PM / 16 / (WPB / RG);  // column tiles (16 of the pass's rows) per wave
    extern __shared__ __attribute__((aligned(16))) unsigned char bt[];  // [2][STAGE], then PM floats: the rows' RMSNorm scales (fused tails)
    const int tid = threadIdx.x, lane = tid & 63;
    GemmCtx c;
    c.wr = (tid >> 6) % RG; c.wt = (tid >> 6) / RG; c.li = lane & 15; c.lq = lane >> 4;
    c.K = a.K; c.KB = a.K >> 7; c.n_tiles = a.rows >> 4;
    constexpr bool SWI = FE == 1 + EPI_SWIGLU;
    static_assert(!SWI || RT == 2, "a gate and an up tile per wave");
    c.n_out_tiles = SWI ? a.N >> 4 : 0;
    const int nb = SWI ? (c.n_out_tiles + RG - 1) / RG : (c.n_tiles + RG * RT - 1) / (RG * RT);
    const int total = nb * c.KB;  // (checked on the host to fit an int)
    // Thread blocks go to the 8 XCDs round-robin by index.  The blocks that share a range of the
    // weights (same range index, different passes) are given indices of one residue mod 8, so that
    // they meet in one L2 and each L2 fetches an eighth of the layer's weights instead of all of them.
    // Here the 8 XCDs form an xa x (8 / xa) array: range indices are dealt to its rows, passes to its
    // columns, so the weights of a range are fetched by 8 / xa of the L2s and the activations of a
    // pass by xa of them (xa is chosen on the host).
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int xb = 8 / xa, npb = (a.n_pass + xb - 1) / xb;
    c.pass = (j % npb) * xb + xcd / xa;
    c.cid = (j / npb) * xa + xcd % xa;
    if (c.pass >= a.n_pass) return;
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
    gemm_load_a<RT, STREAM, RG, FE>(ah[0], c, 2 * it0);
    gemm_load_a<RT, STREAM, RG, FE>(ah[1], c, 2 * it0 + 1);
    gemm_store_b(bt, breg, c);
    if (FE != 0) {  // 1 / rms of this pass's input rows, from the partial sums of squares their producer left
        const int m = tid >> 2, part = tid & 3;
        float t = 0.f;
        if (a.ssq_in && m < c.Mp)
            for (int i = part; i < a.ssq_nb; i += 4) t += a.ssq_in[(size_t)(c.pass * PM + m) * a.ssq_ld + i];
        t += __shfl_xor(t, 1, 64);
        t += __shfl_xor(t, 2, 64);
        if (part == 0) reinterpret_cast<float*>(bt + 2 * STAGE)[m] = a.ssq_in ? 1.0f / sqrtf(t / (float)a.K + a.eps) : 1.0f;
    }
    __syncthreads();
    int buf = 0;  // LDS stage that holds the current pair's activations
    int it = it0;
    // steady state: three pairs = six half-steps, every ring index a constant
    for (; it + 3 <= c.it1; it += 3) {
        gemm_half<RT, STREAM, 0, RG, CTW, FE>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it, q);
        gemm_half<RT, STREAM, 1, RG, CTW, FE>(acc, ah[1], ah[0], breg, bt, buf, a, c, 2 * it + 1, q);
        gemm_half<RT, STREAM, 0, RG, CTW, FE>(acc, ah[2], ah[1], breg, bt, buf, a, c, 2 * it + 2, q);
        gemm_half<RT, STREAM, 1, RG, CTW, FE>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it + 3, q);
        gemm_half<RT, STREAM, 0, RG, CTW, FE>(acc, ah[1], ah[0], breg, bt, buf, a, c, 2 * it + 4, q);
        gemm_half<RT, STREAM, 1, RG, CTW, FE>(acc, ah[2], ah[1], breg, bt, buf, a, c, 2 * it + 5, q);
    }
    if (it < c.it1) {
        gemm_half<RT, STREAM, 0, RG, CTW, FE>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it, q);
        gemm_half<RT, STREAM, 1, RG, CTW, FE>(acc, ah[1], ah[0], breg, bt, buf, a, c, 2 * it + 1, q);
    }
    if (it + 1 < c.it1) {
        gemm_half<RT, STREAM, 0, RG, CTW, FE>(acc, ah[2], ah[1], breg, bt, buf, a, c, 2 * it + 2, q);
        gemm_half<RT, STREAM, 1, RG, CTW, FE>(acc, ah[0], ah[2], breg, bt, buf, a, c, 2 * it + 3, q);
    }
}

hipError_t launch_prefill_gemm(const GemmArgs& a, hipStream_t st) {
    if (a.rows < 16 || a.rows % 16 || a.K < 128 || a.K % 128 || a.M < 1 || a.n_pass < 1 || a.n_pass > SB_PREFILL_PASSES ||
        a.n_pass != (a.M + PM - 1) / PM || a.plane_rows < a.n_pass * PM)
        return hipErrorInvalidValue;
    const GemmPlan p = gemm_plan(a.rows, a.K, a.n_pass);
    if (a.S != p.smax || (long)p.nb * (a.K >> 7) > 0x3fffffffL) return hipErrorInvalidValue;
    if (a.fused != 0 && a.fused != 1 + EPI_STORE && a.fused != 1 + EPI_SWIGLU) return hipErrorInvalidValue;
    if (a.fused == 1 + EPI_SWIGLU && (a.rows != 2 * a.N || a.N % 16 || !a.ys)) return hipErrorInvalidValue;
    if (a.fused == 1 + EPI_STORE && (a.rows != a.N || !a.y || a.ldy < a.N || a.ldy % 4)) return hipErrorInvalidValue;
    if (a.fused && a.ssq_in && (a.ssq_nb < 1 || a.ssq_ld < a.ssq_nb)) return hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        const void* fns[6] = {reinterpret_cast<const void*>(&prefill_gemm_kernel<2, false, 8, 0>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<2, true, 8, 0>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<2, false, 8, 1 + EPI_STORE>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<2, true, 8, 1 + EPI_STORE>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<2, false, 8, 1 + EPI_SWIGLU>),
                              reinterpret_cast<const void*>(&prefill_gemm_kernel<2, true, 8, 1 + EPI_SWIGLU>)};
        for (const void* fn : fns) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    // XCD array shape, by measurement at the 7B shapes: with few passes the weights dominate what the
    // L2s fetch (one L2 per range: 8 % faster than every L2 fetching everything at 4 passes); with many
    // passes the activations weigh as much and 2 x 4 is 2 % ahead of both 8 x 1 and 1 x 8
    const int xa = a.n_pass >= 8 ? 2 : (a.n_pass >= 5 ? 4 : 8);
    const int xb = 8 / xa;
    const int grid = 8 * ((a.n_pass + xb - 1) / xb) * ((p.grid + xa - 1) / xa);
    const bool stream = a.n_pass == 1;
    const dim3 g3(grid), b3(64 * WPB);
    if (a.fused == 1 + EPI_SWIGLU) {
        if (stream) prefill_gemm_kernel<2, true, 8, 1 + EPI_SWIGLU><<<g3, b3, LDS_BYTES, st>>>(a, p.q, xa);
        else prefill_gemm_kernel<2, false, 8, 1 + EPI_SWIGLU><<<g3, b3, LDS_BYTES, st>>>(a, p.q, xa);
    } else if (a.fused == 1 + EPI_STORE) {
        if (stream) prefill_gemm_kernel<2, true, 8, 1 + EPI_STORE><<<g3, b3, LDS_BYTES, st>>>(a, p.q, xa);
        else prefill_gemm_kernel<2, false, 8, 1 + EPI_STORE><<<g3, b3, LDS_BYTES, st>>>(a, p.q, xa);
    } else {
        if (stream) prefill_gemm_kernel<2, true, 8, 0><<<g3, b3, LDS_BYTES, st>>>(a, p.q, xa);
        else prefill_gemm_kernel<2, false, 8, 0><<<g3, b3, LDS_BYTES, st>>>(a, p.q, xa);
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
        if (EPI == EPI_SWIGLU && a.fused) {
            // (row blocks are 128 outputs: gate and up tiles side by side; one partial = finished by the GEMM)
            const int sp = splits_of(mp, n);
            if (sp > 1) {
                const float4 g = sum_splits4(p + n, plane, sp);
                const float4 u = sum_splits4(p + a.N + n, plane, sp);
                const float4 v = make_float4(silu_mul(g.x * inv, u.x * inv), silu_mul(g.y * inv, u.y * inv),
                                             silu_mul(g.z * inv, u.z * inv), silu_mul(g.w * inv, u.w * inv));
                split_store4(a.ys, a.N, a.plane_rows, m, n, v);
            }
        } else if (EPI == EPI_SWIGLU) {
            const float4 g = sum_splits4(p + n, plane, splits_of(mp, n));
            const float4 u = sum_splits4(p + a.N + n, plane, splits_of(mp, a.N + n));
            const float4 v = make_float4(silu_mul(g.x * inv, u.x * inv), silu_mul(g.y * inv, u.y * inv),
                                         silu_mul(g.z * inv, u.z * inv), silu_mul(g.w * inv, u.w * inv));
            split_store4(a.ys, a.N, a.plane_rows, m, n, v);
        } else if (EPI == EPI_STORE && a.fused && splits_of(mp, n) == 1) {
            // (finished by the GEMM)
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
    if (a.fused && a.fused != 1 + a.epi) return hipErrorInvalidValue;
    const GemmSplitMap mp{a.epi == EPI_SWIGLU && a.fused ? BLOCK_ROWS / 2 : BLOCK_ROWS, a.K >> 7, pl.q};
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

// ---------------------------------------------------------------- prompt attention
// The prompt's attention for a bf16 cache: first the keys and values of all rows of the
// super-pass go into the cache (rotary embedding on the keys, both rounded to bf16; V
// transposed per page, as everywhere), then one launch computes every row's attention with
// the running-softmax scheme: a block owns 64 queries of one kv head (rows x the heads of
// its group, 128 in the wide form), walks the 64-key chunks up to its last row's position and
// keeps the running maximum, the sum and the weighted values of each query in registers -- no
// per-chunk partials, no merge pass.  Both products run on the matrix cores with hi + lo pairs
// for the fp32 side (queries, probabilities) like the decode kernel; a query's result depends
// only on its own column of the accumulators, not on the other queries of the block.
//
// grid (pages touched, n_kv_heads), 256 threads: a block writes one head's part of one page --
// K as 16-byte pieces (8 dims of a key), V transposed as 16-byte pieces (8 keys of a dim);
// where the rows cover a page only partly, the V pieces go out key by key.
template <int HD>
__global__ __launch_bounds__(256) void prefill_kv_append_kernel(AttnArgs a) {
    constexpr int HALF = HD / 2, PPK = HD / 8;
    const int g = blockIdx.y, tid = threadIdx.x;
    const int Hq = a.n_heads, Hkv = a.kv.n_kv_heads;
    const int n_total = a.pos0 + a.M;
    const int lpage = a.pos0 / SB_KV_BLOCK + blockIdx.x;
    const int key_lo = lpage * SB_KV_BLOCK > a.pos0 ? lpage * SB_KV_BLOCK : a.pos0;
    const int key_hi = (lpage + 1) * SB_KV_BLOCK < n_total ? (lpage + 1) * SB_KV_BLOCK : n_total;  // keys key_lo .. key_hi - 1
    const size_t page_elems = (size_t)Hkv * SB_KV_BLOCK * HD;
    const size_t page = (size_t)a.kv.table[lpage] * page_elems;
    uint16_t* const kdst = reinterpret_cast<uint16_t*>(a.kv.pool) + (size_t)(a.layer * 2 + 0) * a.kv.n_pages * page_elems + page + (size_t)g * SB_KV_BLOCK * HD;
    uint16_t* const vdst = reinterpret_cast<uint16_t*>(a.kv.pool) + (size_t)(a.layer * 2 + 1) * a.kv.n_pages * page_elems + page + (size_t)g * SB_KV_BLOCK * HD;
    for (int idx = tid; idx < SB_KV_BLOCK * PPK; idx += 256) {
        const int t = idx / PPK, d0 = (idx - t * PPK) * 8;
        const int key = lpage * SB_KV_BLOCK + t;
        if (key < key_lo || key >= key_hi) continue;
        const bool lower = d0 < HALF;
        const int j0 = lower ? d0 : d0 - HALF;
        const float* kp = a.q + (size_t)(key - a.pos0) * a.qkv_rows + (size_t)(Hq + g) * HD;
        const float* cp = a.rope_cos + (size_t)key * HALF + j0;
        const float* sp = a.rope_sin + (size_t)key * HALF + j0;
        uint32_t w[4];
#pragma unroll
        for (int e4 = 0; e4 < 8; e4 += 4) {
            const float4 x = *reinterpret_cast<const float4*>(kp + j0 + e4);
            const float4 y = *reinterpret_cast<const float4*>(kp + j0 + HALF + e4);
            const float4 c = *reinterpret_cast<const float4*>(cp + e4);
            const float4 sn = *reinterpret_cast<const float4*>(sp + e4);
            const float u0 = lower ? x.x * c.x - y.x * sn.x : y.x * c.x + x.x * sn.x;
            const float u1 = lower ? x.y * c.y - y.y * sn.y : y.y * c.y + x.y * sn.y;
            const float u2 = lower ? x.z * c.z - y.z * sn.z : y.z * c.z + x.z * sn.z;
            const float u3 = lower ? x.w * c.w - y.w * sn.w : y.w * c.w + x.w * sn.w;
            w[e4 / 2] = (uint32_t)f2bf(u0) | ((uint32_t)f2bf(u1) << 16);
            w[e4 / 2 + 1] = (uint32_t)f2bf(u2) | ((uint32_t)f2bf(u3) << 16);
        }
        *reinterpret_cast<uint4*>(kdst + (size_t)t * HD + d0) = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (int idx = tid; idx < HD * 2; idx += 256) {
        const int dim = idx >> 1, t0 = (idx & 1) * 8;
        const int key0 = lpage * SB_KV_BLOCK + t0;
        const float* vp = a.q + (size_t)(Hq + Hkv + g) * HD + dim;
        uint16_t b[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            const int key = key0 + x;
            b[x] = (key >= key_lo && key < key_hi) ? f2bf(vp[(size_t)(key - a.pos0) * a.qkv_rows]) : (uint16_t)0;
        }
        uint16_t* dst = vdst + (size_t)dim * SB_KV_BLOCK + t0;
        if (key0 >= key_lo && key0 + 8 <= key_hi) {
            *reinterpret_cast<uint4*>(dst) = make_uint4(b[0] | ((uint32_t)b[1] << 16), b[2] | ((uint32_t)b[3] << 16), b[4] | ((uint32_t)b[5] << 16), b[6] | ((uint32_t)b[7] << 16));
        } else {
#pragma unroll
            for (int x = 0; x < 8; ++x)
                if (key0 + x >= key_lo && key0 + x < key_hi) dst[x] = b[x];
        }
    }
}

// grid (n_kv_heads, ceil(M G / (64 QT))), 256 threads.  A wave owns QT tiles of 16 queries and
// is independent of the other waves but for the K/V chunk (64 keys) the block stages in LDS.
// Scores are computed transposed, S^T = K Q^T, so a lane holds, for ONE query (its column),
// the scores of 4 keys per key tile: the running maximum, sum and rescaling are per-lane
// scalars, and the exponentials -- 4 keys of tile 2s, then 4 of tile 2s+1 -- are already the
// B operand of O^T += V^T P^T when the 32 keys of a k step are taken in that order, which is
// the order the A operand is read in from the transposed V page (two 8-byte runs per lane).
template <int HD, int QT>
__global__ __launch_bounds__(256, 2) void prefill_attn_kernel(AttnArgs a) {
    constexpr int CH = 64, KT = CH / 16, HALF = HD / 2;
    constexpr int KSQ = HD / 32;             // k steps (32 dims) of the score product
    constexpr int DTN = HD / 16;             // 16-dim tiles of the output
    constexpr int PPK = HD / 8;              // 16-byte pieces of a key
    constexpr int SLAB = SB_KV_BLOCK * HD;   // one head's part of a page
    constexpr int NL = KT * SLAB / (256 * 8);  // 16-byte pieces per thread, operand and chunk
    // Two chunks in LDS, filled by direct global -> LDS loads (lane l of a wave lands 16 l bytes
    // after the wave's base).  Which piece lands where is chosen so that operand reads are free of
    // bank conflicts (measured): a K piece (key, p) sits at piece p ^ f(key) of its key's row; the two
    // halves (8 keys each) of a V row change places in every second group of 8 dims.
    __shared__ __attribute__((aligned(16))) uint16_t k_s[2][CH * HD];
    __shared__ __attribute__((aligned(16))) uint16_t v_s[2][KT * SLAB];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, lq = lane >> 4;
    const int g = blockIdx.x;
    const int qtile = gridDim.y - 1 - blockIdx.y;  // the longest blocks (last rows) start first
    const int Hq = a.n_heads, Hkv = a.kv.n_kv_heads, G = Hq / Hkv;
    const int nq_total = a.M * G, q0 = qtile * (64 * QT);
    const int n_total = a.pos0 + a.M;
    const int q_last = (q0 + 64 * QT < nq_total ? q0 + 64 * QT : nq_total) - 1;
    const int n_chunks = (a.pos0 + q_last / G) / CH + 1;  // chunks with a key the block's last row sees
    const int wq0 = q0 + wave * QT * 16;                   // the wave's queries: wq0 .. wq1
    const int wq1 = (wq0 + QT * 16 - 1 < nq_total - 1) ? wq0 + QT * 16 - 1 : nq_total - 1;
    const bool wave_live = wq0 < nq_total;
    const int wpos_min = a.pos0 + wq0 / G, wpos_max = a.pos0 + wq1 / G;
    const float c2 = 1.4426950408889634f / sqrtf((float)HD);  // scores in units of log 2
    const size_t page_elems = (size_t)Hkv * SLAB;
    const uint16_t* const kbase = reinterpret_cast<const uint16_t*>(a.kv.pool) + (size_t)(a.layer * 2 + 0) * a.kv.n_pages * page_elems;
    const uint16_t* const vbase = reinterpret_cast<const uint16_t*>(a.kv.pool) + (size_t)(a.layer * 2 + 1) * a.kv.n_pages * page_elems;

    // ---- this wave's rotated queries as hi + lo B operands: lane (li, lq) has query li, dims 32 ks + 8 lq ..
    bf16x8 qh[QT][KSQ], ql[QT][KSQ];
    int qpos[QT], qrow[QT], qhead[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const int qq = wq0 + qt * 16 + li;
        const bool valid = qq < nq_total;
        const int r = valid ? qq / G : 0, gi = valid ? qq - r * G : 0;
        qrow[qt] = valid ? r : -1;
        qhead[qt] = g * G + gi;
        qpos[qt] = valid ? a.pos0 + r : 0x7fffffff;  // (a query past the end: zeros, nothing masked, never stored)
        const float* qp = a.q + (size_t)r * a.qkv_rows + (size_t)qhead[qt] * HD;
        const float* cp = a.rope_cos + (size_t)(a.pos0 + r) * HALF;
        const float* sp = a.rope_sin + (size_t)(a.pos0 + r) * HALF;
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            const int d0 = ks * 32 + lq * 8;
            const bool lower = d0 < HALF;
            const int j0 = lower ? d0 : d0 - HALF;
            uint16_t h[8], l[8];
#pragma unroll
            for (int e4 = 0; e4 < 8; e4 += 4) {
                const float4 x = *reinterpret_cast<const float4*>(qp + j0 + e4);
                const float4 y = *reinterpret_cast<const float4*>(qp + j0 + HALF + e4);
                const float4 c = *reinterpret_cast<const float4*>(cp + j0 + e4);
                const float4 sn = *reinterpret_cast<const float4*>(sp + j0 + e4);
                const float xs4[4] = {x.x, x.y, x.z, x.w}, ys4[4] = {y.x, y.y, y.z, y.w};
                const float cs4[4] = {c.x, c.y, c.z, c.w}, sn4[4] = {sn.x, sn.y, sn.z, sn.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float u = lower ? xs4[e] * cs4[e] - ys4[e] * sn4[e] : ys4[e] * cs4[e] + xs4[e] * sn4[e];
                    u = valid ? u * c2 : 0.f;  // scores come out in units of log 2
                    h[e4 + e] = f2bf(u);
                    l[e4 + e] = f2bf(u - bf2f(h[e4 + e]));
                }
            }
            const uint4 hv = make_uint4(h[0] | ((uint32_t)h[1] << 16), h[2] | ((uint32_t)h[3] << 16), h[4] | ((uint32_t)h[5] << 16), h[6] | ((uint32_t)h[7] << 16));
            const uint4 lv = make_uint4(l[0] | ((uint32_t)l[1] << 16), l[2] | ((uint32_t)l[3] << 16), l[4] | ((uint32_t)l[5] << 16), l[6] | ((uint32_t)l[7] << 16));
            qh[qt][ks] = __builtin_bit_cast(bf16x8, hv);
            ql[qt][ks] = __builtin_bit_cast(bf16x8, lv);
        }
    }

    f32x4 o[QT][DTN];  // O^T: register r of lane (li, lq) is dim 16 dt + 4 lq + r of query li
    float m_run[QT], l_run[QT];  // running maximum (log-2 units); this lane's part of the running sum
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_run[qt] = -__builtin_inff();
        l_run[qt] = 0.f;
#pragma unroll
        for (int dt = 0; dt < DTN; ++dt) o[qt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- staging of a chunk: thread -> 16-byte pieces of the chunk's 4 pages (K and V slabs of head g)
    int pg[NL];  // physical pages of the chunk issued next (-1: no key there); read one chunk ahead of the issue
    auto lookup = [&](int chunk) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int page = chunk * KT + (i * 256 + tid) / (SB_KV_BLOCK * PPK);
            pg[i] = (page * SB_KV_BLOCK < n_total) ? a.kv.table[page] : -1;
        }
    };
    auto issue = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int slot = i * 256 + tid;             // the piece's place in LDS
            const int key = slot / PPK, pp = slot - key * PPK;
            const int piece = pp ^ (PPK == 16 ? (key & 15) : ((key >> 1) & 7));
            uint16_t* kw = &k_s[buf][(i * 256 + wave * 64) * 8];  // the wave's 64 pieces
            uint16_t* vw = &v_s[buf][(i * 256 + wave * 64) * 8];
            if (pg[i] >= 0) {
                const size_t base = (size_t)pg[i] * page_elems + (size_t)g * SLAB;
                __builtin_amdgcn_global_load_lds(kbase + base + (key % SB_KV_BLOCK) * HD + piece * 8, kw, 16, 0, 0);
                __builtin_amdgcn_global_load_lds(vbase + base + ((slot ^ ((slot >> 4) & 1)) * 8) % SLAB, vw, 16, 0, 0);
            } else {  // past the last key: zeros
                *reinterpret_cast<u32x4*>(kw + lane * 8) = u32x4{0u, 0u, 0u, 0u};
                *reinterpret_cast<u32x4*>(vw + lane * 8) = u32x4{0u, 0u, 0u, 0u};
            }
        }
    };
    const int kswz = PPK == 16 ? li : ((li >> 1) & 7);  // f(key) of this lane's key in a score operand
    const int vq = (((lq >> 1) ^ (li >> 3)) & 1) * 8 + (lq & 1) * 4;  // this lane's 4 keys within a V row in LDS

    lookup(0);
    issue(0);
    lookup(1);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    for (int chunk = 0; chunk < n_chunks; ++chunk) {
        const int key0 = chunk * CH, buf = chunk & 1;
        if (chunk + 1 < n_chunks) {
            issue(buf ^ 1);
            lookup(chunk + 2);
        }
        if (key0 + CH > n_total) {
            // The last page has slots past the last key; what V holds there would meet a zero
            // probability, and 0 x (stale bits that read as NaN) is not 0: zeros instead.  (K needs
            // nothing: those scores are masked.)  Once per block at most.
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int slot = i * 256 + tid;
                const int vk = key0 + (slot / (SB_KV_BLOCK * PPK)) * SB_KV_BLOCK + ((slot ^ (slot >> 4)) & 1) * 8;  // keys vk .. vk+7 of one dim
                if (vk < n_total && vk + 8 > n_total) {
                    u32x4 vv = *reinterpret_cast<u32x4*>(&v_s[buf][slot * 8]);
#pragma unroll
                    for (int x = 0; x < 8; ++x)
                        if (vk + x >= n_total) vv[x >> 1] &= (x & 1) ? 0x0000ffffu : 0xffff0000u;
                    *reinterpret_cast<u32x4*>(&v_s[buf][slot * 8]) = vv;
                } else if (vk >= n_total && vk < (n_total + SB_KV_BLOCK - 1) / SB_KV_BLOCK * SB_KV_BLOCK) {
                    *reinterpret_cast<u32x4*>(&v_s[buf][slot * 8]) = u32x4{0u, 0u, 0u, 0u};
                }
            }
            __syncthreads();
        }
        if (wave_live && key0 <= wpos_max) {
            // ---- S^T = K Q^T for the 4 key tiles
            f32x4 st[KT][QT];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) st[kt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KSQ; ++ks) {
                    const bf16x8 kop = *reinterpret_cast<const bf16x8*>(&k_s[buf][((kt * 16 + li) * PPK + ((ks * 4 + lq) ^ kswz)) * 8]);
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) {
                        st[kt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, qh[qt][ks], st[kt][qt], 0, 0, 0);
                        st[kt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, ql[qt][ks], st[kt][qt], 0, 0, 0);
                    }
                }
            }
            // ---- running soft-max of each query (register r of tile kt: key key0 + 16 kt + 4 lq + r)
            bf16x8 ph[QT][KT / 2], pl[QT][KT / 2];
            auto soft = [&](auto masked) {
#pragma unroll
                for (int qt = 0; qt < QT; ++qt) {
                    float mx = -__builtin_inff();
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            if (decltype(masked)::value && key0 + kt * 16 + 4 * lq + r > qpos[qt]) st[kt][qt][r] = -__builtin_inff();
                            mx = fmaxf(mx, st[kt][qt][r]);
                        }
                    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
                    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
                    const float m_new = fmaxf(m_run[qt], mx);  // finite from the first chunk on: key 0 is visible to all
                    const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_new);
                    m_run[qt] = m_new;
                    float sum = 0.f;
                    uint32_t hw[KT][2], lw[KT][2];
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                        for (int r = 0; r < 4; r += 2) {
                            const float p0 = __builtin_amdgcn_exp2f(st[kt][qt][r] - m_new);
                            const float p1 = __builtin_amdgcn_exp2f(st[kt][qt][r + 1] - m_new);
                            sum += p0 + p1;
                            const uint32_t hp = pack_bf16(p0, p1);
                            hw[kt][r >> 1] = hp;
                            lw[kt][r >> 1] = pack_bf16(p0 - __uint_as_float(hp << 16), p1 - __uint_as_float(hp & 0xffff0000u));
                        }
                    l_run[qt] = l_run[qt] * alpha + sum;
#pragma unroll
                    for (int s2 = 0; s2 < KT / 2; ++s2) {
                        ph[qt][s2] = __builtin_bit_cast(bf16x8, make_uint4(hw[2 * s2][0], hw[2 * s2][1], hw[2 * s2 + 1][0], hw[2 * s2 + 1][1]));
                        pl[qt][s2] = __builtin_bit_cast(bf16x8, make_uint4(lw[2 * s2][0], lw[2 * s2][1], lw[2 * s2 + 1][0], lw[2 * s2 + 1][1]));
                    }
                    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // (no query of the tile has a new maximum: nothing to rescale)
#pragma unroll
                        for (int dt = 0; dt < DTN; ++dt)
#pragma unroll
                            for (int r = 0; r < 4; ++r) o[qt][dt][r] *= alpha;
                    }
                }
            };
            if (key0 + CH - 1 > wpos_min) soft(std::true_type{});
            else soft(std::false_type{});
            // ---- O^T += V^T P^T: k step s2 = keys (tile 2 s2: 4 lq ..+3, tile 2 s2 + 1: 4 lq ..+3) per lane group
#pragma unroll
            for (int s2 = 0; s2 < KT / 2; ++s2)
#pragma unroll
                for (int dt = 0; dt < DTN; ++dt) {
                    const uint2 v0 = *reinterpret_cast<const uint2*>(&v_s[buf][(2 * s2) * SLAB + (dt * 16 + li) * SB_KV_BLOCK + vq]);
                    const uint2 v1 = *reinterpret_cast<const uint2*>(&v_s[buf][(2 * s2 + 1) * SLAB + (dt * 16 + li) * SB_KV_BLOCK + vq]);
                    const bf16x8 vop = __builtin_bit_cast(bf16x8, make_uint4(v0.x, v0.y, v1.x, v1.y));
#pragma unroll
                    for (int qt = 0; qt < QT; ++qt) {
                        o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, ph[qt][s2], o[qt][dt], 0, 0, 0);
                        o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pl[qt][s2], o[qt][dt], 0, 0, 0);
                    }
                }
        }
        __builtin_amdgcn_s_waitcnt(0);  // this wave's pieces of the next chunk have landed
        __syncthreads();                // ... and everybody's; every wave is done with this chunk
    }
    // ---- normalise; a lane has 4 neighbouring dims per tile of its query
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        float lt = l_run[qt];
        lt += __shfl_xor(lt, 16, 64);
        lt += __shfl_xor(lt, 32, 64);
        if (qrow[qt] < 0) continue;
        const float inv_l = 1.0f / lt;
#pragma unroll
        for (int dt = 0; dt < DTN; ++dt) {
            const int col = qhead[qt] * HD + dt * 16 + 4 * lq;
            const float4 val = make_float4(o[qt][dt][0] * inv_l, o[qt][dt][1] * inv_l, o[qt][dt][2] * inv_l, o[qt][dt][3] * inv_l);
            if (a.out) *reinterpret_cast<float4*>(a.out + (size_t)qrow[qt] * Hq * HD + col) = val;
            else split_store4(a.out_split, Hq * HD, a.split_rows, qrow[qt], col, val);
        }
    }
}

// M rows at positions pos0.. (bf16 cache): append their K/V, then attention of all rows,
// output as floats (out) or as bf16 planes (out_split / split_rows as in launch_attention).
hipError_t launch_prefill_attention(const AttnArgs& a, hipStream_t st) {
    const int hd = a.kv.head_dim;
    if ((hd != 64 && hd != 128) || a.kv.kv_dtype != SB_BF16 || a.M < 1 || a.n_heads % a.kv.n_kv_heads ||
        (!a.out && (!a.out_split || a.split_rows < a.M)) || !a.rope_cos || !a.rope_sin)
        return hipErrorInvalidValue;
    const int G = a.n_heads / a.kv.n_kv_heads, nq = a.M * G;
    // 32 queries per wave halve the LDS reads per product; 16 fill the chip at smaller sizes
    const bool wide = (int64_t)a.kv.n_kv_heads * ((nq + 127) / 128) >= 512;
    dim3 agrid((a.pos0 + a.M - 1) / SB_KV_BLOCK - a.pos0 / SB_KV_BLOCK + 1, a.kv.n_kv_heads), grid(a.kv.n_kv_heads, wide ? (nq + 127) / 128 : (nq + 63) / 64);
    if (hd == 128) {
        prefill_kv_append_kernel<128><<<agrid, 256, 0, st>>>(a);
        if (wide) prefill_attn_kernel<128, 2><<<grid, 256, 0, st>>>(a);
        else prefill_attn_kernel<128, 1><<<grid, 256, 0, st>>>(a);
    } else {
        prefill_kv_append_kernel<64><<<agrid, 256, 0, st>>>(a);
        if (wide) prefill_attn_kernel<64, 2><<<grid, 256, 0, st>>>(a);
        else prefill_attn_kernel<64, 1><<<grid, 256, 0, st>>>(a);
    }
    return hipGetLastError();
}

}  // namespace sb
