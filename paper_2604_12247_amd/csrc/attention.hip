// Attention of the decode path over the paged KV cache: rotary embedding and cache append of the new
// rows, partial soft-max attention per 128-key chunk (vector ALUs for an fp32 cache, matrix cores for
// a bf16 cache), the merge of the chunks, and the same for several sequences in one launch pair.
#include "kernels.h"
#include "device_utils.h"

#include <math.h>

namespace sb {

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
// LDS of one block of the matrix-core attention kernels (one work item is computed at a time).
template <int HD>
struct AttnLds {
    static constexpr int CH = 128, QG = 16, QS = HD + 8, PS = CH + 8, SS = CH + 4;   // padded row strides
    __attribute__((aligned(16))) uint16_t q_hi[QG * QS], q_lo[QG * QS];
    __attribute__((aligned(16))) uint16_t p_hi[QG * PS], p_lo[QG * PS];
    __attribute__((aligned(16))) float s_s[QG * SS];
    float s_m[QG], s_l[QG];
};

// One work item of the kernel -- (kv head g, key chunk, slice zb of the query groups) -- in two
// steps: load() requests everything the item reads from memory (the first query group with its
// rotary factors, the chunk's K and V operands) into registers, compute() does the rest.  A block
// that owns several items requests the next item's operands before it computes the current one.
template <int HD>
struct AttnItem {
    static constexpr int CH = 128, QG = 16, HALF = HD / 2;
    static constexpr int KSQ = HD / 32;      // k steps (of 32 dims) of the score product
    static constexpr int KSV = CH / 32;      // k steps (of 32 keys) of the value product
    static constexpr int DT = HD / 64;       // 16-dim output tiles per wave
    static constexpr int QS = HD + 8, PS = CH + 8, SS = CH + 4;
    static constexpr int QIT = QG * HALF / 256;
    int g, chunk, zb;
    float qx[QIT], qy[QIT], qc[QIT], qsn[QIT];
    uint4 kreg[2][KSQ];
    size_t kaddr[2];
    uint4 vreg[DT][KSV];
    size_t vaddr[KSV];

    __device__ __forceinline__ void load_q(const AttnArgs& a, int qg) {
        const int tid = threadIdx.x;
        const int G = a.n_heads / a.kv.n_kv_heads, nq_total = a.M * G;
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
    }

    __device__ __forceinline__ void load(const AttnArgs& a, int g_, int chunk_, int zb_) {
        g = g_; chunk = chunk_; zb = zb_;
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
        (void)lane; (void)wave; (void)li; (void)lq; (void)n_qg; (void)qg_first; (void)qg_last; (void)n_total; (void)scale;
        (void)kbase; (void)vbase; (void)has_new; (void)page_elems; (void)nq_total;
        // ---- every global load of the item: q (+ its rotary factors) of the first group, K, V
        load_q(a, qg_first);
        // K operands: tile t of this wave = keys key0 + wave*32 + t*16 + li (one page), dims ks*32 + lq*8 ..
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

    }

    __device__ __forceinline__ void compute(const AttnArgs& a, AttnLds<HD>& lds) {
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
        (void)lane; (void)wave; (void)li; (void)lq; (void)n_qg; (void)qg_first; (void)qg_last; (void)n_total; (void)scale;
        (void)kbase; (void)vbase; (void)has_new; (void)page_elems; (void)nq_total;
        uint16_t* const q_hi = lds.q_hi; uint16_t* const q_lo = lds.q_lo;
        uint16_t* const p_hi = lds.p_hi; uint16_t* const p_lo = lds.p_lo;
        float* const s_s = lds.s_s; float* const s_m = lds.s_m; float* const s_l = lds.s_l;
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
        if (qg + 1 < qg_last) load_q(a, qg + 1);  // (in flight during this group's products)
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
};

template <int HD>
__device__ __forceinline__ void attn_mfma_body(const AttnArgs& a, const int g, const int chunk, const int zb) {
    __shared__ AttnLds<HD> lds;
    AttnItem<HD> it;
    it.load(a, g, chunk, zb);
    it.compute(a, lds);
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
