// Single-kernel entry points of the C ABI (sb_op_*): one kernel of the decode or prompt path on
// the caller's buffers, used by the parity tests and for roofline measurement.
#include <cmath>

#include "host.h"

using namespace sb;
using namespace sbhost;

extern "C" {

// ---- single kernels -------------------------------------------------------
int32_t sb_op_rmsnorm(const float* x, const float* gain, float* out, int32_t M, int32_t d, float eps, void* stream) {
    if (!x || !gain || !out || M < 1 || M > SB_MAX_W || d < 1) return fail(SB_EINVAL, "op_rmsnorm: bad argument");
    HIP_TRY(launch_rmsnorm(x, gain, out, nullptr, 0, M, d, eps, (hipStream_t)stream));
    return SB_OK;
}

size_t sb_op_gemv_scratch_bytes(int32_t /*M: sized for the maximum*/, int32_t K) { return K > 0 ? align_up((size_t)16 * K * 2, 256) : 0; }

static int op_check(const void* W, int32_t w_dtype, int32_t N, int32_t K, const float* x, int32_t M, int32_t kernel) {
    if (!W || !x) return fail(SB_EINVAL, "op: NULL operand");
    if (w_dtype != SB_FP32 && w_dtype != SB_BF16) return fail(SB_EINVAL, "op: w_dtype");
    if (N < 1 || K < 8 || K % 8 || M < 1 || M > SB_MAX_W) return fail(SB_EINVAL, "op: need N >= 1, K %% 8 == 0, 1 <= M <= %d", SB_MAX_W);
    if (kernel != SB_PROJ_VALU && kernel != SB_PROJ_MFMA && kernel != SB_PROJ_MFMA_PACKED)
        return fail(SB_EINVAL, "op: kernel must be VALU, MFMA or MFMA_PACKED");
    if (kernel != SB_PROJ_VALU && (w_dtype != SB_BF16 || K % 128 || N % 16))
        return fail(SB_EINVAL, "op: MFMA path needs bf16 weights, K %% 128 == 0, N %% 16 == 0");
    if (((uintptr_t)W & 15) || ((uintptr_t)x & 15)) return fail(SB_EINVAL, "op: operands must be 16-byte aligned");
    return SB_OK;
}

int32_t sb_op_gemv(const void* W, int32_t w_dtype, int32_t N, int32_t K, const float* x, float* y, int32_t M,
                   int32_t kernel, void* scratch, void* stream) {
    int rc = op_check(W, w_dtype, N, K, x, M, kernel);
    if (rc) return rc;
    if (!y) return fail(SB_EINVAL, "op_gemv: y is NULL");
    GemvArgs g{};
    g.W = W; g.w_dtype = w_dtype; g.N = N; g.K = K; g.x = x; g.y = y; g.ldy = N; g.M = M; g.epi = EPI_STORE;
    g.packed = kernel == SB_PROJ_MFMA_PACKED;
    if (kernel != SB_PROJ_VALU) {
        if (!scratch || ((uintptr_t)scratch & 15)) return fail(SB_EINVAL, "op_gemv: MFMA path needs aligned scratch");
        g.xs = (uint16_t*)scratch;
        HIP_TRY(launch_split(x, (uint16_t*)scratch, M, K, (hipStream_t)stream));
        HIP_TRY(launch_gemv_mfma(g, (hipStream_t)stream));
    } else {
        HIP_TRY(launch_gemv_valu(g, (hipStream_t)stream));
    }
    return SB_OK;
}

int32_t sb_op_gate_up(const void* W, int32_t w_dtype, int32_t N, int32_t K, const float* x, float* u, int32_t M,
                      int32_t kernel, void* scratch, void* stream) {
    int rc = op_check(W, w_dtype, N, K, x, M, kernel);
    if (rc) return rc;
    if (N > 0x3fffffff) return fail(SB_EINVAL, "op_gate_up: N too large");
    if (!u) return fail(SB_EINVAL, "op_gate_up: u is NULL");
    GemvArgs g{};
    g.W = W; g.w_dtype = w_dtype; g.N = N; g.K = K; g.x = x; g.y = u; g.ldy = N; g.M = M; g.epi = EPI_SWIGLU;
    g.packed = kernel == SB_PROJ_MFMA_PACKED;
    if (kernel != SB_PROJ_VALU) {
        if (!scratch || ((uintptr_t)scratch & 15)) return fail(SB_EINVAL, "op_gate_up: MFMA path needs aligned scratch");
        g.xs = (uint16_t*)scratch;
        HIP_TRY(launch_split(x, (uint16_t*)scratch, M, K, (hipStream_t)stream));
        HIP_TRY(launch_gemv_mfma(g, (hipStream_t)stream));
    } else {
        HIP_TRY(launch_gemv_valu(g, (hipStream_t)stream));
    }
    return SB_OK;
}

int32_t sb_op_repack(const void* W, int32_t N, int32_t K, void* packed, void* stream) {
    if (!W || !packed || ((uintptr_t)W & 15) || ((uintptr_t)packed & 15)) return fail(SB_EINVAL, "op_repack: NULL / misaligned operand");
    if (N < 16 || N % 16 || K < 128 || K % 128) return fail(SB_EINVAL, "op_repack: need N %% 16 == 0 and K %% 128 == 0");
    HIP_TRY(launch_repack(W, packed, N, K, (hipStream_t)stream));
    return SB_OK;
}

size_t sb_op_gemm_scratch_bytes(int32_t N, int32_t K) {
    if (N < 16 || K < 128 || N % 16 || K % 128) return 0;
    return align_up((size_t)2 * SB_PREFILL_ROWS * K * 2, 256) + (size_t)gemm_splits(N, K, 1) * SB_PREFILL_ROWS * N * 4;
}

int32_t sb_op_gemm(const void* Wp, int32_t N, int32_t K, const float* x, float* y, int32_t M, void* scratch,
                   void* stream) {
    if (!Wp || !x || !y || !scratch) return fail(SB_EINVAL, "op_gemm: NULL argument");
    if (N < 16 || K < 128 || N % 16 || K % 128 || M < 1 || M > SB_PREFILL_ROWS)
        return fail(SB_EINVAL, "op_gemm: need N %% 16 == 0, K %% 128 == 0, 1 <= M <= %d", SB_PREFILL_ROWS);
    hipStream_t st = (hipStream_t)stream;
    uint16_t* xs = (uint16_t*)scratch;
    float* part = (float*)((char*)scratch + align_up((size_t)2 * SB_PREFILL_ROWS * K * 2, 256));
    HIP_TRY(launch_prefill_split(x, xs, SB_PREFILL_ROWS, M, K, st));
    GemmArgs g{};
    g.Wp = Wp; g.rows = N; g.K = K; g.xs = xs; g.plane_rows = SB_PREFILL_ROWS; g.M = M; g.n_pass = 1;
    g.part = part; g.S = gemm_splits(N, K, 1);
    HIP_TRY(launch_prefill_gemm(g, st));
    GemmEpiArgs e{};
    e.part = part; e.S = g.S; e.rows = N; e.N = N; e.M = M; e.n_pass = 1; e.plane_rows = SB_PREFILL_ROWS;
    e.epi = EPI_STORE; e.K = K; e.y = y; e.ldy = N;
    HIP_TRY(launch_prefill_epilogue(e, st));
    return SB_OK;
}

size_t sb_op_head_scratch_bytes(int32_t /*M: sized for the maximum*/, int32_t N, int32_t K) {
    if (N < 1 || K < 1) return 0;
    int nb = head_blocks_valu(N);
    return 256 + align_up((size_t)SB_MAX_W * nb * 16, 256) + align_up((size_t)16 * K * 2, 256);
}

int32_t sb_op_head(const void* W, int32_t w_dtype, int32_t N, int32_t K, const float* x, int32_t M, float T,
                   int32_t kernel, int32_t* argmax_out, float* conf_out, float* logits, void* scratch, void* stream) {
    int rc = op_check(W, w_dtype, N, K, x, M, kernel);
    if (rc) return rc;
    if (!argmax_out || !conf_out || !scratch || ((uintptr_t)scratch & 255)) return fail(SB_EINVAL, "op_head: bad output / scratch");
    if (!(T > 0.f)) return fail(SB_EINVAL, "op_head: T must be positive");
    int nb = head_blocks_valu(N);
    char* sc = (char*)scratch;
    GemvArgs g{};
    g.W = W; g.w_dtype = w_dtype; g.N = N; g.K = K; g.x = x; g.M = M; g.epi = EPI_HEAD;
    g.head.T = T; g.head.partials = (float*)(sc + 256);
    g.head.logits = logits; g.head.argmax_out = argmax_out; g.head.conf_out = conf_out; g.head.post = POST_NONE;
    g.packed = kernel == SB_PROJ_MFMA_PACKED;
    if (kernel != SB_PROJ_VALU) {
        g.xs = (uint16_t*)(sc + 256 + align_up((size_t)SB_MAX_W * nb * 16, 256));
        HIP_TRY(launch_split(x, const_cast<uint16_t*>(g.xs), M, K, (hipStream_t)stream));
        HIP_TRY(launch_gemv_mfma(g, (hipStream_t)stream));
    } else {
        HIP_TRY(launch_gemv_valu(g, (hipStream_t)stream));
    }
    return SB_OK;
}

int32_t sb_op_head_static(const void* W, int32_t w_dtype, int32_t N, int32_t K, const float* x, int32_t M, float T,
                          int32_t kernel, int32_t* argmax_out, float* conf_out, void* stream) {
    int rc = op_check(W, w_dtype, N, K, x, M, kernel);
    if (rc) return rc;
    if (!argmax_out || !conf_out) return fail(SB_EINVAL, "op_head_static: NULL output");
    if (!(T > 0.f)) return fail(SB_EINVAL, "op_head_static: T must be positive");
    if (N > SB_STATIC_MAX_N || K > SB_STATIC_MAX_K)
        return fail(SB_ECAPACITY, "op_head_static: N = %d, K = %d exceed the static scratch area (N <= %d, K <= %d)", N, K,
                    SB_STATIC_MAX_N, SB_STATIC_MAX_K);
    static_assert(SB_STATIC_MAX_N % 16 == 0, "partials are sized per 16 output rows");
    void* base = nullptr;
    hipError_t e = static_scratch(&base);   // address of the library's own device array on this GPU
    if (e != hipSuccess) return fail(SB_EDEVICE, "op_head_static: static scratch area: %s", hipGetErrorString(e));
    char* sc = (char*)base;
    const int nb = head_blocks_valu(N);
    GemvArgs g{};
    g.W = W; g.w_dtype = w_dtype; g.N = N; g.K = K; g.x = x; g.M = M; g.epi = EPI_HEAD;
    g.head.T = T; g.head.partials = (float*)(sc + 256);
    g.head.logits = nullptr; g.head.argmax_out = argmax_out; g.head.conf_out = conf_out; g.head.post = POST_NONE;
    g.packed = kernel == SB_PROJ_MFMA_PACKED;
    if (kernel != SB_PROJ_VALU) {
        g.xs = (uint16_t*)(sc + 256 + align_up((size_t)SB_MAX_W * nb * 16, 256));
        HIP_TRY(launch_split(x, const_cast<uint16_t*>(g.xs), M, K, (hipStream_t)stream));
        HIP_TRY(launch_gemv_mfma(g, (hipStream_t)stream));
    } else {
        HIP_TRY(launch_gemv_valu(g, (hipStream_t)stream));
    }
    return SB_OK;
}

int32_t sb_op_copy(void* dst, const void* src, size_t nbytes, void* stream) {
    if (!dst || !src || (nbytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15))
        return fail(SB_EINVAL, "op_copy: NULL / misaligned operand");
    HIP_TRY(launch_copy(dst, src, nbytes, (hipStream_t)stream));
    return SB_OK;
}

int32_t sb_op_read(const void* src, size_t nbytes, float* sink, void* stream) {
    if (!src || !sink || (nbytes & 15) || ((uintptr_t)src & 15)) return fail(SB_EINVAL, "op_read: NULL / misaligned operand");
    HIP_TRY(launch_read(src, nbytes, sink, (hipStream_t)stream));
    return SB_OK;
}

int32_t sb_rope_table_host(int32_t head_dim, float base, int32_t n_pos, float* cos_out, float* sin_out) {
    if (head_dim < 2 || (head_dim & 1) || !(base > 0.f) || n_pos < 0 || !cos_out || !sin_out)
        return fail(SB_EINVAL, "rope_table_host: bad argument");
    const int half = head_dim / 2;
    for (int p = 0; p < n_pos; ++p)
        for (int i = 0; i < half; ++i) {
            double theta = std::pow((double)base, -2.0 * (double)i / (double)head_dim);
            double a = (double)p * theta;
            cos_out[(size_t)p * half + i] = (float)std::cos(a);
            sin_out[(size_t)p * half + i] = (float)std::sin(a);
        }
    return SB_OK;
}

static int attn_op_check(int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, int32_t kv_dtype, const void* pool,
                         const int32_t* table, int32_t n_pages, int32_t layer, int32_t pos0, int32_t M) {
    if (n_heads < 1 || n_kv_heads < 1 || n_heads % n_kv_heads) return fail(SB_EINVAL, "op: head counts");
    if (head_dim != 64 && head_dim != 128) return fail(SB_EINVAL, "op: head_dim must be 64 or 128");
    if (kv_dtype != SB_FP32 && kv_dtype != SB_BF16) return fail(SB_EINVAL, "op: kv_dtype");
    if (!pool || !table || n_pages < 1 || layer < 0) return fail(SB_EINVAL, "op: pool / table");
    if (M < 1 || M > SB_MAX_W || pos0 < 0 || pos0 + M > n_pages * SB_KV_BLOCK)
        return fail(SB_ECAPACITY, "op: rows %d..%d outside the %d-page pool", pos0, pos0 + M - 1, n_pages);
    if ((uintptr_t)pool & 15) return fail(SB_EINVAL, "op: pool must be 16-byte aligned");
    return SB_OK;
}

size_t sb_op_attention_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t kv_dtype, int32_t n_pages) {
    if (n_heads < 1 || n_pages < 1 || (head_dim != 64 && head_dim != 128)) return 0;
    const int ch = attn_chunk_keys(head_dim, kv_dtype);
    const int max_chunks = (n_pages * SB_KV_BLOCK + ch - 1) / ch;
    return align_up((size_t)SB_MAX_W * n_heads * max_chunks * (head_dim + 2) * 4, 256);
}

int32_t sb_op_attention(const float* qkv, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, int32_t kv_dtype,
                        void* pool, const int32_t* table, int32_t n_pages, int32_t layer, const float* rope_cos,
                        const float* rope_sin, int32_t pos0, int32_t M, float* out, void* scratch, void* stream) {
    int rc = attn_op_check(n_heads, n_kv_heads, head_dim, kv_dtype, pool, table, n_pages, layer, pos0, M);
    if (rc) return rc;
    if (!qkv || !out || !rope_cos || !rope_sin || !scratch || ((uintptr_t)scratch & 255))
        return fail(SB_EINVAL, "op_attention: NULL / misaligned operand");
    const int ch = attn_chunk_keys(head_dim, kv_dtype);
    AttnArgs a{};
    a.q = qkv; a.rope_cos = rope_cos; a.rope_sin = rope_sin;
    a.qkv_rows = (n_heads + 2 * n_kv_heads) * head_dim; a.n_heads = n_heads;
    a.kv = KvLayout{pool, table, n_pages, n_kv_heads, head_dim, kv_dtype};
    a.layer = layer; a.pos0 = pos0; a.M = M;
    a.partials = (float*)scratch;
    a.max_chunks = (n_pages * SB_KV_BLOCK + ch - 1) / ch;
    a.out = out; a.out_split = nullptr; a.split_rows = 8;
    HIP_TRY(launch_attention(a, (hipStream_t)stream));
    return SB_OK;
}

int32_t sb_op_prompt_attention(const float* qkv, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, void* pool,
                               const int32_t* table, int32_t n_pages, int32_t layer, const float* rope_cos,
                               const float* rope_sin, int32_t pos0, int32_t M, float* out, void* stream) {
    int rc = attn_op_check(n_heads, n_kv_heads, head_dim, SB_BF16, pool, table, n_pages, layer, pos0, 1);
    if (rc) return rc;
    if (M < 1 || pos0 + (int64_t)M > (int64_t)n_pages * SB_KV_BLOCK)
        return fail(SB_ECAPACITY, "op: rows %d..%lld outside the %d-page pool", pos0, (long long)pos0 + M - 1, n_pages);
    if (!qkv || !out || !rope_cos || !rope_sin) return fail(SB_EINVAL, "op_prompt_attention: NULL operand");
    if (((uintptr_t)qkv | (uintptr_t)out | (uintptr_t)rope_cos | (uintptr_t)rope_sin) & 15)
        return fail(SB_EINVAL, "op_prompt_attention: operands must be 16-byte aligned");
    AttnArgs a{};
    a.q = qkv; a.rope_cos = rope_cos; a.rope_sin = rope_sin;
    a.qkv_rows = (n_heads + 2 * n_kv_heads) * head_dim; a.n_heads = n_heads;
    a.kv = KvLayout{pool, table, n_pages, n_kv_heads, head_dim, SB_BF16};
    a.layer = layer; a.pos0 = pos0; a.M = M;
    a.out = out; a.out_split = nullptr; a.split_rows = M;
    HIP_TRY(launch_prefill_attention(a, (hipStream_t)stream));
    return SB_OK;
}

}  // extern "C"
