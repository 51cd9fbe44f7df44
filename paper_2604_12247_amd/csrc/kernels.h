// Internal launch interface between the host state machine and the HIP kernels.
// Plain pointers and sizes; every function enqueues on `stream` and returns the
// launch status.  Operand shapes are validated by the callers (host side).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/specbound.h"

namespace sb {

// rows of one prompt pass (the decode passes have at most SB_MAX_W)
#define SB_PREFILL_ROWS 128

// ---- device-resident record of the current round (read back once per sync) ----
struct DevRound {
    int32_t slot_tok[SB_MAX_W + 1];  // input token of each row (row 0: pending token)
    int32_t drafts[SB_MAX_W];        // drafted token of each row
    int32_t exit_layer[SB_MAX_W];    // exit layer of each row, 0 = none
    float conf[SB_MAX_W];            // confidence at the row's last evaluated head
    int32_t head_argmax[SB_MAX_W];   // arg max at the row's last evaluated head
    int32_t exit_flag;               // set by the head kernel when the current row exits
    int32_t g[SB_MAX_W];             // verification: greedy token after each row
    float gconf[SB_MAX_W];           // verification: max softmax probability (T = 1)
    int32_t n_matched, n_emit;
};

struct RowToks { int32_t tok[SB_MAX_W]; };  // >= 0: host-known id; -1: read slot_tok on the device

// RMSNorm outputs produced together with an embedding row (first layer's input).
struct EmbedNorm { const float* gain; uint16_t* nx; float* ssq_out; int32_t ssq_ld; };

enum Epilogue { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_HEAD = 3 };
enum HeadPost { POST_NONE = 0, POST_EXIT = 1, POST_ACCEPT = 2 };

// What the merge stage of a head evaluation does once the arg max / confidence
// of all rows are known.
struct HeadArgs {
    float T;               // temperature of Eq. 2
    float* partials;       // [M][n_blocks][4] (max, index, sum, -)
    float* logits;         // optional [M][N] store of z (parity tap), else nullptr
    int32_t* argmax_out;   // optional [M]
    float* conf_out;       // optional [M]
    int32_t post;          // HeadPost
    DevRound* round;       // for POST_EXIT / POST_ACCEPT
    int32_t slot;          // POST_EXIT: row being drafted
    int32_t layer;         // POST_EXIT: 1-based layer of this head
    int32_t forced_exit;   // POST_EXIT: -1 computed, 0 never, else exit iff == layer
    int32_t forced_draft;  // POST_EXIT: >= 0 overrides the drafted id
    float threshold;       // POST_EXIT
    int32_t n_drafts;      // POST_ACCEPT
    int32_t* note;         // POST_EXIT, optional: five ints in host memory the device can write (mapped, coherent) --
                           // the merge leaves {note_seq, exit?, drafted id or -1, confidence bits, arg max} there,
                           // the sequence number last, so that the host can read the decision without a copy
    int32_t note_seq;
    int32_t row0;          // merge: the M rows merged are rows row0 .. row0 + M - 1 of the partials
    int32_t skip_merge;    // projection launch: leave the partials, the caller launches the merges itself
    // POST_EXIT, optional (embed_E != nullptr): when the row exits, the merge also embeds the
    // drafted token as the row after it -- embed_H: that row of the hidden cache, embed_en:
    // what the first layer's projection reads for it (as the embedding kernel leaves it)
    const void* embed_E;
    int32_t embed_dtype, embed_vocab, embed_d;
    float* embed_H;
    EmbedNorm embed_en;
};

struct GemvArgs {
    const void* W;     // [rows][K] row-major, bf16 bits or float; or the packed tile layout (MFMA path)
    int32_t packed;    // W is in the packed tile layout written by launch_repack
    int32_t w_dtype;   // SB_FP32 / SB_BF16
    int32_t N;         // outputs per row of x (EPI_SWIGLU: d_ffn, W has 2N rows)
    int32_t K;
    const float* x;    // [M][K] float (VALU path)
    const uint16_t* xs;  // MFMA path: split bf16 operand, [16][K]: rows 0-7 high parts, 8-15 low parts
    float* y;          // [M][ldy]: STORE writes, RESID adds, SWIGLU writes silu(g)*u (float)
    uint16_t* ys;      // MFMA pipeline: optional split-bf16 copy of the output [16][ldy]
    int32_t ldy;
    int32_t M;
    uint32_t row_mask; // 0: rows 0..M-1 of x / y; else bit m set = row (slot) m takes part (MFMA path, M ignored)
    int32_t epi;       // Epilogue
    HeadArgs head;     // EPI_HEAD
    // RMSNorm folded into the MFMA projections.  Input side: xs holds the two bf16
    // parts of gain * h (not yet scaled); the kernel multiplies its outputs by
    // 1/sqrt(sum_sq/K + eps), sum_sq = ssq_in[m][0..ssq_nb) added in index order.
    const float* ssq_in;  // nullptr: xs is used as it is
    int32_t ssq_nb, ssq_ld;
    float eps;
    // Output side (EPI_RESID): after h += y, also write the parts of gainA * h to nxA
    // (and of gainB * h to nxB) and the sum of squares of the block's 16-row tile
    // to ssq_out[m][tile]; all row-major with the leading dimension of y / ssq_ld.
    const float* gainA; uint16_t* nxA;
    const float* gainB; uint16_t* nxB;
    float* ssq_out;
    float* ssq_out2;   // optional second copy of the same sums (for a reader on another stream)
};

// Sampling-mode acceptance over the final-head logits of the M verified rows (device, [M][V]).
struct SampleArgs {
    const float* logits;
    float* wts;   // scratch [M][V - 32768] for the soft-max weights of a vocabulary's tokens from 32768 on (unused below that)
    int32_t V, M, n_drafts;
    float temp, top_p;
    float ua[SB_MAX_W], ur[SB_MAX_W];  // per row: uniform of the acceptance test, uniform of the draw
    DevRound* round;                   // reads drafts[], writes g[], gconf[] (= P(draft)), n_matched, n_emit
};
hipError_t launch_sample_accept(const SampleArgs& a, hipStream_t st);

// Second stage of a head evaluation (launched by launch_gemv_* unless head.skip_merge is set).
hipError_t launch_head_merge(const HeadArgs& h, int32_t M, int32_t nb, hipStream_t st);
// The same for the first n entries (n <= SB_MAX_W sequences, M[i] rows each) in one launch.
struct HeadMergeBatch {
    HeadArgs h[SB_MAX_W];
    int32_t M[SB_MAX_W];
};
hipError_t launch_head_merge_batch(const HeadMergeBatch& hb, int32_t n, int32_t nb, hipStream_t st);
int head_blocks_valu(int32_t N);
int head_blocks_mfma(int32_t N);

hipError_t launch_embed(const void* E, int32_t w_dtype, int32_t vocab, int32_t d, float* H, int32_t M,
                        RowToks toks, const int32_t* slot_tok, int32_t* exit_flag_to_clear, EmbedNorm en,
                        hipStream_t st);
hipError_t launch_rmsnorm(const float* x, const float* gain, float* out, uint16_t* out_split, int32_t ld_split,
                          int32_t M, int32_t d, float eps, hipStream_t st);
hipError_t launch_gemv_valu(const GemvArgs& a, hipStream_t st);
hipError_t launch_gemv_mfma(const GemvArgs& a, hipStream_t st);
// bf16 W [N][K] row-major -> packed MFMA tile layout (N % 16 == 0, K % 128 == 0), same size
hipError_t launch_repack(const void* W, void* P, int32_t N, int32_t K, hipStream_t st);
hipError_t launch_split(const float* x, uint16_t* xs, int32_t M, int32_t K, hipStream_t st);

struct KvLayout {
    void* pool;            // [layer][2][n_pages][n_kv_heads][SB_KV_BLOCK][head_dim]; V slabs of a bf16
                           // pool are transposed: [head_dim][SB_KV_BLOCK]
    const int32_t* table;  // logical page -> physical page (device)
    int32_t n_pages, n_kv_heads, head_dim, kv_dtype;
};

struct AttnArgs {
    const float* q;      // [M][qkv_rows]: raw projections, q heads, then k heads, then v heads
    const float* rope_cos;  // [pos][head_dim/2]
    const float* rope_sin;
    int32_t qkv_rows, n_heads;
    KvLayout kv;
    int32_t layer, pos0, M;
    float* partials;     // [M*n_heads][max_chunks][head_dim + 2]
    int32_t max_chunks;
    float* out;          // [M][n_heads*head_dim]
    uint16_t* out_split; // optional bf16 hi/lo copy: rows 0.. high parts, rows split_rows.. low parts
    int32_t split_rows;  // 8 for decode passes, SB_PREFILL_ROWS for prompt passes
    int32_t qg_per_block;  // set by launch_attention
};
int attn_chunk_keys(int32_t head_dim, int32_t kv_dtype);
hipError_t launch_attention(const AttnArgs& a, hipStream_t st);
// The passes of up to SB_MAX_W sequences (each on its own cache, at most SB_MAX_W rows) in one
// pair of launches; every value equals the one launch_attention computes for that sequence.
struct AttnBatchArgs {
    AttnArgs seq[SB_MAX_W];
    int32_t zdim;  // query-group slices per sequence in grid.z
};
hipError_t launch_attention_batch(const AttnArgs* seqs, int n, hipStream_t st);
// The prompt's attention for a bf16 cache: K/V append for all M rows, then every row's attention
// with a running softmax per query (no partials; `partials` is not used); M is not limited.
hipError_t launch_prefill_attention(const AttnArgs& a, hipStream_t st);

// ---- prompt passes: SB_PREFILL_ROWS rows each, against tile-packed bf16 weights ----
// Up to SB_PREFILL_PASSES passes of one layer go into one launch (a "super-pass"), so
// that the passes' thread blocks meet on the same weights in the caches.  Activations
// come as bf16 planes xs [2][plane_rows][K] (high parts, then low parts; row r of pass p
// is row p * SB_PREFILL_ROWS + r); the product is left as k-split partial sums
// part [n_pass][S][SB_PREFILL_ROWS][rows] for the epilogue that follows.
#define SB_PREFILL_PASSES 16
struct GemmArgs {
    const void* Wp;      // packed weights [rows][K]
    int32_t rows, K;
    const uint16_t* xs;
    int32_t plane_rows;
    int32_t M;           // live rows over all passes
    int32_t n_pass;      // ceil(M / SB_PREFILL_ROWS)
    float* part;
    int32_t S;           // partial-sum slots per row block, from gemm_splits()
    // Tail done by the GEMM itself for the row blocks (256 weight rows) whose whole k range one thread
    // block owns; the epilogue, which must be given the same `fused`, then only finishes the row blocks
    // that were cut along k.  0: none.  1 + EPI_STORE: y = scale * product.  1 + EPI_SWIGLU (rows = 2 N:
    // N gate rows, then N up rows; a thread block takes matching gate and up tiles together):
    // silu(g) * u of the scaled products as bf16 planes ys [2][plane_rows][N].
    int32_t fused;
    int32_t N;           // outputs
    const float* ssq_in; // partial sums of squares of the input rows (nullable: no scale; as in GemmEpiArgs)
    int32_t ssq_nb, ssq_ld;
    float eps;
    uint16_t* ys;        // SWIGLU
    float* y;            // STORE: [M][ldy]
    int32_t ldy;
};
int gemm_splits(int32_t rows, int32_t K, int32_t n_pass);
hipError_t launch_prefill_gemm(const GemmArgs& a, hipStream_t st);

// Sums the k splits in order, applies the RMSNorm scale of the input row (from the
// partial sums of squares its producer left; nullable) and finishes the projection.
// Rows are indexed over the whole super-pass.
struct GemmEpiArgs {
    const float* part;
    int32_t S, rows;
    int32_t N, M, n_pass;  // output columns (rows, or rows / 2 for the gate/up pair), live rows, passes
    int32_t plane_rows;    // rows between the high and the low plane of nx / ys
    int32_t epi;           // EPI_STORE, EPI_RESID, EPI_SWIGLU
    const float* ssq_in;   // [M][ssq_ld] partial sums of squares of the input rows
    int32_t ssq_nb, ssq_ld, K;
    float eps;
    float* y;              // STORE: y = v; RESID: y += v        [M][ldy]
    int32_t ldy;
    const float* gain;     // RESID: nx = bf16 planes of gain * y (nullable)
    uint16_t* nx;
    float* ssq_out;        // RESID: partial sums of squares of y per 256 columns
    uint16_t* ys;          // SWIGLU: bf16 planes of silu(gate) * up
    int32_t fused;         // the GEMM ran with this `fused` (row blocks with one partial are done)
};
hipError_t launch_prefill_epilogue(const GemmEpiArgs& a, hipStream_t st);
// Embedding rows of tokens[0..M) (device ids): H [M][d], bf16 planes of gain * h, sums of squares.
hipError_t launch_prefill_embed(const void* E, int32_t w_dtype, int32_t vocab, int32_t d, const int32_t* tokens,
                                int32_t M, float* H, const float* gain, uint16_t* nx, int32_t plane_rows,
                                float* ssq_out, int32_t ssq_ld, hipStream_t st);
// x [M][K] float -> bf16 planes [2][plane_rows][K]
hipError_t launch_prefill_split(const float* x, uint16_t* xs, int32_t plane_rows, int32_t M, int32_t K, hipStream_t st);

// Device memory that belongs to the library itself (a file-scope device array, one copy per
// GPU): *out receives its address on the current device.  No allocation takes place.
#define SB_STATIC_SCRATCH_BYTES (256 + SB_MAX_W * (SB_STATIC_MAX_N / 16) * 16 + 16 * SB_STATIC_MAX_K * 2)
hipError_t static_scratch(void** out);

hipError_t launch_copy(void* dst, const void* src, size_t nbytes, hipStream_t st);
hipError_t launch_read(const void* src, size_t nbytes, float* sink, hipStream_t st);
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t st);

}  // namespace sb
