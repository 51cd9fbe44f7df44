/*
 * specbound.h -- C ABI of libspecbound: the bounded self-speculative decode step
 * (SpecBound; batch 1 as in the paper, and batches of sessions) as hand-written
 * gfx950 kernels.
 *
 * The calls follow the paper's statement of the method: a draft phase that runs
 * each new token through the shallow layers and tests an early-exit head after
 * every layer (Annealed Confidence Threshold, Sec. 3.2, Eq. 1-2), bounded by a
 * depth bound d_max and a width bound w_max (Bounded Speculation with Cached
 * States, Sec. 3.3, Appendix A), and a verify phase that sends the cached hidden
 * states of at most w_max rows through the remaining layers in one causal pass
 * and keeps the longest prefix that matches greedy decoding, so that the output
 * is exactly that of greedy autoregressive decoding.
 *
 * Conventions
 *  - Every call returns SB_OK (0) or a negative error; sb_last_error() gives the
 *    message of the calling thread's last failure.  Arguments and state are
 *    checked before anything is changed, so a call that fails with SB_EINVAL,
 *    SB_ESTATE, SB_ECAPACITY or SB_ENOMEM leaves the session as it was.  When a
 *    kernel launch or a copy fails inside sb_draft_step, sb_verify, sb_decode or
 *    sb_generate (SB_EDEVICE), the open round is abandoned: its rows and drafts are
 *    dropped, the committed tokens, their KV entries and the pending token stay as
 *    they were, and the next draft step starts a new round.
 *  - "device" pointers are HIP device memory on the model's GPU; "host" pointers
 *    are ordinary memory.  Nothing the caller passes is freed by the library.
 *  - Weights are BORROWED: the device buffers named in sb_weights must outlive
 *    the model.  The host arrays of pointers are copied at load time.  With
 *    SB_PROJ_MFMA_PACKED sb_load_model makes a tile-packed copy of every projection
 *    matrix (same size), into sb_weights.packed if the caller provides that buffer,
 *    else into memory it allocates; the row-major projections are not read again
 *    after the call.  The embedding table and the norm gains are always read from
 *    the caller's buffers.
 *  - The KV pool and the workspace are caller-owned device memory, borrowed for
 *    the session's lifetime.  sb_query_sizes() says how large they must be.
 *  - All kernels are enqueued on the stream given to sb_load_model (a
 *    hipStream_t cast to void*; NULL = the default stream).  Calls that return
 *    results to the host synchronise that stream before returning.
 *  - One session = one sequence (batch 1).  Calls on one session must not
 *    overlap; sessions of one model share its stream.  sb_new_batch groups
 *    prefilled sessions so that sb_batch_decode runs their rounds side by side.
 *
 * Typical sequence
 *    sb_query_sizes(&cfg, &sizes);                    sizes of the caller's buffers
 *    sb_load_model(&cfg, &weights, stream, &model);   once per model
 *    sb_new_session(model, kv_pool, .., workspace, .., &session);
 *    sb_prefill(session, prompt, n, &first_token);
 *    loop { loop { sb_draft_step(session, &params, &d); } while (d.status == SB_EXITED);
 *           sb_verify(session, &params, &v);  emit v.tokens[0 .. v.n_emit) }
 *    -- or sb_decode / sb_generate, which run that loop inside the library.
 */
#ifndef SPECBOUND_H
#define SPECBOUND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SB_MAX_W 8      /* largest width bound / rows per pass */
#define SB_KV_BLOCK 16  /* tokens per KV page */
#define SB_MAX_EXIT_LAYERS 64

enum { SB_OK = 0, SB_EINVAL = -1, SB_ENOMEM = -2, SB_ECAPACITY = -3, SB_ESTATE = -4, SB_EDEVICE = -5 };
enum { SB_FP32 = 0, SB_BF16 = 1 };
/* status of a draft step */
enum { SB_EXITED = 1, SB_WIDTH_BOUND = 2, SB_DEPTH_BOUND = 3 };
/* projection kernels: plain vector-ALU dot products, MFMA tiles reading the caller's
 * row-major weights, or MFMA tiles reading a tile-packed copy of the weights that
 * sb_load_model makes (bf16 weights only; results identical to SB_PROJ_MFMA) */
enum { SB_PROJ_AUTO = 0, SB_PROJ_VALU = 1, SB_PROJ_MFMA = 2, SB_PROJ_MFMA_PACKED = 3 };

/* LLaMA-style pre-norm decoder: RMSNorm, rotary embedding (half-split pairing,
 * theta_i = rope_base^(-2i/head_dim)), multi-head or grouped-query causal
 * attention with scale 1/sqrt(head_dim), SwiGLU feed-forward, untied LM head;
 * one exit head (own RMSNorm gain + own [vocab x d_model] matrix) after each of
 * layers 1..n_exit_heads (the per-layer early-exit heads of Sec. 3.1 / 4.1). */
typedef struct sb_config {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_base;
    int32_t weight_dtype;  /* SB_FP32 or SB_BF16: element type of every matrix */
    int32_t kv_dtype;      /* SB_FP32 or SB_BF16: K and V are rounded to this on cache store */
    int32_t n_exit_heads;
    int32_t max_seq;       /* capacity in tokens, a multiple of SB_KV_BLOCK, at most 65536 (32768 with an
                              fp32 cache and head_dim 128) */
    int32_t proj_kernel;   /* SB_PROJ_*; AUTO = MFMA_PACKED for bf16 weights, VALU for fp32 */
    int32_t kv_block;      /* tokens per KV page: SB_KV_BLOCK, or 0 for that default (the page size is
                              built into the attention kernels) */
    int32_t max_w;         /* largest width bound the sessions of this model accept, 1..SB_MAX_W;
                              0 = SB_MAX_W */
} sb_config;

/* Device pointers.  Matrices are row-major [out][in] in weight_dtype; norm gains
 * are float32 vectors of d_model.  w_qkv stacks the q heads, then the k heads,
 * then the v heads: [(n_heads + 2 n_kv_heads) head_dim][d_model].  w_gate_up
 * stacks the gate rows above the up rows: [2 d_ffn][d_model].  The arrays of
 * pointers are host arrays with n_layers (resp. n_exit_heads) entries. */
typedef struct sb_weights {
    const void *embed;        /* [vocab][d_model] */
    const float *final_norm;
    const void *lm_head;      /* [vocab][d_model] */
    const float *const *attn_norm;
    const void *const *w_qkv;
    const void *const *w_o;   /* [d_model][n_heads head_dim] */
    const float *const *ffn_norm;
    const void *const *w_gate_up;
    const void *const *w_down; /* [d_model][d_ffn] */
    const float *const *exit_norm;
    const void *const *exit_head; /* [vocab][d_model] each */
    /* SB_PROJ_MFMA_PACKED only.  Device buffer of packed_bytes >= sb_sizes.packed_weight_bytes,
     * 256-byte aligned, that receives the tile-packed copy of every projection matrix and is
     * borrowed for the model's lifetime (SB_ENOMEM if too small, SB_EINVAL if misaligned).
     * NULL: the library allocates that copy itself and frees it in sb_free_model.  Either way,
     * once sb_load_model has returned the row-major projection matrices (w_qkv, w_o, w_gate_up,
     * w_down, exit_head, lm_head) are no longer read and may be released by the caller; embed
     * and the norm gains stay borrowed. */
    void *packed;
    size_t packed_bytes;
} sb_weights;

/* Speculation parameters (Sec. 3.2-3.3; evaluation values in Sec. 4.1).  All
 * pointers are host memory, read during the call only.
 *  d_max      depth bound, 0..min(n_exit_heads, n_layers-1).  0 disables
 *             drafting: every round is one row through all layers, i.e. plain
 *             greedy decoding (the library's own baseline).
 *  w_max      width bound, 1..SB_MAX_W: number of exited drafts that ends a round.
 *  T          T[l-1] > 0 is the temperature of layer l = 1..d_max (Eq. 1 gives
 *             one such schedule; any array is accepted).
 *  threshold  exit when max softmax(z/T_l) >= threshold (Eq. 2); > 1 never exits.
 *  forced_exit / forced_draft  optional per-draft-step overrides, indexed by the
 *             session's draft-step counter, n_forced entries each: forced_exit[k]
 *             in 1..d_max makes step k exit exactly there, 0 makes it never exit;
 *             forced_draft[k] >= 0 replaces the drafted token id, -1 keeps the
 *             head's arg max.  Exit heads of all layers up to the exit layer are
 *             still evaluated.  Steps past n_forced use the computed test.
 *  head_mask  0: an exit head is evaluated after every layer 1..d_max, the
 *             paper's rule (Sec. 3.2).  Otherwise bit l-1 set means layer l has
 *             its head evaluated; the other layers are passed without a test, so
 *             a token can only exit at a layer of the mask (a cheaper variant, not
 *             the paper's rule; forced_exit must then name layers of the mask; 32 bits, so a
 *             nonzero mask needs d_max <= 32, else SB_EINVAL). */
typedef struct sb_params {
    int32_t d_max, w_max;
    const float *T;
    float threshold;
    int32_t eos_id; /* -1: none */
    const int32_t *forced_exit;
    const int32_t *forced_draft;
    int64_t n_forced;
    uint32_t head_mask;
    /* Sampling-mode verification (Sec. 4.3, sampling strategies).  sample_temperature == 0:
     * greedy verification (the fields below are ignored).  sample_temperature > 0: every emitted
     * token is a sample of softmax(z / sample_temperature) of the full model, restricted to its
     * nucleus of mass top_p in (0, 1] (1: no restriction) -- the draft x of a row (the exit
     * head's arg max, as in greedy mode) is accepted with probability P(x), at the first
     * rejection the token is drawn from P without x, and after the last accepted draft of a
     * depth-bound round from P.  sample_u: host array of n_sample_u uniforms in [0, 1); the row
     * at position pos uses sample_u[2 pos] for its acceptance test and sample_u[2 pos + 1] for
     * its draw (SB_EINVAL if the array is too short for the rows of a round).  The first token
     * of sb_prefill stays the greedy one; a caller who wants it sampled passes its own choice
     * to sb_rewind. */
    float sample_temperature;
    float top_p;
    const float *sample_u;
    int64_t n_sample_u;
    /* 0: under a forced schedule the host knows every exit in advance, enqueues a round without
     * waiting and lets the exit heads run beside the following layers.  1: the host takes every exit
     * decision from the device's flag after each head, as it has to when exits are computed -- the
     * same decisions, tokens and counters, with the control flow (and cost) of computed exits.  Steps
     * without a forced entry always work this way.  sb_batch_decode ignores the field. */
    int32_t exit_readback;
} sb_params;

typedef struct sb_draft_result {
    int32_t token;      /* drafted token id, -1 if the step hit the depth bound */
    int32_t exit_layer; /* 1..d_max, 0 if none */
    int32_t status;     /* SB_EXITED, SB_WIDTH_BOUND or SB_DEPTH_BOUND */
    float confidence;   /* Eq. 2 at the last evaluated layer */
} sb_draft_result;

typedef struct sb_verify_result {
    int32_t n_rows;      /* M: rows verified */
    int32_t n_drafts;    /* drafts checked */
    int32_t n_matched;   /* m: leading drafts equal to the greedy tokens */
    int32_t n_emit;      /* min(m + 1, M) tokens emitted, >= 1 */
    int32_t align_layer; /* D: deepest layer reached while drafting */
    int32_t tokens[SB_MAX_W]; /* greedy token after each row; the first n_emit are emitted.  Sampling
                                 mode: the emitted tokens, -1 for the rows after them */
    float accept_prob[SB_MAX_W]; /* sampling mode: P(draft) of each row that was examined, else 0 */
} sb_verify_result;

typedef struct sb_stats {
    int64_t rounds, draft_steps, drafts, emitted;
    int64_t layer_sweeps; /* layer passes: one sweep over a layer's weights each */
    int64_t row_layers;   /* sum of rows over layer passes */
    int64_t head_evals;   /* exit-head evaluations */
    int64_t final_head_sweeps;
    int64_t accept_hist[SB_MAX_W + 1];
    int64_t exit_hist[SB_MAX_EXIT_LAYERS + 1]; /* [0] = depth bound */
    int64_t weight_bytes; /* algorithmic bytes of weights swept (layers + heads) */
    int64_t kv_bytes;     /* algorithmic bytes of K/V read by attention */
    double prefill_ms, decode_ms; /* wall time of the last sb_generate */
    /* Time account of the decode phase, summed over its rounds, in ms.
     * host_*: wall time of the calling thread -- enqueueing the draft steps, enqueueing
     * alignment + verification, and blocked until the round record has come back.  When
     * host_wait_ms is near zero the host, not the GPU, paces the rounds.
     * gpu_*: time on the model's stream between HIP events at the phase boundaries (first
     * draft kernel .. last exit head joined | alignment | remaining layers + final head |
     * copy of the round record); filled only while sb_phase_timing is on. */
    double host_draft_ms, host_verify_ms, host_wait_ms;
    double gpu_draft_ms, gpu_align_ms, gpu_verify_ms, gpu_readback_ms;
    /* algorithmic bytes (weights swept + K/V read) of the decode phase by phase: drafting
     * (layers and exit heads), alignment, verification (remaining layers + final head) */
    int64_t draft_bytes, align_bytes, verify_bytes;
} sb_stats;

typedef struct sb_sizes {
    size_t kv_pool_bytes, workspace_bytes;
    size_t packed_weight_bytes; /* tile-packed copy of the projections (0 unless SB_PROJ_MFMA_PACKED) */
} sb_sizes;

typedef struct sb_model sb_model;
typedef struct sb_session sb_session;

const char *sb_last_error(void);

/* Eq. 1: T[l-1] = 1 + alpha (1 - l / L) for l = 1..n.  Host arithmetic. */
int32_t sb_temperature_schedule(double alpha, int32_t L, int32_t n, float *T /*host, n floats*/);

/* Bytes of device memory a session of this configuration needs. */
int32_t sb_query_sizes(const sb_config *cfg, sb_sizes *out);

/* Validates cfg and weights (SB_EINVAL), builds the rotary table on the device
 * (SB_EDEVICE / SB_ENOMEM on failure).  stream: hipStream_t or NULL. */
int32_t sb_load_model(const sb_config *cfg, const sb_weights *w, void *stream, sb_model **out);
void sb_free_model(sb_model *m);

/* kv_pool, workspace: device memory of at least sb_query_sizes() bytes, 256-byte
 * aligned (SB_ENOMEM if too small, SB_EINVAL if NULL / misaligned).  page_order:
 * optional host array with a permutation of 0..max_seq/SB_KV_BLOCK-1, the
 * physical page used for each logical KV page (NULL = identity). */
int32_t sb_new_session(sb_model *m, void *kv_pool, size_t kv_pool_bytes, void *workspace,
                       size_t workspace_bytes, const int32_t *page_order, sb_session **out);
void sb_free_session(sb_session *s);

/* Prefill (identical to the base model, Sec. 4.3): all n prompt tokens (host
 * ids in [0, vocab)) through all layers; *first_token is the greedy token after
 * the prompt.  Resets the session.  SB_ECAPACITY if n > max_seq. */
int32_t sb_prefill(sb_session *s, const int32_t *prompt, int32_t n, int32_t *first_token);

/* One draft step (Sec. 3.3): the next token (the last emitted token, or the
 * previous draft) goes through layers 1..d_max; after each layer its exit head is
 * evaluated (RMSNorm, full-vocabulary projection, softmax at temperature T_l, Eq. 2)
 * and the token exits at the first layer whose confidence reaches the threshold.
 * Earlier rows of the round whose hidden state stands one layer below are taken
 * through the same layer in the same weight sweep (cache "Reuse").  SB_ESTATE if
 * there is no pending token or a bound was already hit this round; SB_ECAPACITY
 * if the KV capacity would be exceeded. */
int32_t sb_draft_step(sb_session *s, const sb_params *p, sb_draft_result *out);

/* Verification: align every cached row to the deepest layer reached, run all
 * rows through the remaining layers in one causal pass over the paged KV cache,
 * compare the drafts with the full model's greedy tokens, emit min(m+1, M)
 * tokens, commit their KV entries and drop the rest.  SB_ESTATE with no open row. */
int32_t sb_verify(sb_session *s, const sb_params *p, sb_verify_result *out);

/* Prefill + rounds of draft steps and verification until max_new tokens are out
 * (or eos_id was emitted).  out_tokens: host, out_cap >= max_new.  The first
 * output token is the one the prefill yields.  SB_ECAPACITY if
 * n + max_new + w_max > max_seq.  stats may be NULL. */
int32_t sb_generate(sb_session *s, const int32_t *prompt, int32_t n, int32_t max_new,
                    const sb_params *p, int32_t *out_tokens, int32_t out_cap, int32_t *n_out,
                    sb_stats *stats);

/* Continue from the current state (after sb_prefill, sb_verify or sb_rewind):
 * rounds of draft steps and verification until max_new further tokens are out or
 * eos_id was emitted.  SB_ESTATE without a pending token or with open rows;
 * SB_ECAPACITY if committed + max_new + w_max > max_seq.  Fills decode_ms. */
int32_t sb_decode(sb_session *s, int32_t max_new, const sb_params *p, int32_t *out_tokens, int32_t out_cap,
                  int32_t *n_out, sb_stats *stats);

/* Drop every cached position >= n_keep (0 < n_keep <= committed length) and any
 * open rows, make `pending_token` the next token to feed, set the draft-step
 * counter (index into forced_exit / forced_draft) and clear the statistics.
 * Lets a caller decode again from the end of a prefill. */
int32_t sb_rewind(sb_session *s, int32_t n_keep, int32_t pending_token, int64_t draft_counter);

/* on != 0: every round records five events on the model's stream (phase boundaries) and adds
 * the times between them to the gpu_*_ms fields of the statistics.  SB_ENOMEM if the events
 * cannot be created. */
int32_t sb_phase_timing(sb_session *s, int32_t on);

/* ---- batch > 1: several sequences decoded together ------------------------ */
/* The rounds of B sequences run side by side (the paper evaluates batch 1, Sec. 4.3; this is
 * the same method with the rows of several sequences in every pass): each draft super-step
 * adds a row to every sequence that is still drafting, a layer pass takes the rows of all
 * sequences that need that layer in ONE sweep over its weights, each sequence attends to its
 * own KV cache, exits, bounds and acceptance are decided per sequence.  Every sequence's
 * output is bit-identical to what sb_decode gives for it alone.
 * sessions: B in 2..SB_MAX_W sessions of one model (MFMA projection path), each with its own
 * KV pool and workspace, each after sb_prefill / sb_rewind.  The sessions stay usable on their
 * own between calls; the batch borrows them.  A sequence has SB_MAX_W / B rows per round, so
 * params[b]->w_max must not exceed that (SB_EINVAL).  The shared layer sweeps are counted in
 * the statistics of sessions[0]; per-sequence counters (rounds, drafts, emitted, histograms)
 * in each session's own. */
typedef struct sb_batch sb_batch;
int32_t sb_new_batch(sb_session *const *sessions, int32_t B, sb_batch **out);
void sb_free_batch(sb_batch *b);
/* Rounds until every sequence has max_new further tokens (or emitted its eos_id).
 * params: B pointers (a sequence's forced arrays are indexed by its own draft-step counter);
 * out_tokens: B host arrays of max_new ids; n_out: B counts.  Errors as sb_decode; on
 * SB_EDEVICE the open rounds of all sequences are abandoned. */
int32_t sb_batch_decode(sb_batch *b, int32_t max_new, const sb_params *const *params, int32_t *const *out_tokens,
                        int32_t *n_out);

int32_t sb_get_stats(const sb_session *s, sb_stats *out);
int32_t sb_committed_len(const sb_session *s);

/* ---- parity taps (not for timed runs) ---------------------------------- */
/* With debug on, head kernels also store their logits. */
int32_t sb_debug_enable(sb_session *s, int32_t on);
/* layer >= 1: logits of the last evaluation of that layer's exit head (row is
 * ignored); layer == 0: final-head logits of verified row `row` (or of the
 * prefill's last position, row 0).  out: host, cap >= vocab floats. */
int32_t sb_debug_logits(sb_session *s, int32_t layer, int32_t row, float *out, int32_t cap);
/* Hidden state (d_model floats, host) of open row `slot`. */
int32_t sb_debug_hidden(sb_session *s, int32_t slot, float *out, int32_t cap);
/* K and V (as floats, n_kv_heads*head_dim each, host) cached for (layer, pos). */
int32_t sb_debug_kv(sb_session *s, int32_t layer, int32_t pos, float *k_out, float *v_out, int32_t cap);

/* Test tap: the n-th projection launch from now on (n >= 1) is not enqueued and reports a
 * device error instead, as a failed launch would; 0 disarms.  Lets a host test walk the
 * SB_EDEVICE path of sb_draft_step / sb_verify without a fault on the GPU. */
int32_t sb_debug_fail_launch(sb_session *s, int32_t n);
/* Open rows of the current round (0 between rounds). */
int32_t sb_open_rows(const sb_session *s);

/* ---- per-kernel timing with HIP events on the model's stream -------------- */
enum { SB_K_RMSNORM = 0, SB_K_QKV, SB_K_ATTN, SB_K_WO, SB_K_GATEUP, SB_K_DOWN, SB_K_EXIT_HEAD,
       SB_K_FINAL_HEAD, SB_K_COUNT };
/* From now on every sample_every-th launch of a kernel class whose bit
 * (1 << SB_K_*) is set in class_mask is bracketed by a pair of events, up to
 * max_launches pairs in all (further launches run untimed).  An event pair costs
 * several microseconds of idle GPU time, so sample sparsely inside timed runs.
 * SB_ENOMEM if the events cannot be created. */
int32_t sb_profile_begin(sb_session *s, uint32_t class_mask, int32_t max_launches, int32_t sample_every);
/* Synchronises, then per class: timed launches, their summed duration in ms and
 * their summed algorithmic bytes (weights + activations in/out for projections,
 * K/V read for attention).  Arrays of SB_K_COUNT, host.  empty_pair_ms (nullable)
 * receives the average time between the two events of a pair with no kernel in
 * between, measured when the timing began: what a bracket adds to a kernel's own
 * duration.  Ends the timing. */
int32_t sb_profile_end(sb_session *s, int64_t *launches, double *total_ms, int64_t *bytes, double *empty_pair_ms);

/* ---- single kernels, for parity tests and roofline measurement ---------- */
/* All pointers are device memory; stream as above; calls do not synchronise.
 * M rows, 1 <= M <= SB_MAX_W. */

/* out[m][i] = x[m][i] / sqrt(mean_i x[m][i]^2 + eps) * gain[i]; x, out: [M][d] float. */
int32_t sb_op_rmsnorm(const float *x, const float *gain, float *out, int32_t M, int32_t d, float eps,
                      void *stream);
/* y[m][n] = sum_k W[n][k] x[m][k]; W [N][K] in w_dtype, x [M][K], y [M][N] float.
 * kernel: SB_PROJ_VALU, SB_PROJ_MFMA or SB_PROJ_MFMA_PACKED (bf16 only; K % 128 == 0,
 * N % 16 == 0; PACKED: W is the output of sb_op_repack).
 * scratch: device, sb_op_gemv_scratch_bytes(M, K) bytes (MFMA operand staging). */
int32_t sb_op_gemv(const void *W, int32_t w_dtype, int32_t N, int32_t K, const float *x, float *y,
                   int32_t M, int32_t kernel, void *scratch, void *stream);
size_t sb_op_gemv_scratch_bytes(int32_t M, int32_t K);
/* The FFN's first half as the decode path runs it (step S7: one sweep over the gate and up
 * matrices with the SwiGLU in the epilogue; the decoder's definition, Sec. 4.1 model families):
 * u[m][n] = silu(W[n] . x[m]) * (W[N + n] . x[m]), W [2N][K] = gate rows, then up rows (for
 * SB_PROJ_MFMA_PACKED: sb_op_repack of that matrix, N % 16 == 0).  x [M][K], u [M][N] float,
 * device; scratch as for sb_op_gemv.  Errors as sb_op_gemv. */
int32_t sb_op_gate_up(const void *W, int32_t w_dtype, int32_t N, int32_t K, const float *x, float *u,
                      int32_t M, int32_t kernel, void *scratch, void *stream);
/* Tile-packed copy of a bf16 matrix W [N][K] (N % 16 == 0, K % 128 == 0) for
 * kernel = SB_PROJ_MFMA_PACKED of sb_op_gemv / sb_op_head: packed, N*K*2 bytes. */
int32_t sb_op_repack(const void *W, int32_t N, int32_t K, void *packed, void *stream);
/* Exit-head evaluation on already normalised rows x [M][K]: z = W x (never
 * written unless logits != NULL, [M][N] float), arg max (lowest index on ties) and
 * confidence p = 1 / sum_j exp((z_j - z_max)/T) (Eq. 2).  argmax_out [M] int32,
 * conf_out [M] float.  scratch: sb_op_head_scratch_bytes(M, N, K) bytes. */
int32_t sb_op_head(const void *W, int32_t w_dtype, int32_t N, int32_t K, const float *x, int32_t M,
                   float T, int32_t kernel, int32_t *argmax_out, float *conf_out, float *logits,
                   void *scratch, void *stream);
size_t sb_op_head_scratch_bytes(int32_t M, int32_t N, int32_t K);

/* sb_op_head for callers that cannot allocate device memory or carry a workspace (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels
 * and the same results as sb_op_head with logits == NULL, with the scratch area in a static
 * device array of the library (1.3 MB, held by every GPU the library runs on until the
 * process ends) instead of a caller's buffer.  The call allocates nothing.  Limits:
 * N <= SB_STATIC_MAX_N and K <= SB_STATIC_MAX_K, else SB_ECAPACITY; otherwise arguments and
 * errors as sb_op_head.  All calls on one GPU share the array (its contents are whatever the
 * last call left; nothing in it needs clearing), so calls that overlap on one GPU -- on
 * different streams or from different threads -- race: serialise them. */
#define SB_STATIC_MAX_N 131072
#define SB_STATIC_MAX_K 8192
int32_t sb_op_head_static(const void *W, int32_t w_dtype, int32_t N, int32_t K, const float *x, int32_t M,
                          float T, int32_t kernel, int32_t *argmax_out, float *conf_out, void *stream);

/* Plain device-to-device copy kernel (128-bit loads and stores), nbytes % 16 == 0,
 * both pointers 16-byte aligned.  A bandwidth yardstick of known traffic
 * (nbytes read + nbytes written) for calibrating profiler counters. */
int32_t sb_op_copy(void *dst, const void *src, size_t nbytes, void *stream);
/* Plain streaming read of nbytes (sum-reduced into *sink, 4 bytes, device). */
int32_t sb_op_read(const void *src, size_t nbytes, float *sink, void *stream);

/* The projection of the prompt passes (prefill is the base model's, Sec. 4.3): y [M][N] =
 * x [M][K] W^T for 1 <= M <= 128 rows against tile-packed bf16 weights (sb_op_repack),
 * N % 16 == 0, K % 128 == 0.  x is used as a bf16 high + low pair per element, products
 * accumulate in fp32 over k splits that are added in index order.  x, y, Wp, scratch:
 * device; scratch of sb_op_gemm_scratch_bytes(N, K) bytes, 256-byte aligned. */
int32_t sb_op_gemm(const void *Wp, int32_t N, int32_t K, const float *x, float *y, int32_t M, void *scratch,
                   void *stream);
size_t sb_op_gemm_scratch_bytes(int32_t N, int32_t K);
/* Rotary table as the library builds it: cos/sin of pos * base^(-2i/head_dim),
 * evaluated in double and rounded to float; [n_pos][head_dim/2] each, host. */
int32_t sb_rope_table_host(int32_t head_dim, float base, int32_t n_pos, float *cos_out, float *sin_out);
/* Rotary embedding, KV append and causal attention for M new rows at positions
 * pos0..pos0+M-1.  qkv [M][(n_heads + 2 n_kv_heads) head_dim] float holds the
 * rows' raw projections (q heads, k heads, v heads).  Rotated k and v of the new
 * rows are written (rounded to kv_dtype) into the paged pool
 * [layer][2 (k, v)][n_pages][n_kv_heads][SB_KV_BLOCK][head_dim] (in a bf16 pool
 * the v slabs are held transposed, [head_dim][SB_KV_BLOCK]: the layout is the
 * library's own, read it back with sb_debug_kv); table [n_pages] maps logical
 * to physical pages; rope_cos/sin: device tables with at least pos0+M
 * rows.  Each row attends to keys 0..its own position (scale 1/sqrt(head_dim));
 * out [M][n_heads head_dim] float.  scratch: sb_op_attention_scratch_bytes(). */
int32_t sb_op_attention(const float *qkv, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, int32_t kv_dtype,
                        void *pool, const int32_t *table, int32_t n_pages, int32_t layer, const float *rope_cos,
                        const float *rope_sin, int32_t pos0, int32_t M, float *out, void *scratch, void *stream);
size_t sb_op_attention_scratch_bytes(int32_t n_heads, int32_t head_dim, int32_t kv_dtype, int32_t n_pages);

/* The same operation in the form the prompt uses (any number of rows, bf16 pool only):
 * the k and v of all M rows are appended first, then every row's causal attention is
 * computed with a running soft-max per query (no scratch).  Arguments, layouts and
 * errors as sb_op_attention; M >= 1 is limited only by the pool (pos0 + M <= 16 n_pages);
 * qkv, out and the rope tables 16-byte aligned. */
int32_t sb_op_prompt_attention(const float *qkv, int32_t n_heads, int32_t n_kv_heads, int32_t head_dim, void *pool,
                               const int32_t *table, int32_t n_pages, int32_t layer, const float *rope_cos,
                               const float *rope_sin, int32_t pos0, int32_t M, float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECBOUND_H */
