/*
 * specbound_oracle.c -- plain CPU oracle for the bounded self-speculative decode
 * step (SpecBound: Annealed Confidence Threshold, Sec. 3.2, and Bounded
 * Speculation with Cached States, Sec. 3.3 and Appendix A).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is slow on purpose: one token row at a time,
 * one dot product at a time, no blocking, no fusion.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code with
 * the HIP library and must never be used as a fallback for it.
 *
 * Arithmetic type `real` is double (default) or float (-DORC_F32).  Weights are
 * kept exactly as handed in (fp32, or bf16 bit patterns upcast on the fly);
 * K and V are rounded to bf16 when written to the cache if kv_dtype says so.
 *
 * What each function follows is cited next to it.  Readings of points the paper
 * leaves open (argmax ties, what the width bound counts, what a round emits) are
 * stated where they are taken.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifdef ORC_F32
typedef float real;
#define R_EXP expf
#define R_SQRT sqrtf
#else
typedef double real;
#define R_EXP exp
#define R_SQRT sqrt
#endif

#define ORC_MAX_W 16

enum { ORC_FP32 = 0, ORC_BF16 = 1 };
enum { ORC_OK = 0, ORC_EINVAL = -1, ORC_ENOMEM = -2, ORC_ECAPACITY = -3, ORC_ESTATE = -4 };
enum { ORC_EXITED = 1, ORC_WIDTH_BOUND = 2, ORC_DEPTH_BOUND = 3 };
enum { ORC_PH_DRAFT = 0, ORC_PH_ALIGN = 1, ORC_PH_VERIFY = 2, ORC_PH_PREFILL = 3 };

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_base;
    int32_t weight_dtype, kv_dtype, n_exit_heads, max_seq;
} orc_config;

/* Host pointers.  Matrices are row-major [out][in] in weight_dtype; norm gains are
 * float.  w_qkv stacks q heads, k heads, v heads; w_gate_up stacks gate above up. */
typedef struct {
    const void *embed, *lm_head;
    const float *final_norm;
    const float *const *attn_norm;
    const void *const *w_qkv;
    const void *const *w_o;
    const float *const *ffn_norm;
    const void *const *w_gate_up;
    const void *const *w_down;
    const float *const *exit_norm;
    const void *const *exit_head;
} orc_weights;

typedef struct {
    int32_t d_max, w_max;
    const float *T;              /* T[l-1] for layer l = 1..d_max */
    float threshold;
    int32_t eos_id;              /* -1: none */
    const int32_t *forced_exit;  /* per draft step: 1..d_max, 0 = never exit; NULL = computed */
    const int32_t *forced_draft; /* per draft step: token override, -1 = head argmax; NULL */
    int64_t n_forced;
    uint32_t head_mask;          /* 0: an exit head after every layer 1..d_max (Sec. 3.2); else bit l-1
                                    set = layer l has its head evaluated, the others are passed without a
                                    test (a variant, not the paper's rule) */
    /* Sampling-mode verification (Sec. 4.3, "sampling strategies"; the paper gives results for
     * temperature and top-p sampling but not the mechanism -- the rule taken here is stated at
     * orc_verify).  sample_temperature == 0: greedy verification. */
    float sample_temperature;    /* > 0: the output is sampled from softmax(z / sample_temperature) ... */
    float top_p;                 /* ... restricted to its nucleus of mass top_p (1: no restriction) */
    const float *sample_u;       /* uniforms in [0, 1): the row at position pos uses sample_u[2 pos] for its
                                    acceptance test and sample_u[2 pos + 1] to draw a token */
    int64_t n_sample_u;
} orc_params;

typedef struct { int32_t token, exit_layer, status; float confidence; } orc_draft_result;
typedef struct {
    int32_t n_rows, n_drafts, n_matched, n_emit, align_layer;
    int32_t tokens[ORC_MAX_W];
} orc_verify_result;
typedef struct { int32_t phase, layer, first_slot, n_rows; } orc_trace_entry;
typedef struct {
    int64_t rounds, draft_steps, drafts, emitted;
    int64_t layer_sweeps;   /* layer passes (one weight sweep each, whatever the row count) */
    int64_t row_layers;     /* sum of rows over layer passes */
    int64_t head_evals;     /* exit-head evaluations */
    int64_t final_head_rows;
    int64_t accept_hist[ORC_MAX_W + 1];
    int64_t exit_hist[65];  /* [0] = no exit (depth bound) */
} orc_stats;

typedef struct {
    orc_config cfg;
    orc_weights w;
    float *rope_cos, *rope_sin; /* [max_seq][head_dim/2], double -> float */
} orc_model;

typedef struct {
    int32_t pos, tok, reached, exit_layer;
    real *h;
} orc_slot;

typedef struct {
    orc_model *m;
    float *kc, *vc;            /* [layer][pos][n_kv_heads*head_dim] */
    int32_t c;                 /* committed length: positions < c valid at all layers */
    int32_t pending, has_pending;
    orc_slot slots[ORC_MAX_W];
    int32_t n_slots;
    int32_t drafts[ORC_MAX_W];
    int32_t n_drafts;
    int32_t round_closed;
    int64_t draft_counter;     /* index into forced_exit / forced_draft */
    int32_t eager_align;       /* test switch: align all slots after every draft step */
    orc_stats st;
    orc_trace_entry *trace;
    int64_t trace_cap, trace_n;
    real *head_logits;         /* [vocab] last exit-head logits */
    real *verify_logits;       /* [ORC_MAX_W][vocab] logits of the last verify / prefill / step */
    real *verify_dist;         /* [ORC_MAX_W][vocab] sampling distributions of the last sampled verify */
    real *sort_buf;            /* [vocab] */
    int32_t last_argmax; real last_conf;
    /* scratch */
    real *xn, *qkv, *att, *o, *gu, *u, *dn, *sc;
} orc_session;

/* ------------------------------------------------------------------ helpers */

static inline float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

/* round-to-nearest-even to 8 bits of mantissa; the value comes back as a float */
static inline float round_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return f;
}

/* y[n] = sum_k W[n][k] x[k] -- the definition of a matrix-vector product */
void orc_matvec(const void *W, int32_t dtype, int32_t N, int32_t K, const real *x, real *y) {
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        real acc = 0;
        if (dtype == ORC_BF16) {
            const uint16_t *w = (const uint16_t *)W + (size_t)n * K;
#pragma omp simd reduction(+ : acc)
            for (int32_t k = 0; k < K; ++k) acc += (real)bf16_bits_to_float(w[k]) * x[k];
        } else {
            const float *w = (const float *)W + (size_t)n * K;
#pragma omp simd reduction(+ : acc)
            for (int32_t k = 0; k < K; ++k) acc += (real)w[k] * x[k];
        }
        y[n] = acc;
    }
}

/* RMSNorm: x / sqrt(mean(x^2) + eps) * g */
void orc_rmsnorm(const real *x, const float *g, int32_t d, float eps, real *out) {
    real ss = 0;
    for (int32_t i = 0; i < d; ++i) ss += x[i] * x[i];
    real inv = (real)1 / R_SQRT(ss / (real)d + (real)eps);
    for (int32_t i = 0; i < d; ++i) out[i] = x[i] * inv * (real)g[i];
}

/* Rotary embedding, half-split pairing (i, i + hd/2), theta_i = base^(-2i/hd),
 * angle = pos * theta_i evaluated in double and rounded to float. */
/* Gated FFN activation of the LLaMA-family decoders the paper evaluates (Sec. 4.1):
 * u_i = silu(g_i) * v_i with silu(g) = g / (1 + exp(-g)); gu holds the f gate values, then
 * the f up values. */
void orc_swiglu(const real *gu, int32_t f, real *u) {
    for (int32_t i = 0; i < f; ++i) {
        real g = gu[i];
        u[i] = g / ((real)1 + R_EXP(-g)) * gu[f + i];
    }
}

void orc_rope_angles(int32_t pos, int32_t hd, float base, float *cos_out, float *sin_out) {
    for (int32_t i = 0; i < hd / 2; ++i) {
        double theta = pow((double)base, -2.0 * (double)i / (double)hd);
        double a = (double)pos * theta;
        cos_out[i] = (float)cos(a);
        sin_out[i] = (float)sin(a);
    }
}

void orc_rope_apply(real *v, int32_t hd, const float *c, const float *s) {
    int32_t half = hd / 2;
    for (int32_t i = 0; i < half; ++i) {
        real a = v[i], b = v[i + half];
        v[i] = a * (real)c[i] - b * (real)s[i];
        v[i + half] = b * (real)c[i] + a * (real)s[i];
    }
}

/* Annealed Confidence Threshold, Eq. 2: p = max softmax(z / T).  With i* the
 * arg max (lowest index on ties), p = 1 / sum_j exp((z_j - z_i*) / T). */
void orc_act(const real *z, int32_t V, real T, int32_t *argmax, real *conf) {
    int32_t im = 0;
    for (int32_t j = 1; j < V; ++j)
        if (z[j] > z[im]) im = j;
    real s = 0;
    for (int32_t j = 0; j < V; ++j) s += R_EXP((z[j] - z[im]) / T);
    *argmax = im;
    *conf = (real)1 / s;
}

/* Eq. 1: T_l = 1 + alpha (1 - l / L), l = 1..n */
void orc_temperature_schedule(double alpha, int32_t L, int32_t n, float *T) {
    for (int32_t l = 1; l <= n; ++l) T[l - 1] = (float)(1.0 + alpha * (1.0 - (double)l / (double)L));
}

/* Eq. 3-5: round time in units of T_AR, expected accepted tokens, speedup. */
double orc_round_time(int32_t L, int32_t d_max, int32_t w) {
    return ((double)w * d_max + L - d_max) / (double)L;
}
double orc_expected_accept(double a, int32_t w) {
    double s = 0;
    for (int32_t k = 0; k < w; ++k) s += k * pow(a, k) * (1.0 - a);
    return s + w * pow(a, w);
}
double orc_speedup(int32_t L, int32_t d_max, int32_t w, double a) {
    return orc_expected_accept(a, w) / orc_round_time(L, d_max, w);
}

/* ------------------------------------------------------------------ model */

static int check_config(const orc_config *c) {
    if (!c) return ORC_EINVAL;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1) return ORC_EINVAL;
    if (c->n_heads % c->n_kv_heads) return ORC_EINVAL;
    if (c->head_dim < 2 || (c->head_dim & 1)) return ORC_EINVAL;
    if (c->d_ffn < 1 || c->vocab < 1 || c->max_seq < 1) return ORC_EINVAL;
    if (c->n_exit_heads < 0 || c->n_exit_heads > c->n_layers) return ORC_EINVAL;
    if (c->weight_dtype != ORC_FP32 && c->weight_dtype != ORC_BF16) return ORC_EINVAL;
    if (c->kv_dtype != ORC_FP32 && c->kv_dtype != ORC_BF16) return ORC_EINVAL;
    return ORC_OK;
}

int32_t orc_model_new(const orc_config *cfg, const orc_weights *w, orc_model **out) {
    if (!w || !out || check_config(cfg) != ORC_OK) return ORC_EINVAL;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    if (!m) return ORC_ENOMEM;
    m->cfg = *cfg;
    m->w = *w;
    int32_t half = cfg->head_dim / 2;
    m->rope_cos = (float *)malloc(sizeof(float) * (size_t)cfg->max_seq * half);
    m->rope_sin = (float *)malloc(sizeof(float) * (size_t)cfg->max_seq * half);
    if (!m->rope_cos || !m->rope_sin) return ORC_ENOMEM;
    for (int32_t p = 0; p < cfg->max_seq; ++p)
        orc_rope_angles(p, cfg->head_dim, cfg->rope_base, m->rope_cos + (size_t)p * half,
                        m->rope_sin + (size_t)p * half);
    *out = m;
    return ORC_OK;
}

void orc_model_free(orc_model *m) {
    if (!m) return;
    free(m->rope_cos);
    free(m->rope_sin);
    free(m);
}

int32_t orc_session_new(orc_model *m, orc_session **out) {
    if (!m || !out) return ORC_EINVAL;
    const orc_config *c = &m->cfg;
    orc_session *s = (orc_session *)calloc(1, sizeof(orc_session));
    if (!s) return ORC_ENOMEM;
    s->m = m;
    size_t kvw = (size_t)c->n_kv_heads * c->head_dim;
    size_t kvn = (size_t)c->n_layers * c->max_seq * kvw;
    s->kc = (float *)calloc(kvn, sizeof(float));
    s->vc = (float *)calloc(kvn, sizeof(float));
    int32_t qkv_rows = (c->n_heads + 2 * c->n_kv_heads) * c->head_dim;
    for (int i = 0; i < ORC_MAX_W; ++i) s->slots[i].h = (real *)calloc(c->d_model, sizeof(real));
    s->head_logits = (real *)calloc(c->vocab, sizeof(real));
    s->verify_logits = (real *)calloc((size_t)ORC_MAX_W * c->vocab, sizeof(real));
    s->verify_dist = (real *)calloc((size_t)ORC_MAX_W * c->vocab, sizeof(real));
    s->sort_buf = (real *)calloc(c->vocab, sizeof(real));
    s->xn = (real *)calloc(c->d_model, sizeof(real));
    s->qkv = (real *)calloc(qkv_rows, sizeof(real));
    s->att = (real *)calloc((size_t)c->n_heads * c->head_dim, sizeof(real));
    s->o = (real *)calloc(c->d_model, sizeof(real));
    s->gu = (real *)calloc((size_t)2 * c->d_ffn, sizeof(real));
    s->u = (real *)calloc(c->d_ffn, sizeof(real));
    s->dn = (real *)calloc(c->d_model, sizeof(real));
    s->sc = (real *)calloc(c->max_seq, sizeof(real));
    if (!s->kc || !s->vc || !s->head_logits || !s->verify_logits || !s->sc) return ORC_ENOMEM;
    *out = s;
    return ORC_OK;
}

void orc_session_free(orc_session *s) {
    if (!s) return;
    free(s->kc); free(s->vc);
    for (int i = 0; i < ORC_MAX_W; ++i) free(s->slots[i].h);
    free(s->head_logits); free(s->verify_logits); free(s->verify_dist); free(s->sort_buf);
    free(s->xn); free(s->qkv); free(s->att); free(s->o); free(s->gu); free(s->u); free(s->dn); free(s->sc);
    free(s->trace);
    free(s);
}

void orc_session_reset(orc_session *s) {
    s->c = 0; s->has_pending = 0; s->n_slots = 0; s->n_drafts = 0; s->round_closed = 0;
    s->draft_counter = 0; s->trace_n = 0;
    memset(&s->st, 0, sizeof(s->st));
}

void orc_set_eager_align(orc_session *s, int32_t on) { s->eager_align = on; }

int32_t orc_trace_enable(orc_session *s, int64_t cap) {
    free(s->trace);
    s->trace = (orc_trace_entry *)calloc((size_t)cap, sizeof(orc_trace_entry));
    s->trace_cap = s->trace ? cap : 0;
    s->trace_n = 0;
    return s->trace ? ORC_OK : ORC_ENOMEM;
}
int64_t orc_trace_read(const orc_session *s, orc_trace_entry *out, int64_t cap) {
    int64_t n = s->trace_n < cap ? s->trace_n : cap;
    memcpy(out, s->trace, (size_t)n * sizeof(orc_trace_entry));
    return s->trace_n;
}
void orc_get_stats(const orc_session *s, orc_stats *out) { *out = s->st; }
/* Drop every cached position >= n_keep and any open rows; `pending` is the next token to feed. */
int32_t orc_rewind(orc_session *s, int32_t n_keep, int32_t pending) {
    if (n_keep < 1 || n_keep > s->c || pending < 0 || pending >= s->m->cfg.vocab) return ORC_EINVAL;
    s->c = n_keep; s->pending = pending; s->has_pending = 1;
    s->n_slots = 0; s->n_drafts = 0; s->round_closed = 0; s->draft_counter = 0;
    return ORC_OK;
}
int32_t orc_committed_len(const orc_session *s) { return s->c; }
int32_t orc_open_slots(const orc_session *s) { return s->n_slots; }
int32_t orc_slot_reached(const orc_session *s, int32_t i) { return s->slots[i].reached; }
void orc_slot_hidden(const orc_session *s, int32_t i, double *out) {
    for (int32_t k = 0; k < s->m->cfg.d_model; ++k) out[k] = (double)s->slots[i].h[k];
}
void orc_head_logits(const orc_session *s, double *out) {
    for (int32_t k = 0; k < s->m->cfg.vocab; ++k) out[k] = (double)s->head_logits[k];
}
void orc_verify_dist(const orc_session *s, int32_t row, double *out) {
    if (row < 0 || row >= ORC_MAX_W) return;
    for (int32_t j = 0; j < s->m->cfg.vocab; ++j) out[j] = (double)s->verify_dist[(size_t)row * s->m->cfg.vocab + j];
}
void orc_verify_logits(const orc_session *s, int32_t row, double *out) {
    const real *z = s->verify_logits + (size_t)row * s->m->cfg.vocab;
    for (int32_t k = 0; k < s->m->cfg.vocab; ++k) out[k] = (double)z[k];
}
void orc_kv_read(const orc_session *s, int32_t layer, int32_t pos, float *k_out, float *v_out) {
    const orc_config *c = &s->m->cfg;
    size_t kvw = (size_t)c->n_kv_heads * c->head_dim;
    size_t off = ((size_t)layer * c->max_seq + pos) * kvw;
    memcpy(k_out, s->kc + off, kvw * sizeof(float));
    memcpy(v_out, s->vc + off, kvw * sizeof(float));
}

static void trace_add(orc_session *s, int phase, int layer, int first, int rows) {
    s->st.layer_sweeps += 1;
    s->st.row_layers += rows;
    if (s->trace && s->trace_n < s->trace_cap) {
        orc_trace_entry e = {phase, layer, first, rows};
        s->trace[s->trace_n] = e;
    }
    if (s->trace) s->trace_n++;
}

static void embed_row(const orc_model *m, int32_t tok, real *h) {
    int32_t d = m->cfg.d_model;
    if (m->cfg.weight_dtype == ORC_BF16) {
        const uint16_t *e = (const uint16_t *)m->w.embed + (size_t)tok * d;
        for (int32_t i = 0; i < d; ++i) h[i] = (real)bf16_bits_to_float(e[i]);
    } else {
        const float *e = (const float *)m->w.embed + (size_t)tok * d;
        for (int32_t i = 0; i < d; ++i) h[i] = (real)e[i];
    }
}

/* softmax(q K^T / sqrt(hd)) V for one query head over keys 0..n_keys-1.
 * K, V rows are `stride` floats apart. */
void orc_attention_head(const real *q, const float *K, const float *Vv, int32_t n_keys,
                        int32_t hd, size_t stride, real *sc, real *out) {
    real scale = (real)1 / R_SQRT((real)hd);
    real mx = 0;
    for (int32_t t = 0; t < n_keys; ++t) {
        const float *k = K + (size_t)t * stride;
        real a = 0;
        for (int32_t i = 0; i < hd; ++i) a += q[i] * (real)k[i];
        sc[t] = a * scale;
        if (t == 0 || sc[t] > mx) mx = sc[t];
    }
    real den = 0;
    for (int32_t t = 0; t < n_keys; ++t) { sc[t] = R_EXP(sc[t] - mx); den += sc[t]; }
    for (int32_t i = 0; i < hd; ++i) out[i] = 0;
    for (int32_t t = 0; t < n_keys; ++t) {
        const float *v = Vv + (size_t)t * stride;
        real p = sc[t] / den;
        for (int32_t i = 0; i < hd; ++i) out[i] += p * (real)v[i];
    }
}

/* One pre-norm LLaMA block applied to one row at position pos, using (and
 * extending) the KV cache of layer l (0-based):
 *   a  = h + W_o Attn(RoPE(W_q n1), RoPE(W_k n1), W_v n1),  n1 = RMSNorm(h)
 *   h' = a + W_d (silu(W_g n2) * W_u n2),                   n2 = RMSNorm(a)   */
static void layer_row(orc_session *s, int32_t l, int32_t pos, real *h) {
    const orc_model *m = s->m;
    const orc_config *c = &m->cfg;
    int32_t d = c->d_model, hd = c->head_dim, Hq = c->n_heads, Hkv = c->n_kv_heads, f = c->d_ffn;
    int32_t half = hd / 2, group = Hq / Hkv;
    size_t kvw = (size_t)Hkv * hd;
    const float *cs = m->rope_cos + (size_t)pos * half, *sn = m->rope_sin + (size_t)pos * half;

    orc_rmsnorm(h, m->w.attn_norm[l], d, c->rms_eps, s->xn);
    orc_matvec(m->w.w_qkv[l], c->weight_dtype, (Hq + 2 * Hkv) * hd, d, s->xn, s->qkv);
    real *q = s->qkv, *k = s->qkv + (size_t)Hq * hd, *v = k + kvw;
    for (int32_t i = 0; i < Hq; ++i) orc_rope_apply(q + (size_t)i * hd, hd, cs, sn);
    for (int32_t i = 0; i < Hkv; ++i) orc_rope_apply(k + (size_t)i * hd, hd, cs, sn);
    float *kc = s->kc + ((size_t)l * c->max_seq + pos) * kvw;
    float *vc = s->vc + ((size_t)l * c->max_seq + pos) * kvw;
    for (size_t i = 0; i < kvw; ++i) {
        float kf = (float)k[i], vf = (float)v[i];
        kc[i] = c->kv_dtype == ORC_BF16 ? round_bf16(kf) : kf;
        vc[i] = c->kv_dtype == ORC_BF16 ? round_bf16(vf) : vf;
    }
    const float *K0 = s->kc + (size_t)l * c->max_seq * kvw, *V0 = s->vc + (size_t)l * c->max_seq * kvw;
    for (int32_t i = 0; i < Hq; ++i) {
        int32_t g = i / group;
        orc_attention_head(q + (size_t)i * hd, K0 + (size_t)g * hd, V0 + (size_t)g * hd, pos + 1, hd,
                           kvw, s->sc, s->att + (size_t)i * hd);
    }
    orc_matvec(m->w.w_o[l], c->weight_dtype, d, Hq * hd, s->att, s->o);
    for (int32_t i = 0; i < d; ++i) h[i] += s->o[i];

    orc_rmsnorm(h, m->w.ffn_norm[l], d, c->rms_eps, s->xn);
    orc_matvec(m->w.w_gate_up[l], c->weight_dtype, 2 * f, d, s->xn, s->gu);
    orc_swiglu(s->gu, f, s->u);
    orc_matvec(m->w.w_down[l], c->weight_dtype, d, f, s->u, s->dn);
    for (int32_t i = 0; i < d; ++i) h[i] += s->dn[i];
}

/* Run layer l (1-based) on every open slot whose hidden state stands at layer
 * l-1, in position order ("Reuse": earlier tokens' missing KV is filled when a
 * later token goes deeper, Sec. 3.3 Hidden-State Cache Management). */
static int32_t advance_rows(orc_session *s, int32_t l, int phase) {
    int32_t first = -1, rows = 0;
    for (int32_t j = 0; j < s->n_slots; ++j) {
        if (s->slots[j].reached == l - 1) {
            if (first < 0) first = j;
            layer_row(s, l - 1, s->slots[j].pos, s->slots[j].h);
            s->slots[j].reached = l;
            rows++;
        }
    }
    if (rows) trace_add(s, phase, l, first, rows);
    return rows;
}

/* greedy token of the full model for hidden state h (lowest index on ties) */
static int32_t final_head(orc_session *s, const real *h, real *logits) {
    const orc_model *m = s->m;
    orc_rmsnorm(h, m->w.final_norm, m->cfg.d_model, m->cfg.rms_eps, s->xn);
    orc_matvec(m->w.lm_head, m->cfg.weight_dtype, m->cfg.vocab, m->cfg.d_model, s->xn, logits);
    int32_t im = 0;
    for (int32_t j = 1; j < m->cfg.vocab; ++j)
        if (logits[j] > logits[im]) im = j;
    s->st.final_head_rows++;
    return im;
}

/* Distribution a token is sampled from (Sec. 4.3, sampling strategies: temperature, top-p):
 * p_j proportional to exp(z_j / temp); with top_p < 1 only the nucleus keeps its mass -- the
 * tokens of the shortest prefix, in order of decreasing probability, whose mass reaches top_p,
 * together with every token as probable as the last of them (ties are not split) -- and is
 * renormalised.  `tmp` is scratch of V reals. */
void orc_sample_dist(const real *z, int32_t V, real temp, real top_p, real *p, real *tmp) {
    real zmax = z[0];
    for (int32_t j = 1; j < V; ++j)
        if (z[j] > zmax) zmax = z[j];
    real sum = 0;
    for (int32_t j = 0; j < V; ++j) { p[j] = R_EXP((z[j] - zmax) / temp); sum += p[j]; }
    for (int32_t j = 0; j < V; ++j) p[j] /= sum;
    if (!(top_p < (real)1)) return;
    /* selection sort of the largest values until their mass reaches top_p: plain and quadratic
     * in the nucleus size, which is small whenever a nucleus is worth taking */
    memcpy(tmp, p, sizeof(real) * V);
    real mass = 0, cut = 0;
    for (int32_t k = 0; k < V; ++k) {
        int32_t im = 0;
        for (int32_t j = 1; j < V; ++j)
            if (tmp[j] > tmp[im]) im = j;
        cut = tmp[im];
        mass += cut;
        tmp[im] = -1;
        if (mass >= top_p) break;
    }
    real keep = 0;
    for (int32_t j = 0; j < V; ++j) { if (p[j] < cut) p[j] = 0; keep += p[j]; }
    for (int32_t j = 0; j < V; ++j) p[j] /= keep;
}

/* Inverse-CDF draw with the uniform u in [0, 1) from p, tokens in index order, leaving out
 * token `exclude` (-1: none) and renormalising the rest: the first j with
 * sum_{k <= j, k != exclude} p_k > u * sum_{k != exclude} p_k. */
int32_t orc_sample_token(const real *p, int32_t V, real u, int32_t exclude) {
    real total = 0;
    for (int32_t j = 0; j < V; ++j)
        if (j != exclude) total += p[j];
    real target = u * total, c = 0;
    int32_t last = -1;
    for (int32_t j = 0; j < V; ++j) {
        if (j == exclude || !(p[j] > 0)) continue;
        c += p[j];
        last = j;
        if (c > target) return j;
    }
    return last;   /* rounding at the upper end: the last token that has mass */
}

static int check_params(const orc_session *s, const orc_params *p) {
    const orc_config *c = &s->m->cfg;
    if (!p) return ORC_EINVAL;
    if (p->w_max < 1 || p->w_max > ORC_MAX_W) return ORC_EINVAL;
    if (p->d_max < 0 || p->d_max > c->n_exit_heads || p->d_max > c->n_layers - 1) return ORC_EINVAL;
    if (p->d_max > 0 && !p->T) return ORC_EINVAL;
    for (int32_t l = 0; l < p->d_max; ++l)
        if (!(p->T[l] > 0)) return ORC_EINVAL;
    if (p->head_mask && p->d_max > 32) return ORC_EINVAL;   /* the mask has 32 bits */
    if (p->sample_temperature < 0 || (p->sample_temperature > 0 && (!p->sample_u || !(p->top_p > 0) || p->top_p > 1)))
        return ORC_EINVAL;
    return ORC_OK;
}

/* Prefill: every prompt position through every layer; the first generated token
 * is the greedy token at the last prompt position (prefill is that of the base
 * model, Sec. 4.3 latency paragraph). */
int32_t orc_prefill(orc_session *s, const int32_t *prompt, int32_t n, int32_t *first_token) {
    const orc_config *c = &s->m->cfg;
    if (!prompt || n < 1 || !first_token) return ORC_EINVAL;
    if (n > c->max_seq) return ORC_ECAPACITY;
    for (int32_t i = 0; i < n; ++i)
        if (prompt[i] < 0 || prompt[i] >= c->vocab) return ORC_EINVAL;
    orc_session_reset(s);
    real *h = s->slots[0].h;
    for (int32_t i = 0; i < n; ++i) {
        embed_row(s->m, prompt[i], h);
        for (int32_t l = 0; l < c->n_layers; ++l) {
            layer_row(s, l, i, h);
            s->st.layer_sweeps++; s->st.row_layers++;
        }
    }
    s->c = n;
    s->pending = final_head(s, h, s->verify_logits);
    s->has_pending = 1;
    *first_token = s->pending;
    return ORC_OK;
}

/* Teacher-forced single step: token tok at position c through all layers;
 * returns the full model's logits for the next token.  Commits the position. */
int32_t orc_step(orc_session *s, int32_t tok, double *logits_out, int32_t *argmax_out) {
    const orc_config *c = &s->m->cfg;
    if (tok < 0 || tok >= c->vocab) return ORC_EINVAL;
    if (s->n_slots) return ORC_ESTATE;
    if (s->c >= c->max_seq) return ORC_ECAPACITY;
    real *h = s->slots[0].h;
    embed_row(s->m, tok, h);
    for (int32_t l = 0; l < c->n_layers; ++l) {
        layer_row(s, l, s->c, h);
        s->st.layer_sweeps++; s->st.row_layers++;
    }
    s->c += 1;
    int32_t g = final_head(s, h, s->verify_logits);
    s->pending = g; s->has_pending = 1;
    if (logits_out)
        for (int32_t j = 0; j < c->vocab; ++j) logits_out[j] = (double)s->verify_logits[j];
    if (argmax_out) *argmax_out = g;
    return ORC_OK;
}

/* One draft step (Sec. 3.3): the newest token goes through layers 1..d_max; after
 * each layer its exit head is evaluated with temperature T_l (Eq. 2) and it exits
 * at the first layer whose confidence reaches the threshold (or at the forced
 * layer).  Exit at layer d_max is allowed (Appendix A: a token exits at layer 6
 * with d_max = 6).  No exit by d_max ends the round (depth bound); the w_max-th
 * exited draft ends it too (width bound counts exited drafts). */
int32_t orc_draft_step(orc_session *s, const orc_params *p, orc_draft_result *res) {
    int rc = check_params(s, p);
    if (rc != ORC_OK) return rc;
    if (!res) return ORC_EINVAL;
    if (!s->has_pending || s->round_closed) return ORC_ESTATE;
    if (s->n_slots >= p->w_max) return ORC_ESTATE;
    const orc_config *c = &s->m->cfg;
    if (s->c + s->n_slots >= c->max_seq) return ORC_ECAPACITY;

    int64_t k = s->draft_counter;
    int32_t forced = (p->forced_exit && k < p->n_forced) ? p->forced_exit[k] : -1;
    int32_t override = (p->forced_draft && k < p->n_forced) ? p->forced_draft[k] : -1;
    if (forced > p->d_max || override >= c->vocab) return ORC_EINVAL;
    if (forced >= 1 && p->head_mask && !((p->head_mask >> (forced - 1)) & 1u)) return ORC_EINVAL;
    s->draft_counter++;
    s->st.draft_steps++;

    int32_t idx = s->n_slots;
    int32_t cur = idx == 0 ? s->pending : s->drafts[s->n_drafts - 1];
    orc_slot *sl = &s->slots[idx];
    sl->pos = s->c + idx; sl->tok = cur; sl->reached = 0; sl->exit_layer = 0;
    embed_row(s->m, cur, sl->h);
    s->n_slots++;

    res->token = -1; res->exit_layer = 0; res->status = ORC_DEPTH_BOUND; res->confidence = 0;
    for (int32_t l = 1; l <= p->d_max; ++l) {
        advance_rows(s, l, ORC_PH_DRAFT);
        if (p->head_mask && !((p->head_mask >> (l - 1)) & 1u)) continue;   /* no head at this layer */
        orc_rmsnorm(sl->h, s->m->w.exit_norm[l - 1], c->d_model, c->rms_eps, s->xn);
        orc_matvec(s->m->w.exit_head[l - 1], c->weight_dtype, c->vocab, c->d_model, s->xn, s->head_logits);
        orc_act(s->head_logits, c->vocab, (real)p->T[l - 1], &s->last_argmax, &s->last_conf);
        s->st.head_evals++;
        res->confidence = (float)s->last_conf;
        int exit_now = forced >= 0 ? (l == forced) : (s->last_conf >= (real)p->threshold);
        if (exit_now) {
            int32_t t = override >= 0 ? override : s->last_argmax;
            s->drafts[s->n_drafts++] = t;
            sl->exit_layer = l;
            res->token = t; res->exit_layer = l;
            res->status = s->n_drafts == p->w_max ? ORC_WIDTH_BOUND : ORC_EXITED;
            s->st.drafts++;
            s->st.exit_hist[l < 64 ? l : 64]++;
            break;
        }
    }
    if (res->status != ORC_EXITED) s->round_closed = 1;
    if (res->status == ORC_DEPTH_BOUND) s->st.exit_hist[0]++;
    if (s->eager_align) {
        int32_t D = s->slots[0].reached;
        for (int32_t l = 2; l <= D; ++l) advance_rows(s, l, ORC_PH_ALIGN);
    }
    return ORC_OK;
}

/* Verification (Sec. 3.3, Appendix A): bring every cached row up to the deepest
 * layer any of them reached, send all rows through the remaining layers in one
 * pass with causal attention, take the full model's greedy token g_i after each
 * row, and keep the longest prefix of drafts that equals them.  The row after the
 * last match yields one more full-model token (the "difficult" or corrected
 * token), so a round emits min(m + 1, rows) >= 1 tokens.  Cached KV of rows past
 * the emitted ones is dropped at every layer. */
int32_t orc_verify(orc_session *s, const orc_params *p, orc_verify_result *res) {
    int rc = check_params(s, p);
    if (rc != ORC_OK) return rc;
    if (!res) return ORC_EINVAL;
    if (s->n_slots == 0) return ORC_ESTATE;
    const orc_config *c = &s->m->cfg;
    int32_t M = s->n_slots;
    int32_t D = s->slots[0].reached;
    for (int32_t j = 1; j < M; ++j)
        if (s->slots[j].reached > s->slots[j - 1].reached) return ORC_ESTATE; /* invariant */
    for (int32_t l = 2; l <= D; ++l) advance_rows(s, l, ORC_PH_ALIGN);
    for (int32_t l = D + 1; l <= c->n_layers; ++l) advance_rows(s, l, ORC_PH_VERIFY);
    int32_t g[ORC_MAX_W];
    for (int32_t i = 0; i < M; ++i)
        g[i] = final_head(s, s->slots[i].h, s->verify_logits + (size_t)i * c->vocab);
    int32_t m = 0;
    if (p->sample_temperature > 0) {
        /* Sampling-mode verification.  The paper reports it (Sec. 4.3, Table 3) without giving
         * the rule; taken here: the rule of speculative sampling for a draft that was proposed
         * deterministically (the exit head's arg max x_i, as in greedy mode).  With P_i the
         * distribution the full model samples from after row i (temperature, top-p):
         *   draft x_i is accepted with probability P_i(x_i)            (u_accept < P_i(x_i));
         *   at the first rejection the token is drawn from P_i without x_i, renormalised;
         *   if every draft is accepted and a further row exists, its token is drawn from P_i.
         * Then Pr[token = x] = P(x) and Pr[token = y != x] = (1 - P(x)) P(y) / (1 - P(x)) = P(y):
         * every emitted token is distributed as the full model's own sample, and a temperature
         * towards 0 gives back the greedy rule.  min(m + 1, rows) tokens are emitted as before. */
        if (p->n_sample_u < 2 * (int64_t)(s->slots[M - 1].pos + 1)) return ORC_EINVAL;
        for (int32_t i = 0; i < M; ++i)
            orc_sample_dist(s->verify_logits + (size_t)i * c->vocab, c->vocab, (real)p->sample_temperature,
                            (real)p->top_p, s->verify_dist + (size_t)i * c->vocab, s->sort_buf);
        while (m < s->n_drafts && m < M) {
            const real *P = s->verify_dist + (size_t)m * c->vocab;
            if ((real)p->sample_u[2 * (int64_t)s->slots[m].pos] < P[s->drafts[m]]) { g[m] = s->drafts[m]; ++m; }
            else break;
        }
        if (m < M)
            g[m] = orc_sample_token(s->verify_dist + (size_t)m * c->vocab, c->vocab,
                                    (real)p->sample_u[2 * (int64_t)s->slots[m].pos + 1], m < s->n_drafts ? s->drafts[m] : -1);
        for (int32_t i = m + 1; i < M; ++i) g[i] = -1;   /* rows past the first rejection decide nothing */
    } else {
        while (m < s->n_drafts && m < M && s->drafts[m] == g[m]) ++m;
    }
    int32_t n_emit = m + 1 < M ? m + 1 : M;
    res->n_rows = M; res->n_drafts = s->n_drafts; res->n_matched = m; res->n_emit = n_emit;
    res->align_layer = D;
    for (int32_t i = 0; i < ORC_MAX_W; ++i) res->tokens[i] = i < M ? g[i] : -1;
    s->c += n_emit;
    s->pending = g[n_emit - 1];
    s->n_slots = 0; s->n_drafts = 0; s->round_closed = 0;
    s->st.rounds++; s->st.emitted += n_emit; s->st.accept_hist[n_emit]++;
    return ORC_OK;
}

/* Give back the last `n` committed positions (used when a round's emission is cut
 * short by max_new or an end-of-sequence id). */
static void uncommit(orc_session *s, int32_t n, int32_t new_pending) {
    s->c -= n;
    s->st.emitted -= n;
    s->pending = new_pending;
}

int32_t orc_generate(orc_session *s, const int32_t *prompt, int32_t n, int32_t max_new,
                     const orc_params *p, int32_t *out, int32_t out_cap, int32_t *n_out) {
    int rc = check_params(s, p);
    if (rc != ORC_OK) return rc;
    if (!out || !n_out || max_new < 1 || out_cap < max_new) return ORC_EINVAL;
    if ((int64_t)n + max_new + p->w_max > s->m->cfg.max_seq) return ORC_ECAPACITY;
    int32_t tok;
    rc = orc_prefill(s, prompt, n, &tok);
    if (rc != ORC_OK) return rc;
    int32_t cnt = 0;
    out[cnt++] = tok;
    while (cnt < max_new && !(p->eos_id >= 0 && out[cnt - 1] == p->eos_id)) {
        orc_draft_result dr;
        do {
            rc = orc_draft_step(s, p, &dr);
            if (rc != ORC_OK) return rc;
        } while (dr.status == ORC_EXITED);
        orc_verify_result vr;
        rc = orc_verify(s, p, &vr);
        if (rc != ORC_OK) return rc;
        int32_t take = 0;
        while (take < vr.n_emit && cnt < max_new) {
            out[cnt++] = vr.tokens[take++];
            if (p->eos_id >= 0 && out[cnt - 1] == p->eos_id) break;
        }
        if (take < vr.n_emit) uncommit(s, vr.n_emit - take, out[cnt - 1]);
    }
    *n_out = cnt;
    return ORC_OK;
}

/* Brute force: greedy decoding with NO KV cache.  For every new token the whole
 * sequence is recomputed from the embeddings, layer by layer over all positions,
 * with K and V built afresh.  This is the definition the cached paths are pinned
 * to: x_{t+1} = argmax lm_head(final_norm(Decoder(x_{<=t}))).  last_logits
 * (nullable) receives the logits that chose the last token. */
int32_t orc_greedy_nocache(orc_model *m, const int32_t *prompt, int32_t n, int32_t max_new,
                           int32_t *out, double *last_logits) {
    const orc_config *c = &m->cfg;
    int32_t d = c->d_model, hd = c->head_dim, Hq = c->n_heads, Hkv = c->n_kv_heads, f = c->d_ffn;
    int32_t half = hd / 2, group = Hq / Hkv, total = n + max_new;
    size_t kvw = (size_t)Hkv * hd;
    int32_t qkv_rows = (Hq + 2 * Hkv) * hd;
    if (total > c->max_seq) return ORC_ECAPACITY;
    int32_t *seq = (int32_t *)malloc(sizeof(int32_t) * total);
    real *H = (real *)malloc(sizeof(real) * (size_t)total * d);
    real *Q = (real *)malloc(sizeof(real) * (size_t)total * Hq * hd);
    float *K = (float *)malloc(sizeof(float) * (size_t)total * kvw);
    float *Vv = (float *)malloc(sizeof(float) * (size_t)total * kvw);
    real *xn = (real *)malloc(sizeof(real) * d), *qkv = (real *)malloc(sizeof(real) * qkv_rows);
    real *att = (real *)malloc(sizeof(real) * (size_t)Hq * hd), *o = (real *)malloc(sizeof(real) * d);
    real *gu = (real *)malloc(sizeof(real) * 2 * f), *u = (real *)malloc(sizeof(real) * f);
    real *sc = (real *)malloc(sizeof(real) * total), *z = (real *)malloc(sizeof(real) * c->vocab);
    memcpy(seq, prompt, sizeof(int32_t) * n);
    for (int32_t step = 0; step < max_new; ++step) {
        int32_t len = n + step;
        for (int32_t t = 0; t < len; ++t) {
            if (c->weight_dtype == ORC_BF16) {
                const uint16_t *e = (const uint16_t *)m->w.embed + (size_t)seq[t] * d;
                for (int32_t i = 0; i < d; ++i) H[(size_t)t * d + i] = (real)bf16_bits_to_float(e[i]);
            } else {
                const float *e = (const float *)m->w.embed + (size_t)seq[t] * d;
                for (int32_t i = 0; i < d; ++i) H[(size_t)t * d + i] = (real)e[i];
            }
        }
        for (int32_t l = 0; l < c->n_layers; ++l) {
            for (int32_t t = 0; t < len; ++t) {
                orc_rmsnorm(H + (size_t)t * d, m->w.attn_norm[l], d, c->rms_eps, xn);
                orc_matvec(m->w.w_qkv[l], c->weight_dtype, qkv_rows, d, xn, qkv);
                const float *cs = m->rope_cos + (size_t)t * half, *sn = m->rope_sin + (size_t)t * half;
                for (int32_t i = 0; i < Hq; ++i) orc_rope_apply(qkv + (size_t)i * hd, hd, cs, sn);
                for (int32_t i = 0; i < Hkv; ++i) orc_rope_apply(qkv + (size_t)(Hq + i) * hd, hd, cs, sn);
                memcpy(Q + (size_t)t * Hq * hd, qkv, sizeof(real) * (size_t)Hq * hd);
                for (size_t i = 0; i < kvw; ++i) {
                    float kf = (float)qkv[(size_t)Hq * hd + i], vf = (float)qkv[(size_t)Hq * hd + kvw + i];
                    K[(size_t)t * kvw + i] = c->kv_dtype == ORC_BF16 ? round_bf16(kf) : kf;
                    Vv[(size_t)t * kvw + i] = c->kv_dtype == ORC_BF16 ? round_bf16(vf) : vf;
                }
            }
            for (int32_t t = 0; t < len; ++t) {
                real *h = H + (size_t)t * d;
                for (int32_t i = 0; i < Hq; ++i)
                    orc_attention_head(Q + ((size_t)t * Hq + i) * hd, K + (size_t)(i / group) * hd,
                                       Vv + (size_t)(i / group) * hd, t + 1, hd, kvw, sc, att + (size_t)i * hd);
                orc_matvec(m->w.w_o[l], c->weight_dtype, d, Hq * hd, att, o);
                for (int32_t i = 0; i < d; ++i) h[i] += o[i];
                orc_rmsnorm(h, m->w.ffn_norm[l], d, c->rms_eps, xn);
                orc_matvec(m->w.w_gate_up[l], c->weight_dtype, 2 * f, d, xn, gu);
                for (int32_t i = 0; i < f; ++i) u[i] = gu[i] / ((real)1 + R_EXP(-gu[i])) * gu[f + i];
                orc_matvec(m->w.w_down[l], c->weight_dtype, d, f, u, o);
                for (int32_t i = 0; i < d; ++i) h[i] += o[i];
            }
        }
        orc_rmsnorm(H + (size_t)(len - 1) * d, m->w.final_norm, d, c->rms_eps, xn);
        orc_matvec(m->w.lm_head, c->weight_dtype, c->vocab, d, xn, z);
        int32_t im = 0;
        for (int32_t j = 1; j < c->vocab; ++j)
            if (z[j] > z[im]) im = j;
        seq[len] = im;
        out[step] = im;
        if (last_logits && step == max_new - 1)
            for (int32_t j = 0; j < c->vocab; ++j) last_logits[j] = (double)z[j];
    }
    free(seq); free(H); free(Q); free(K); free(Vv); free(xn); free(qkv); free(att); free(o);
    free(gu); free(u); free(sc); free(z);
    return ORC_OK;
}

int32_t orc_real_bytes(void) { return (int32_t)sizeof(real); }

/* threads the matrix-vector loops run on */
int32_t orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
