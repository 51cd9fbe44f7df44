/* Drives the CPU oracle (test infrastructure) through every entry point on a tiny random model,
 * as one translation unit, so that it can be built with AddressSanitizer and
 * UndefinedBehaviorSanitizer and run as a plain executable (tests/test_oracle_sanitizers.py).
 * It checks what the method guarantees (Sec. 3.3: the speculative output is the greedy one)
 * and otherwise only that every path runs clean; values are pinned by the Python tests. */
#include <stdio.h>
#include "../oracle/specbound_oracle.c"

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static double rnd(void) {   /* xorshift64*, uniform in [0, 1) */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0;
}
static float *randn(size_t n, float std) {
    float *p = malloc(n * sizeof(float));
    for (size_t i = 0; i < n; ++i) {   /* sum of uniforms: close enough to normal for a smoke model */
        double s = 0; for (int k = 0; k < 6; ++k) s += rnd();
        p[i] = (float)((s - 3.0) * 1.41421356 * std);
    }
    return p;
}
static uint16_t *to_bf16(const float *f, size_t n) {
    uint16_t *b = malloc(n * 2);
    for (size_t i = 0; i < n; ++i) { float r = round_bf16(f[i]); uint32_t u; memcpy(&u, &r, 4); b[i] = (uint16_t)(u >> 16); }
    return b;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int run(int bf16, int n_kv_heads) {
    enum { L = 5, NE = 3, D = 64, H = 4, HD = 16, F = 96, V = 211, SEQ = 96 };
    orc_config cfg = {L, D, H, n_kv_heads, HD, F, V, 1e-6f, 10000.0f, bf16 ? ORC_BF16 : ORC_FP32,
                      bf16 ? ORC_BF16 : ORC_FP32, NE, SEQ};
    const int qkv = (H + 2 * n_kv_heads) * HD;
    const void *wq[L], *wo[L], *wgu[L], *wd[L], *eh[NE];
    const float *an[L], *fn[L], *en[NE];
    void *owned[6 * L + 3 * NE + 8]; int n_owned = 0;
#define MAT(rows, cols, std) ({ float *f_ = randn((size_t)(rows) * (cols), std); void *r_ = f_; \
        if (bf16) { r_ = to_bf16(f_, (size_t)(rows) * (cols)); free(f_); } owned[n_owned++] = r_; (const void *)r_; })
#define GAIN() ({ float *g_ = randn(D, 0.1f); for (int i_ = 0; i_ < D; ++i_) g_[i_] += 1.0f; owned[n_owned++] = g_; (const float *)g_; })
    for (int l = 0; l < L; ++l) {
        wq[l] = MAT(qkv, D, 0.08f); wo[l] = MAT(D, H * HD, 0.05f); wgu[l] = MAT(2 * F, D, 0.08f); wd[l] = MAT(D, F, 0.05f);
        an[l] = GAIN(); fn[l] = GAIN();
    }
    for (int l = 0; l < NE; ++l) { eh[l] = MAT(V, D, 0.3f); en[l] = GAIN(); }
    orc_weights w = {MAT(V, D, 1.0f), MAT(V, D, 0.3f), GAIN(), an, wq, wo, fn, wgu, wd, en, eh};
    orc_model *m = NULL; orc_session *s = NULL;
    CHECK(orc_model_new(&cfg, &w, &m) == ORC_OK);
    CHECK(orc_session_new(m, &s) == ORC_OK);
    CHECK(orc_trace_enable(s, 4096) == ORC_OK);

    int32_t prompt[9] = {3, 17, 200, 5, 5, 99, 150, 42, 7};
    int32_t ref[40], out[40], n_out = 0;
    CHECK(orc_greedy_nocache(m, prompt, 9, 24, ref, NULL) == ORC_OK);

    float T[NE]; orc_temperature_schedule(0.2, L, NE, T);
    /* computed exits at a low threshold, then forced schedules with wrong drafts injected */
    orc_params p = {NE, 4, T, 0.02f, -1, NULL, NULL, 0, 0, 0.f, 1.f, NULL, 0};
    CHECK(orc_generate(s, prompt, 9, 24, &p, out, 40, &n_out) == ORC_OK && n_out == 24);
    for (int i = 0; i < 24; ++i) CHECK(out[i] == ref[i]);
    int32_t fe[64], fd[64];
    for (int i = 0; i < 64; ++i) { fe[i] = i % (NE + 1); fd[i] = (i % 3 == 0) ? (i * 7) % V : -1; }
    p.forced_exit = fe; p.forced_draft = fd; p.n_forced = 64; p.head_mask = 0x5; /* heads at layers 1 and 3 */
    for (int i = 0; i < 64; ++i) if (fe[i] == 2) fe[i] = 3;
    orc_session_reset(s);
    CHECK(orc_generate(s, prompt, 9, 24, &p, out, 40, &n_out) == ORC_OK && n_out == 24);
    for (int i = 0; i < 24; ++i) CHECK(out[i] == ref[i]);
    /* a width-bound round at the largest width, by hand, with the eager alignment switch on */
    orc_session_reset(s); orc_set_eager_align(s, 1);
    int32_t first; CHECK(orc_prefill(s, prompt, 9, &first) == ORC_OK && first == ref[0]);
    int32_t fe2[ORC_MAX_W]; for (int i = 0; i < ORC_MAX_W; ++i) fe2[i] = 1 + i % NE;
    orc_params pw = {NE, ORC_MAX_W, T, 0.5f, -1, fe2, NULL, ORC_MAX_W, 0, 0.f, 1.f, NULL, 0};
    orc_draft_result dr; orc_verify_result vr;
    do { CHECK(orc_draft_step(s, &pw, &dr) == ORC_OK); } while (dr.status == ORC_EXITED);
    CHECK(dr.status == ORC_WIDTH_BOUND && orc_open_slots(s) == ORC_MAX_W);
    CHECK(orc_draft_step(s, &pw, &dr) == ORC_ESTATE);
    CHECK(orc_verify(s, &pw, &vr) == ORC_OK && vr.n_emit >= 1 && vr.tokens[0] == ref[1]);
    double hid[D]; float kk[H * HD], vv[H * HD];
    orc_kv_read(s, L - 1, 9, kk, vv);
    /* sampling-mode rounds: uniforms for every position, nucleus and temperature */
    orc_session_reset(s); orc_set_eager_align(s, 0);
    float U[2 * SEQ]; for (int i = 0; i < 2 * SEQ; ++i) U[i] = (float)rnd();
    orc_params ps = {NE, 3, T, 0.02f, -1, NULL, NULL, 0, 0, 0.8f, 0.9f, U, 2 * SEQ};
    CHECK(orc_generate(s, prompt, 9, 20, &ps, out, 40, &n_out) == ORC_OK && n_out == 20);
    for (int i = 0; i < 20; ++i) CHECK(out[i] >= 0 && out[i] < V);
    /* rewind and continue greedily, single steps with logits, bad arguments */
    CHECK(orc_rewind(s, 9, ref[0]) == ORC_OK);
    orc_params pg = {NE, 1, T, 2.0f, -1, NULL, NULL, 0, 0, 0.f, 1.f, NULL, 0};
    CHECK(orc_draft_step(s, &pg, &dr) == ORC_OK && dr.status == ORC_DEPTH_BOUND);
    orc_slot_hidden(s, 0, hid);
    CHECK(orc_verify(s, &pg, &vr) == ORC_OK && vr.n_emit == 1 && vr.tokens[0] == ref[1]);
    double *lg = malloc(sizeof(double) * V); int32_t am;
    CHECK(orc_step(s, ref[1], lg, &am) == ORC_OK && am == ref[2]);
    free(lg);
    CHECK(orc_rewind(s, 0, 1) == ORC_EINVAL && orc_step(s, V, NULL, NULL) == ORC_EINVAL);
    orc_params bad = pg; bad.d_max = NE + 1;
    CHECK(orc_draft_step(s, &bad, &dr) == ORC_EINVAL);
    orc_trace_entry tr[64]; CHECK(orc_trace_read(s, tr, 64) > 0);
    orc_stats st; orc_get_stats(s, &st); CHECK(st.rounds > 0);
    orc_session_free(s); orc_model_free(m);
    for (int i = 0; i < n_owned; ++i) free(owned[i]);
    return 0;
}

int main(void) {
    if (run(0, 4)) return 1;   /* fp32 weights and cache, one kv head per query head */
    if (run(1, 2)) return 1;   /* bf16 weights and cache, two query heads per kv head */
    /* primitives on their own */
    real z[7] = {0.1f, 2.5f, -1.f, 2.5f, 0.f, 1.f, -3.f}, pr[7], tmp[7], conf; int32_t am;
    orc_act(z, 7, (real)1.3, &am, &conf);
    if (am != 1 || !(conf > 0 && conf < 1)) return 1;
    orc_sample_dist(z, 7, (real)0.7, (real)0.6, pr, tmp);
    if (orc_sample_token(pr, 7, (real)0.999999, 1) == 1) return 1;
    printf("oracle sanitizer run: ok\n");
    return 0;
}
