// Rounds of several sequences side by side (sb_new_batch / sb_batch_decode): the batch > 1 form of
// Bounded Speculation with Cached States (Sec. 3.3; Sec. 4.3 evaluates batch 1).
#include "host.h"

using namespace sb;
using namespace sbhost;

namespace {

// ---------------------------------------------------------------- batch > 1
// One decoder layer (0-based l) on the rows of `mask`: sequence b contributes its local rows
// j0[b] .. j0[b] + cnt[b] - 1 (cnt 0: none).  Projections: one launch each for all rows (the rows
// are gathered by slot).  Attention: per sequence, on its own cache.  Values of a row are what the
// single-sequence pass computes for it (a row's result never depends on the rows beside it).
int batch_layer(sb_batch* bt, int l, uint32_t mask, const int* j0, const int* cnt, const float* head_gain) {
    sb_session* hs = bt->seq[0];
    sb_model* m = bt->m;
    const sb_config& c = m->cfg;
    hipStream_t st = m->stream;
    const int d = c.d_model, f = c.d_ffn, hq = c.n_heads * c.head_dim;
    const int qkv_rows = (c.n_heads + 2 * c.n_kv_heads) * c.head_dim;
    float* H = wsp<float>(hs, hs->L.H);
    uint16_t* xs_attn = wsp<uint16_t>(hs, hs->L.xs_attn);
    uint16_t* xs_ffn = wsp<uint16_t>(hs, hs->L.xs_ffn);
    uint16_t* xs_exit = wsp<uint16_t>(hs, hs->L.xs_exit);
    float* ssq_attn = wsp<float>(hs, hs->L.ssq_attn);
    float* ssq_ffn = wsp<float>(hs, hs->L.ssq_ffn);
    float* qkv = wsp<float>(hs, hs->L.qkv);
    uint16_t* atts = wsp<uint16_t>(hs, hs->L.atts);
    uint16_t* us = wsp<uint16_t>(hs, hs->L.us);
    int rc;
    GemvArgs g{};
    g.w_dtype = c.weight_dtype; g.M = SB_MAX_W; g.row_mask = mask; g.eps = c.rms_eps; g.ssq_ld = hs->L.ssq_ld;
    g.W = m->w_qkv[l]; g.N = qkv_rows; g.K = d; g.xs = xs_attn; g.y = qkv; g.ldy = qkv_rows; g.epi = EPI_STORE;
    g.ssq_in = ssq_attn; g.ssq_nb = l == 0 ? 1 : d / 16;
    if ((rc = gemv(hs, g, SB_K_QKV, st))) return rc;
    int64_t kv_total = 0;
    AttnArgs passes[SB_MAX_W];
    int n_pass = 0;
    for (int b = 0; b < bt->B; ++b) {
        if (!cnt[b]) continue;
        sb_session* s = bt->seq[b];
        const int slot = b * bt->w_cap + j0[b];
        AttnArgs a{};
        a.q = qkv + (size_t)slot * qkv_rows; a.rope_cos = m->rope_cos; a.rope_sin = m->rope_sin; a.qkv_rows = qkv_rows;
        a.n_heads = c.n_heads; a.kv = s->kv; a.layer = l; a.pos0 = s->c + j0[b]; a.M = cnt[b];
        a.partials = wsp<float>(s, s->L.attn_part); a.max_chunks = s->L.max_chunks;
        a.out = nullptr; a.out_split = atts + (size_t)slot * hq; a.split_rows = 8;
        const int64_t kv_read = (int64_t)(a.pos0 + a.M) * 2 * c.n_kv_heads * c.head_dim * (int64_t)esize(c.kv_dtype);
        passes[n_pass++] = a;
        s->st.kv_bytes += kv_read;
        s->st.row_layers += cnt[b];
        kv_total += kv_read;
    }
    if (n_pass) {  // all sequences' passes in one pair of launches
        ProfScope ps(hs, SB_K_ATTN, kv_total, st);
        HIP_TRY(launch_attention_batch(passes, n_pass, st));
    }
    g.ssq_in = nullptr;
    g.W = m->w_o[l]; g.N = d; g.K = hq; g.xs = atts; g.y = H; g.ldy = d; g.epi = EPI_RESID;
    g.gainA = m->ffn_norm[l]; g.nxA = xs_ffn; g.ssq_out = ssq_ffn;
    if ((rc = gemv(hs, g, SB_K_WO, st))) return rc;
    g.gainA = nullptr; g.nxA = nullptr; g.ssq_out = nullptr;
    g.W = m->w_gate_up[l]; g.N = f; g.K = d; g.xs = xs_ffn; g.y = nullptr; g.ys = us; g.ldy = f; g.epi = EPI_SWIGLU;
    g.ssq_in = ssq_ffn; g.ssq_nb = d / 16;
    if ((rc = gemv(hs, g, SB_K_GATEUP, st))) return rc;
    g.ssq_in = nullptr;
    g.W = m->w_down[l]; g.N = d; g.K = f; g.xs = us; g.y = H; g.ys = nullptr; g.ldy = d; g.epi = EPI_RESID;
    if (l + 1 < c.n_layers) { g.gainA = m->attn_norm[l + 1]; g.nxA = xs_attn; }
    if (head_gain) { g.gainB = head_gain; g.nxB = xs_exit; }
    g.ssq_out = ssq_attn;
    if ((rc = gemv(hs, g, SB_K_DOWN, st))) return rc;
    hs->st.layer_sweeps += 1;      // the shared sweep is counted once, on the first sequence
    hs->st.weight_bytes += m->layer_bytes;
    if (hs->phase_bytes) *hs->phase_bytes += m->layer_bytes + kv_total;
    return SB_OK;
}

// Head projection of the rows of `mask` (partials only; the caller merges per sequence).
int batch_head(sb_batch* bt, const void* W, uint32_t mask, float T, float* logits, int cls) {
    sb_session* hs = bt->seq[0];
    const sb_config& c = bt->m->cfg;
    GemvArgs g{};
    g.W = W; g.w_dtype = c.weight_dtype; g.N = c.vocab; g.K = c.d_model; g.M = SB_MAX_W; g.row_mask = mask;
    g.xs = wsp<uint16_t>(hs, hs->L.xs_exit);
    g.ssq_in = wsp<float>(hs, hs->L.ssq_attn); g.ssq_nb = c.d_model / 16; g.ssq_ld = hs->L.ssq_ld; g.eps = c.rms_eps;
    g.epi = EPI_HEAD;
    g.head.T = T; g.head.partials = wsp<float>(hs, hs->L.head_part); g.head.logits = logits; g.head.skip_merge = 1;
    int rc = gemv(hs, g, cls, bt->m->stream);
    if (rc) return rc;
    hs->st.weight_bytes += bt->m->head_bytes;
    if (hs->phase_bytes) *hs->phase_bytes += bt->m->head_bytes;
    return SB_OK;
}

int batch_readback(sb_batch* bt, const std::vector<int>& who) {
    for (int b : who) {
        sb_session* s = bt->seq[b];
        HIP_TRY(hipMemcpyAsync(s->h_round, s->d_round, sizeof(DevRound), hipMemcpyDeviceToHost, bt->m->stream));
    }
    HIP_TRY(hipStreamSynchronize(bt->m->stream));
    return SB_OK;
}

// One round of every sequence of `act`: draft super-steps (each adds a row to every sequence that
// is still drafting; layer passes gather the rows of all of them), then alignment and
// verification of all open rows layer by layer, one head sweep, and per sequence the accept rule.
int batch_round(sb_batch* bt, const std::vector<int>& act, const sb_params* const* P, sb_verify_result* vres) {
    sb_model* m = bt->m;
    const sb_config& c = m->cfg;
    sb_session* hs = bt->seq[0];
    hipStream_t st = m->stream;
    const int B = bt->B, wc = bt->w_cap, d = c.d_model;
    const int nb_head = head_blocks_mfma(c.vocab);
    int rc;
    std::vector<char> drafting(B, 0), inflight(B, 0);
    for (int b : act) { drafting[b] = 1; bt->seq[b]->n_slots = 0; bt->seq[b]->n_drafts = 0; bt->seq[b]->round_closed = false; }
    int d_max_all = 0;
    for (int b : act) d_max_all = P[b]->d_max > d_max_all ? P[b]->d_max : d_max_all;
    hs->phase_bytes = &hs->st.draft_bytes;
    // ---- draft super-steps
    for (;;) {
        std::vector<int> step;  // sequences that add a row in this super-step
        for (int b : act)
            if (drafting[b]) step.push_back(b);
        if (step.empty()) break;
        std::vector<int> forced(B, -1), over(B, -1);
        for (int b : step) {
            sb_session* s = bt->seq[b];
            const sb_params* p = P[b];
            if (s->c + s->n_slots >= c.max_seq) return fail(SB_ECAPACITY, "batch_decode: KV capacity of sequence %d exceeded", b);
            const int64_t k = s->draft_counter;
            forced[b] = (p->forced_exit && k < p->n_forced) ? p->forced_exit[k] : -1;
            over[b] = (p->forced_draft && k < p->n_forced) ? p->forced_draft[k] : -1;
            if (forced[b] > p->d_max) return fail(SB_EINVAL, "forced_exit[%lld] = %d exceeds d_max", (long long)k, forced[b]);
            if (forced[b] >= 1 && p->head_mask && !((p->head_mask >> (forced[b] - 1)) & 1u))
                return fail(SB_EINVAL, "forced_exit[%lld] = %d names a layer outside head_mask", (long long)k, forced[b]);
            if (over[b] >= c.vocab) return fail(SB_EINVAL, "forced_draft[%lld] = %d out of range", (long long)k, over[b]);
            if (forced[b] < -1) forced[b] = -1;
            if (over[b] < -1) over[b] = -1;
            const int idx = s->n_slots, slot = b * wc + idx;
            if (!(idx > 0 && s->next_embedded)) {
                RowToks t;
                for (int r = 0; r < SB_MAX_W; ++r) t.tok[r] = 0;
                t.tok[0] = idx == 0 ? s->pending : s->draft_host[idx - 1];
                EmbedNorm en{m->attn_norm[0], wsp<uint16_t>(hs, hs->L.xs_attn) + (size_t)slot * d,
                             wsp<float>(hs, hs->L.ssq_attn) + (size_t)slot * hs->L.ssq_ld, hs->L.ssq_ld};
                HIP_TRY(launch_embed(m->embed, c.weight_dtype, c.vocab, d, wsp<float>(hs, hs->L.H) + (size_t)slot * d, 1, t,
                                     s->d_round->slot_tok + idx, &s->d_round->exit_flag, en, st));
            }
            s->next_embedded = false;
            s->draft_counter++; s->st.draft_steps++; s->n_slots++;
            s->reached[idx] = 0; s->exit_layer[idx] = 0; s->draft_host[idx] = -1;
            inflight[b] = 1;
        }
        std::vector<int> exit_at(B, 0), heads_run(B, 0);
        for (int l = 1; l <= d_max_all; ++l) {
            uint32_t mask = 0, newest = 0;
            int j0[SB_MAX_W] = {0}, cnt[SB_MAX_W] = {0};
            bool any_head = false;
            for (int b : step) {
                if (!inflight[b] || l > P[b]->d_max) { inflight[b] = 0; continue; }
                sb_session* s = bt->seq[b];
                const int idx = s->n_slots - 1;
                int j = idx;
                while (j > 0 && s->reached[j - 1] == l - 1) --j;
                j0[b] = j; cnt[b] = idx - j + 1;
                for (int r = j; r <= idx; ++r) mask |= 1u << (b * wc + r);
                if (!P[b]->head_mask || ((P[b]->head_mask >> (l - 1)) & 1u)) { newest |= 1u << (b * wc + idx); any_head = true; }
            }
            if (!mask) break;
            if ((rc = batch_layer(bt, l - 1, mask, j0, cnt, any_head ? m->exit_norm[l - 1] : nullptr))) return rc;
            for (int b : step)
                for (int r = j0[b]; r < j0[b] + cnt[b]; ++r) bt->seq[b]->reached[r] = l;
            if (!newest) continue;
            // the exit head of layer l for the newest row of every sequence that tests here: one sweep.
            // (Each row's logits are scaled by its own temperature in the merge: T enters the partial
            // sums, so the sweep is taken per distinct temperature; the usual case is one.)
            std::vector<int> todo;
            for (int b : step)
                if (cnt[b] && ((newest >> (b * wc + bt->seq[b]->n_slots - 1)) & 1u)) todo.push_back(b);
            while (!todo.empty()) {
                const float T = P[todo[0]]->T[l - 1];
                uint32_t hm = 0;
                std::vector<int> now, later;
                for (int b : todo) (P[b]->T[l - 1] == T ? now : later).push_back(b);
                for (int b : now) hm |= 1u << (b * wc + bt->seq[b]->n_slots - 1);
                float* logits = hs->debug ? wsp<float>(hs, hs->L.logits_exit) + (size_t)(l - 1) * c.vocab : nullptr;
                (void)logits;
                if ((rc = batch_head(bt, m->exit_head[l - 1], hm, T, nullptr, SB_K_EXIT_HEAD))) return rc;
                HeadMergeBatch hb{};
                int n_merge = 0;
                for (int b : now) {
                    sb_session* s = bt->seq[b];
                    const int idx = s->n_slots - 1, slot = b * wc + idx;
                    HeadArgs& h = hb.h[n_merge];
                    h.T = T; h.partials = wsp<float>(hs, hs->L.head_part); h.post = POST_EXIT; h.round = s->d_round;
                    h.slot = idx; h.layer = l; h.forced_exit = forced[b]; h.forced_draft = over[b]; h.threshold = P[b]->threshold;
                    h.row0 = slot;
                    if (s->n_drafts + 1 < P[b]->w_max && idx + 1 < wc) {
                        h.embed_E = m->embed; h.embed_dtype = c.weight_dtype; h.embed_vocab = c.vocab; h.embed_d = d;
                        h.embed_H = wsp<float>(hs, hs->L.H) + (size_t)(slot + 1) * d;
                        h.embed_en = EmbedNorm{m->attn_norm[0], wsp<uint16_t>(hs, hs->L.xs_attn) + (size_t)(slot + 1) * d,
                                               wsp<float>(hs, hs->L.ssq_attn) + (size_t)(slot + 1) * hs->L.ssq_ld, hs->L.ssq_ld};
                    }
                    hb.M[n_merge++] = 1;
                    s->st.head_evals++;
                    heads_run[b]++;
                }
                HIP_TRY(launch_head_merge_batch(hb, n_merge, nb_head, st));
                todo.swap(later);
            }
            // exits: known to the host under a forced schedule, else read back
            std::vector<int> ask;
            for (int b : step)
                if (cnt[b] && ((newest >> (b * wc + bt->seq[b]->n_slots - 1)) & 1u)) {
                    if (forced[b] >= 0) { if (l == forced[b]) { exit_at[b] = l; inflight[b] = 0; } }
                    else ask.push_back(b);
                }
            if (!ask.empty()) {
                if ((rc = batch_readback(bt, ask))) return rc;
                for (int b : ask)
                    if (bt->seq[b]->h_round->exit_flag) { exit_at[b] = l; inflight[b] = 0; }
            }
        }
        for (int b : step) {
            sb_session* s = bt->seq[b];
            const int idx = s->n_slots - 1;
            inflight[b] = 0;
            if (exit_at[b]) {
                s->exit_layer[idx] = exit_at[b];
                s->next_embedded = s->n_drafts + 1 < P[b]->w_max && idx + 1 < wc;
                s->draft_host[idx] = over[b] >= 0 ? over[b] : (forced[b] < 0 ? s->h_round->drafts[idx] : -1);
                s->n_drafts++; s->st.drafts++; s->st.exit_hist[exit_at[b]]++;
                if (s->n_drafts == P[b]->w_max) { s->round_closed = true; drafting[b] = 0; }
            } else {
                s->st.exit_hist[0]++;
                s->round_closed = true; drafting[b] = 0;
            }
        }
    }
    // ---- alignment and verification: every open row of every sequence through the layers it has not seen
    hs->phase_bytes = &hs->st.verify_bytes;
    std::vector<int> D(B, 0);
    for (int b : act) D[b] = bt->seq[b]->reached[0];
    for (int l = 1; l <= c.n_layers; ++l) {
        uint32_t mask = 0;
        int j0[SB_MAX_W] = {0}, cnt[SB_MAX_W] = {0};
        for (int b : act) {
            sb_session* s = bt->seq[b];
            int j = s->n_slots;
            while (j > 0 && s->reached[j - 1] == l - 1) --j;
            j0[b] = j; cnt[b] = s->n_slots - j;
            for (int r = j; r < s->n_slots; ++r) mask |= 1u << (b * wc + r);
        }
        if (!mask) continue;
        if ((rc = batch_layer(bt, l - 1, mask, j0, cnt, l == c.n_layers ? m->final_norm : nullptr))) return rc;
        for (int b : act)
            for (int r = j0[b]; r < j0[b] + cnt[b]; ++r) bt->seq[b]->reached[r] = l;
    }
    uint32_t all = 0;
    bool sampling = false;
    for (int b : act) {
        for (int r = 0; r < bt->seq[b]->n_slots; ++r) all |= 1u << (b * wc + r);
        sampling = sampling || P[b]->sample_temperature > 0.f;
    }
    float* logits = (sampling || hs->debug) ? wsp<float>(hs, hs->L.logits_final) : nullptr;
    if ((rc = batch_head(bt, m->lm_head, all, 1.0f, logits, SB_K_FINAL_HEAD))) return rc;
    hs->st.final_head_sweeps++;
    HeadMergeBatch hb{};
    int n_merge = 0;
    for (int b : act) {
        sb_session* s = bt->seq[b];
        const sb_params* p = P[b];
        const int M = s->n_slots;
        if (p->sample_temperature > 0.f) {
            if (p->n_sample_u < 2 * (int64_t)(s->c + M))
                return fail(SB_EINVAL, "batch_decode: sample_u of sequence %d has %lld entries, this round needs %lld", b,
                            (long long)p->n_sample_u, 2 * (long long)(s->c + M));
            SampleArgs sa{};
            sa.logits = logits + (size_t)(b * wc) * c.vocab; sa.wts = wsp<float>(hs, hs->L.sample_w) + (size_t)(b * wc) * (c.vocab > 32 * 1024 ? c.vocab - 32 * 1024 : 0);
            sa.V = c.vocab; sa.M = M; sa.n_drafts = s->n_drafts;
            sa.temp = p->sample_temperature; sa.top_p = p->top_p; sa.round = s->d_round;
            for (int i = 0; i < M; ++i) {
                sa.ua[i] = p->sample_u[2 * (int64_t)(s->c + i)];
                sa.ur[i] = p->sample_u[2 * (int64_t)(s->c + i) + 1];
            }
            HIP_TRY(launch_sample_accept(sa, st));
        } else {
            HeadArgs& h = hb.h[n_merge];
            h.T = 1.0f; h.partials = wsp<float>(hs, hs->L.head_part); h.post = POST_ACCEPT; h.round = s->d_round;
            h.n_drafts = s->n_drafts; h.row0 = b * wc;
            hb.M[n_merge++] = M;
        }
    }
    if (n_merge) HIP_TRY(launch_head_merge_batch(hb, n_merge, nb_head, st));
    if ((rc = batch_readback(bt, act))) return rc;
    for (int b : act) {
        sb_session* s = bt->seq[b];
        const DevRound& R = *s->h_round;
        const int M = s->n_slots;
        if (R.n_emit < 1 || R.n_emit > M) return fail(SB_EDEVICE, "batch_decode: device returned n_emit = %d for sequence %d", R.n_emit, b);
        sb_verify_result& res = vres[b];
        res = sb_verify_result{};
        res.n_rows = M; res.n_drafts = s->n_drafts; res.n_matched = R.n_matched; res.n_emit = R.n_emit; res.align_layer = D[b];
        for (int i = 0; i < SB_MAX_W; ++i) res.tokens[i] = i < M ? R.g[i] : -1;
        s->c += R.n_emit;
        s->pending = R.g[R.n_emit - 1];
        s->n_slots = 0; s->n_drafts = 0; s->round_closed = false; s->next_embedded = false;
        s->st.rounds++; s->st.emitted += R.n_emit; s->st.accept_hist[R.n_emit]++;
    }
    return SB_OK;
}

}  // namespace

extern "C" {

int32_t sb_new_batch(sb_session* const* sessions, int32_t B, sb_batch** out) {
    if (!sessions || !out) return fail(SB_EINVAL, "new_batch: NULL argument");
    if (B < 2 || B > SB_MAX_W) return fail(SB_EINVAL, "new_batch: B must be in 2..%d", SB_MAX_W);
    for (int b = 0; b < B; ++b) {
        if (!sessions[b]) return fail(SB_EINVAL, "new_batch: session %d is NULL", b);
        if (sessions[b]->m != sessions[0]->m) return fail(SB_EINVAL, "new_batch: the sessions must share one model");
        for (int a = 0; a < b; ++a)
            if (sessions[a] == sessions[b]) return fail(SB_EINVAL, "new_batch: session %d is listed twice", b);
    }
    if (sessions[0]->m->proj != SB_PROJ_MFMA) return fail(SB_EINVAL, "new_batch: needs the MFMA projection path (bf16 weights)");
    sb_batch* bt = new sb_batch();
    bt->m = sessions[0]->m; bt->B = B; bt->w_cap = SB_MAX_W / B;
    bt->seq.assign(sessions, sessions + B);
    *out = bt;
    return SB_OK;
}

void sb_free_batch(sb_batch* bt) { delete bt; }

int32_t sb_batch_decode(sb_batch* bt, int32_t max_new, const sb_params* const* params, int32_t* const* out_tokens,
                        int32_t* n_out) {
    if (!bt || !params || !out_tokens || !n_out || max_new < 1) return fail(SB_EINVAL, "batch_decode: bad argument");
    const int B = bt->B;
    int rc;
    for (int b = 0; b < B; ++b) {
        sb_session* s = bt->seq[b];
        if (!params[b] || !out_tokens[b]) return fail(SB_EINVAL, "batch_decode: NULL params / output of sequence %d", b);
        if ((rc = check_params(s, params[b]))) return rc;
        if (params[b]->w_max > bt->w_cap)
            return fail(SB_EINVAL, "batch_decode: w_max = %d exceeds the %d rows a sequence has in a batch of %d", params[b]->w_max,
                        bt->w_cap, B);
        if (!s->has_pending) return fail(SB_ESTATE, "batch_decode: sequence %d has no pending token (prefill first)", b);
        if (s->n_slots) return fail(SB_ESTATE, "batch_decode: sequence %d has an open round", b);
        if ((int64_t)s->c + max_new + params[b]->w_max > bt->m->cfg.max_seq)
            return fail(SB_ECAPACITY, "batch_decode: committed + max_new + w_max exceeds max_seq for sequence %d", b);
        if ((rc = join_head(s))) return rc;
    }
    std::vector<int> cnt(B, 0);
    std::vector<sb_verify_result> vres(B);
    const double t0 = now_ms();
    for (;;) {
        std::vector<int> act;
        for (int b = 0; b < B; ++b) {
            const sb_params* p = params[b];
            const bool eos = p->eos_id >= 0 && cnt[b] > 0 && out_tokens[b][cnt[b] - 1] == p->eos_id;
            if (cnt[b] < max_new && !eos) act.push_back(b);
        }
        if (act.empty()) break;
        if ((rc = batch_round(bt, act, params, vres.data()))) {
            if (rc == SB_EDEVICE)
                for (int b : act) (void)round_guard(bt->seq[b], rc);
            else
                for (int b : act) {   // refused before the device was touched for this sequence: drop the rows that were opened
                    sb_session* s = bt->seq[b];
                    s->draft_counter -= s->n_slots;
                    s->n_slots = 0; s->n_drafts = 0; s->round_closed = false; s->next_embedded = false;
                }
            return rc;
        }
        for (int b : act) {
            sb_session* s = bt->seq[b];
            const sb_params* p = params[b];
            const sb_verify_result& vr = vres[b];
            int take = 0;
            while (take < vr.n_emit && cnt[b] < max_new) {
                out_tokens[b][cnt[b]++] = vr.tokens[take++];
                if (p->eos_id >= 0 && out_tokens[b][cnt[b] - 1] == p->eos_id) break;
            }
            if (take < vr.n_emit) {
                s->c -= vr.n_emit - take;
                s->st.emitted -= vr.n_emit - take;
                s->pending = out_tokens[b][cnt[b] - 1];
            }
        }
    }
    const double ms = now_ms() - t0;
    for (int b = 0; b < B; ++b) { n_out[b] = cnt[b]; bt->seq[b]->st.decode_ms = ms; }
    return SB_OK;
}

}  // extern "C"
