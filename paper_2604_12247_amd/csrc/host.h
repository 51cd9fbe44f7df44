// Internals shared by the host-side sources of libspecbound (specbound.cpp: configuration, model
// and session life cycle, the single-sequence rounds and their C ABI; batch.cpp: rounds of several
// sequences side by side; ops.cpp: the single-kernel entry points).  Not part of the boundary.
#pragma once
#include <cstdarg>
#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

#include "kernels.h"

namespace sbhost {

// Message of the calling thread's last failure (sb_last_error).
extern thread_local std::string g_err;
int fail(int code, const char* fmt, ...);

#define HIP_TRY(expr)                                                                                  \
    do {                                                                                               \
        hipError_t e_ = (expr);                                                                        \
        if (e_ != hipSuccess) return sbhost::fail(SB_EDEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

double now_ms();
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t esize(int dtype) { return dtype == SB_BF16 ? 2 : 4; }

struct WsLayout {
    size_t H, xn, xs_attn, xs_ffn, xs_exit, xs_exit2, ssq_exit, ssq_attn, ssq_ffn, qkv, att, atts, u, us, attn_part, head_part,
        logits_exit, logits_final, sample_w, round, table, total;
    int max_chunks, head_blocks, n_pages, ssq_ld;
    // prompt passes of SB_PREFILL_ROWS rows (packed bf16 weights only)
    bool prefill_gemm;
    size_t p_tok, p_H, p_xs, p_ssq, p_qkv, p_atts, p_us, p_part, p_attn_part;
    int p_ssq_ld, p_rows;
};

}  // namespace sbhost

struct sb_model {
    sb_config cfg;
    const void *embed, *lm_head;
    const float* final_norm;
    std::vector<const float*> attn_norm, ffn_norm, exit_norm;
    std::vector<const void*> w_qkv, w_o, w_gate_up, w_down, exit_head;
    hipStream_t stream;
    float *rope_cos, *rope_sin;
    int proj;      // SB_PROJ_VALU or SB_PROJ_MFMA (row-major or packed, see `packed`)
    bool packed;   // the projection pointers below name tile-packed copies owned by the model
    std::vector<void*> owned;  // device allocations to free
    int64_t layer_bytes, head_bytes;
};

struct sb_session {
    sb_model* m;
    char* ws;
    sbhost::WsLayout L;
    sb::KvLayout kv;
    sb::DevRound* d_round;
    sb::DevRound* h_round;  // pinned host copy
    // Exit decisions that gate the host's next launch (computed exits) arrive without a copy: the
    // head merge writes them into this mapped host memory, the host polls the sequence number.
    int32_t* note_h;
    int32_t* note_d;    // the same memory as the device addresses it
    int32_t note_seq;
    int32_t c, pending;
    bool has_pending;
    int n_slots, n_drafts;
    int reached[SB_MAX_W], exit_layer[SB_MAX_W];
    int32_t draft_host[SB_MAX_W];  // drafted id if the host knows it, else -1
    bool round_closed;
    bool next_embedded;  // the last draft step's head merge has already embedded the next row
    int fail_countdown;  // test tap: the n-th projection launch from now reports a failure
    int64_t* phase_bytes;  // where run_layer / run_head account their bytes (a field of st), or null
    int64_t draft_counter;
    bool debug;
    sb_stats st;
    // Exit heads run on a second stream next to the following layer when the exit
    // layer is known in advance (forced schedules): events order the two streams.
    hipStream_t head_stream;
    hipEvent_t ev_main[4], ev_head[4];
    unsigned ev_i;
    // What W_down leaves for an exit head (the row's bf16 parts with the exit norm's gains, its sums
    // of squares) goes to one of two buffers, by layer parity: the head of layer l on the head stream
    // may still be reading its buffer while W_down of layer l + 1 writes the other one.
    bool head_pending[2];   // a head on the head stream reads buffer b; ev_head[head_pending_ev[b]] marks its end
    int head_pending_ev[2];
    // phase timing: events at the boundaries of a round's phases (sb_phase_timing)
    bool phase_timing;
    hipEvent_t ev_ph[5];
    // per-kernel event timing
    uint32_t prof_mask;
    int prof_every;                    // time every n-th launch of a class
    int64_t prof_seen[SB_K_COUNT];
    std::vector<hipEvent_t> prof_ev;   // pairs
    std::vector<hipEvent_t> prof_cal;  // empty pairs (calibration)
    std::vector<int> prof_cls;
    std::vector<int64_t> prof_bytes;
    size_t prof_used;                  // pairs used
};

// Several sequences decoded together (Sec. 4.3 evaluates batch 1; this is the batch > 1 form of
// the same rounds): the rows of all sequences share every sweep over a layer's or a head's
// weights, each sequence keeps its own KV cache and its own round.  Sequence b owns the rows
// (slots) b * w_cap .. b * w_cap + w_cap - 1 of the first session's hidden cache.
struct sb_batch {
    sb_model* m;
    int B, w_cap;
    std::vector<sb_session*> seq;
};

namespace sbhost {

template <typename T>
T* wsp(sb_session* s, size_t off) { return reinterpret_cast<T*>(s->ws + off); }

int check_params(const sb_session* s, const sb_params* p);
int join_head(sb_session* s);              // the main stream waits for every head still running on the head stream
int round_guard(sb_session* s, int rc);
int gemv(sb_session* s, sb::GemvArgs& a, int cls, hipStream_t st);

// Event pair around the launches of one kernel class, when that class is timed.
struct ProfScope {
    sb_session* s;
    hipStream_t st;
    long idx;
    ProfScope(sb_session* s_, int cls, int64_t bytes, hipStream_t st_) : s(s_), st(st_), idx(-1) {
        if (!(s->prof_mask & (1u << cls)) || s->prof_used * 2 + 2 > s->prof_ev.size()) return;
        if (s->prof_seen[cls]++ % s->prof_every) return;
        idx = (long)s->prof_used++;
        s->prof_cls[idx] = cls;
        s->prof_bytes[idx] = bytes;
        (void)hipEventRecord(s->prof_ev[2 * idx], st);
    }
    ~ProfScope() {
        if (idx >= 0) (void)hipEventRecord(s->prof_ev[2 * idx + 1], st);
    }
};

}  // namespace sbhost
