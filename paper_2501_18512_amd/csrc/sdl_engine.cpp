// Host-side driver of Algorithm 2's outer-optimization schedule: at every inner step it
// issues the send-side and receive-side calls of the fragments that are due (Section 2.2:
// staggered fragments; Section 2.3: the result of a send is consumed tau steps later, with
// an optional different delay per worker, Section 3.3.2 on workers of unequal speed).
// Uses only the plan-level entry points of sdl.h; no device code here.
#include <algorithm>
#include <new>
#include <utility>
#include <vector>

#include "sdl.h"

struct sdl_engine {
    const sdl_plan_t* plan = nullptr;
    uint32_t P = 0, M = 0, H = 0;
    sdl_format_t fmt = SDL_FMT_E3M0;
    float lr = 0, mu = 0, alpha = 0;
    std::vector<uint32_t> offset;        // t_p
    std::vector<uint32_t> delay;         // tau_m per worker
    uint32_t delay_min = 0, delay_max = 0;
    // bound memory
    float* g = nullptr;
    float* mom = nullptr;
    std::vector<void*> w;                // M live replicas
    std::vector<void*> codes, scales;    // P*M message buffers (index p*M + m); unused when all delays are 0
    bool bound = false;
    // outer state in host memory: fragments are staged through `offload` (may be null)
    sdl_offload_t* offload = nullptr;
    void* copy_stream = nullptr;
    uint32_t lookahead = 0;
    // per fragment: step at which the message in flight was sent (0 = none), reduce done?, merged[m]
    std::vector<uint64_t> sent_at;
    std::vector<uint8_t> reduced;
    std::vector<uint8_t> merged;         // P*M
    std::vector<std::pair<uint64_t, uint32_t>> due;   // (next send step, fragment) of the prefetch candidates
    // optional diagnostics: cosine similarity of the outer gradients at every send
    bool track_cosine = false;
    std::vector<double*> cos_span_results;   // per fragment, may hold null pointers
    double* cos_fragment_results = nullptr;  // [P][2*M*M + 1]
    void* cos_workspace = nullptr;
    size_t cos_workspace_bytes = 0;
};

extern "C" {

int sdl_engine_create(const sdl_plan_t* plan, uint32_t H, uint32_t M, const uint32_t* tau_m, sdl_format_t fmt,
                      float lr, float mu, float alpha, sdl_engine_t** out)
{
    if (!plan || !out || !tau_m || M == 0 || M > SDL_MAX_WORKERS || H == 0) return SDL_ERR_INVALID_ARG;
    if (fmt < SDL_FMT_FP32 || fmt > SDL_FMT_E3M0_RN) return SDL_ERR_INVALID_ARG;
    for (uint32_t m = 0; m < M; ++m)
        if (tau_m[m] >= H) return SDL_ERR_INVALID_ARG;
    sdl_engine* e = nullptr;
    try {
        e = new sdl_engine();
        e->plan = plan; e->P = sdl_plan_num_fragments(plan); e->M = M; e->H = H; e->fmt = fmt;
        e->lr = lr; e->mu = mu; e->alpha = alpha;
        e->offset.resize(e->P);
        for (uint32_t p = 0; p < e->P; ++p) {
            int rc = sdl_plan_offset(plan, p, &e->offset[p]);
            if (rc != SDL_OK || e->offset[p] >= H) { delete e; return SDL_ERR_INVALID_ARG; }
        }
        e->delay.assign(tau_m, tau_m + M);
        e->delay_min = e->delay_max = tau_m[0];
        for (uint32_t m = 1; m < M; ++m) {
            if (tau_m[m] < e->delay_min) e->delay_min = tau_m[m];
            if (tau_m[m] > e->delay_max) e->delay_max = tau_m[m];
        }
        e->w.assign(M, nullptr);
        e->codes.assign((size_t)e->P * M, nullptr);
        e->scales.assign((size_t)e->P * M, nullptr);
        e->sent_at.assign(e->P, 0);
        e->reduced.assign(e->P, 0);
        e->merged.assign((size_t)e->P * M, 0);
        e->due.reserve(e->P);
    } catch (const std::bad_alloc&) {
        delete e;
        return SDL_ERR_NOMEM;
    }
    *out = e;
    return SDL_OK;
}

void sdl_engine_destroy(sdl_engine_t* e) { delete e; }

// The part of binding that does not depend on where the outer state lives.
static int bind_replicas_and_messages(sdl_engine* e, void* const* w_base, void* const* codes, void* const* scales)
{
    if (!w_base) return SDL_ERR_INVALID_ARG;
    // without any delay the fused call is used, which keeps the messages in registers; the
    // whole-span scale still needs its scale words (as workspace)
    const bool need_codes = e->delay_max > 0;
    const bool scaled = e->fmt >= SDL_FMT_E4M3;
    const bool need_scales = (need_codes && scaled) || e->fmt == SDL_FMT_E3M0_SPAN;
    if ((need_codes && !codes) || (need_scales && !scales)) return SDL_ERR_INVALID_ARG;
    for (uint32_t m = 0; m < e->M; ++m)
        if (!w_base[m]) return SDL_ERR_INVALID_ARG;
    for (size_t i = 0; i < (size_t)e->P * e->M; ++i)
        if ((need_codes && !codes[i]) || (need_scales && !scales[i])) return SDL_ERR_INVALID_ARG;
    for (uint32_t m = 0; m < e->M; ++m) e->w[m] = w_base[m];
    for (size_t i = 0; i < (size_t)e->P * e->M; ++i) {
        e->codes[i] = need_codes ? codes[i] : nullptr;
        e->scales[i] = need_scales ? scales[i] : nullptr;
    }
    return SDL_OK;
}

// Largest number of fragments that are between their send step and their last merge at the same
// inner step (at least 1: a fragment that is synchronised within one step still needs a slot).
static uint32_t slots_needed(const sdl_engine* e)
{
    uint32_t most = 1;
    for (uint32_t phase = 0; phase < e->H; ++phase) {
        uint32_t n = 0;
        for (uint32_t p = 0; p < e->P; ++p)
            if ((phase + e->H - e->offset[p]) % e->H <= e->delay_max) ++n;
        if (n > most) most = n;
    }
    return most;
}

int sdl_engine_bind(sdl_engine_t* e, float* g_base, float* mom_base, void* const* w_base, void* const* codes,
                    void* const* scales)
{
    if (!e || !g_base || !mom_base) return SDL_ERR_INVALID_ARG;
    int rc = bind_replicas_and_messages(e, w_base, codes, scales);
    if (rc != SDL_OK) return rc;
    e->g = g_base; e->mom = mom_base;
    e->offload = nullptr;
    e->bound = true;
    return SDL_OK;
}

int sdl_engine_bind_offload(sdl_engine_t* e, sdl_offload_t* offload, void* const* w_base, void* const* codes,
                            void* const* scales, void* copy_stream, uint32_t lookahead)
{
    if (!e || !offload) return SDL_ERR_INVALID_ARG;
    // a fragment holds its slot from its send step until its last worker has merged (delay_max steps
    // later): the pool must have a slot for every fragment that can be in that state at once
    if (sdl_offload_num_slots(offload) < slots_needed(e)) return SDL_ERR_INVALID_ARG;
    int rc = bind_replicas_and_messages(e, w_base, codes, scales);
    if (rc != SDL_OK) return rc;
    e->g = e->mom = nullptr;          // the outer state is reached through the staging pool only
    e->offload = offload;
    e->copy_stream = copy_stream;
    e->lookahead = lookahead;
    e->bound = true;
    return SDL_OK;
}

int sdl_engine_track_cosine(sdl_engine_t* e, double* const* span_results, double* fragment_results, void* workspace,
                            size_t workspace_bytes)
{
    if (!e) return SDL_ERR_INVALID_ARG;
    if (!fragment_results) {             // switch the diagnostics off
        e->track_cosine = false;
        return SDL_OK;
    }
    if (!workspace) return SDL_ERR_INVALID_ARG;
    size_t need = 0;
    for (uint32_t p = 0; p < e->P; ++p) {
        const sdl_span_t* spans = nullptr;
        uint32_t n_spans = 0;
        int rc = sdl_plan_fragment_spans(e->plan, p, &spans, &n_spans);
        if (rc != SDL_OK) return rc;
        const size_t bytes = sdl_cosine_workspace_bytes(e->M, n_spans);
        if (bytes > need) need = bytes;
    }
    if (workspace_bytes < need) return SDL_ERR_INVALID_ARG;
    try {
        e->cos_span_results.assign(e->P, nullptr);
    } catch (const std::bad_alloc&) {
        return SDL_ERR_NOMEM;
    }
    for (uint32_t p = 0; p < e->P && span_results; ++p) e->cos_span_results[p] = span_results[p];
    e->cos_fragment_results = fragment_results;
    e->cos_workspace = workspace;
    e->cos_workspace_bytes = workspace_bytes;
    e->track_cosine = true;
    return SDL_OK;
}

int sdl_engine_step(sdl_engine_t* e, uint64_t t, void* stream, uint32_t* n_sent, uint32_t* n_received)
{
    if (!e || !e->bound || t == 0) return SDL_ERR_INVALID_ARG;
    uint32_t sent = 0, received = 0;
    const uint32_t M = e->M;
    const bool staged = e->offload != nullptr;
    // everything that depends on the engine's own state is checked before the first launch, so that a
    // step that is refused has done nothing
    for (uint32_t p = 0; p < e->P; ++p) {
        const uint64_t s0 = e->offset[p];
        const bool sends = t > s0 && (t - s0) % e->H == 0;
        if (sends && e->sent_at[p] != 0) return SDL_ERR_INVALID_ARG;         // previous message not consumed: steps skipped
        if (sends && e->track_cosine && staged) return SDL_ERR_UNSUPPORTED;
        if (e->sent_at[p] != 0) {
            const uint64_t ts = e->sent_at[p];
            if (!e->reduced[p] && t > ts + e->delay_min) return SDL_ERR_INVALID_ARG;   // the receive step was skipped
            if (t > ts + e->delay_max) return SDL_ERR_INVALID_ARG;                   // a merge step was skipped
        }
    }
    for (uint32_t p = 0; p < e->P; ++p) {
        void* const* codes = e->codes.data() + (size_t)p * M;
        void* const* scales = e->scales.data() + (size_t)p * M;
        float* g = e->g;
        float* mom = e->mom;
        // ---- send side: t = t_p + k*H, k >= 1
        const uint64_t s0 = e->offset[p];
        const bool sends = t > s0 && (t - s0) % e->H == 0;
        if (staged && (sends || e->sent_at[p] != 0)) {
            // outer state of this fragment comes from its staging slot (copied in on demand if
            // it was not prefetched); the compute stream waits for the copy
            int rc = sdl_offload_acquire(e->offload, p, stream, e->copy_stream, &g, &mom);
            if (rc != SDL_OK) return rc;
        }
        if (sends) {
            if (e->track_cosine) {
                // the outer gradients that are about to be sent, before anything is updated
                int rc = sdl_outer_grad_cosine_plan(e->plan, p, g, e->w.data(), M, e->cos_span_results[p],
                                                    e->cos_fragment_results + (size_t)p * SDL_COSINE_RESULT_DOUBLES(M),
                                                    e->cos_workspace, e->cos_workspace_bytes, stream);
                if (rc != SDL_OK) return rc;
            }
            if (e->delay_max == 0) {
                // no overlap anywhere: the whole outer step at once, messages kept in registers (the
                // whole-span scale uses the fragment's scale words as workspace)
                void* const* work = e->fmt == SDL_FMT_E3M0_SPAN ? scales : nullptr;
                int rc = staged ? sdl_fragment_outer_step_staged_ex(e->plan, p, g, mom, e->w.data(), e->w.data(), M,
                                                                    e->fmt, e->lr, e->mu, e->alpha, nullptr, work, stream)
                                : sdl_fragment_outer_step_plan_ex(e->plan, p, g, mom, e->w.data(), e->w.data(), M,
                                                                  e->fmt, e->lr, e->mu, e->alpha, nullptr, work, stream);
                if (rc != SDL_OK) return rc;
                if (staged) {
                    rc = sdl_offload_release(e->offload, p, stream, e->copy_stream);
                    if (rc != SDL_OK) return rc;
                }
                ++sent; ++received;
                continue;
            }
            int rc = staged ? sdl_quantize_outer_grad_staged(e->plan, p, g, e->w.data(), M, e->fmt, codes, scales, stream)
                            : sdl_quantize_outer_grad_plan(e->plan, p, g, e->w.data(), M, e->fmt, codes, scales, stream);
            if (rc != SDL_OK) return rc;
            e->sent_at[p] = t;
            e->reduced[p] = 0;
            for (uint32_t m = 0; m < M; ++m) e->merged[(size_t)p * M + m] = 0;
            ++sent;
        }
        // ---- receive side of the message in flight
        if (e->sent_at[p] != 0) {
            const uint64_t ts = e->sent_at[p];
            if (!e->reduced[p] && t == ts + e->delay_min && e->delay_min == e->delay_max) {
                // one common delay: mean, Nesterov and the merge of every replica in a single pass
                int rc = staged ? sdl_receive_outer_step_staged(e->plan, p, g, mom, codes, scales, e->w.data(), M,
                                                                e->fmt, e->lr, e->mu, e->alpha, stream)
                                : sdl_receive_outer_step_plan(e->plan, p, g, mom, codes, scales, e->w.data(), M,
                                                              e->fmt, e->lr, e->mu, e->alpha, stream);
                if (rc != SDL_OK) return rc;
                e->reduced[p] = 1;
                for (uint32_t m = 0; m < M; ++m) e->merged[(size_t)p * M + m] = 1;
                ++received;
            }
            if (!e->reduced[p] && t == ts + e->delay_min) {
                int rc = staged ? sdl_dequant_reduce_nesterov_staged(e->plan, p, g, mom, codes, scales, M, e->fmt,
                                                                     e->lr, e->mu, stream)
                                : sdl_dequant_reduce_nesterov_plan(e->plan, p, g, mom, codes, scales, M, e->fmt,
                                                                   e->lr, e->mu, stream);
                if (rc != SDL_OK) return rc;
                e->reduced[p] = 1;
                ++received;
            }
            // merge into every worker whose delay expires now (one launch for all of them)
            void* due[SDL_MAX_WORKERS];
            uint32_t n_due = 0, n_done = 0;
            for (uint32_t m = 0; m < M; ++m) {
                uint8_t& done = e->merged[(size_t)p * M + m];
                if (!done && t == ts + e->delay[m]) { due[n_due++] = e->w[m]; done = 1; }
                n_done += done;
            }
            if (n_due) {
                int rc = staged ? sdl_merge_overlap_staged(e->plan, p, g, due, n_due, e->alpha, stream)
                                : sdl_merge_overlap_plan(e->plan, p, g, due, n_due, e->alpha, stream);
                if (rc != SDL_OK) return rc;
            }
            if (n_done == M) {
                e->sent_at[p] = 0;
                if (staged) {
                    // synchronisation of this fragment is complete: write its outer state back
                    int rc = sdl_offload_release(e->offload, p, stream, e->copy_stream);
                    if (rc != SDL_OK) return rc;
                }
            }
        }
    }
    if (staged && e->lookahead > 0) {
        // the schedule is known in advance: start copying in the fragments that send within the next
        // `lookahead` steps, the one that is due first first.  A full pool ends the round: a fragment
        // that could not be prefetched is copied in when it is due, where a copy that was prefetched
        // too early and not used yet gives way to it.
        e->due.clear();                           // capacity P since creation: no allocation here
        for (uint32_t p = 0; p < e->P; ++p) {
            if (e->sent_at[p] != 0) continue;
            const uint64_t s0 = e->offset[p];
            const uint64_t k = t >= s0 ? (t - s0) / e->H + 1 : 1;     // next send strictly after t
            const uint64_t next = s0 + k * e->H;
            if (next - t <= e->lookahead) e->due.push_back(std::make_pair(next, p));
        }
        std::sort(e->due.begin(), e->due.end());
        for (const auto& d : e->due) {
            const int rc = sdl_offload_prefetch(e->offload, d.second, e->copy_stream);
            if (rc == SDL_ERR_NOMEM) break;
            if (rc != SDL_OK) return rc;
        }
    }
    if (n_sent) *n_sent = sent;
    if (n_received) *n_received = received;
    return SDL_OK;
}

}  // extern "C"
