// Host side of the library: fragment map, span / run tables and the send / receive
// schedule of Streaming DiLoCo (Section 2.2 and Algorithm 2 of the paper).  Pure
// integer work, no device code.
#include <cstdlib>
#include <new>
#include <vector>

#include "sdl.h"

struct sdl_plan {
    uint32_t P = 0, H = 0, tau = 0, n_blocks = 0;
    uint64_t total = 0;
    std::vector<uint32_t> offset;                  // t_p
    std::vector<uint32_t> block_owner;             // fragment of each transformer block
    std::vector<std::vector<sdl_span_t>> spans;    // per fragment, model order
    std::vector<std::vector<sdl_span_t>> runs;     // per fragment, joined spans
};

namespace {

// Fragment of block i.  Strided: round robin.  Sequential: fragment p starts at block
// floor(p*L/P); the owner of block i is the last fragment whose start is <= i, which is
// floor((i*P + P - 1) / L).
uint32_t owner_of_block(uint32_t i, uint32_t L, uint32_t P, sdl_pattern_t pattern)
{
    if (pattern == SDL_PATTERN_STRIDED) return i % P;
    return (uint32_t)(((uint64_t)i * P + P - 1) / L);
}

// Join neighbouring spans into runs.  A span may be appended to the current run only
// if it starts where the run ends and the run's length so far is a multiple of the
// largest scale-block size (128), so that block boundaries counted from the run start
// coincide with those counted from each span start for every block-scaled format.
std::vector<sdl_span_t> join_spans(const std::vector<sdl_span_t>& spans)
{
    std::vector<sdl_span_t> runs;
    for (const sdl_span_t& s : spans) {
        if (s.numel == 0) continue;
        if (!runs.empty()) {
            sdl_span_t& r = runs.back();
            if (r.offset + r.numel == s.offset && r.numel % SDL_MAX_BLOCK == 0) {
                r.numel += s.numel;
                continue;
            }
        }
        runs.push_back(s);
    }
    return runs;
}

}  // namespace

extern "C" {

int sdl_fragment_plan(const uint64_t* unit_numel, const int32_t* unit_block, uint32_t n_units,
                      uint32_t n_blocks, uint32_t P, sdl_pattern_t pattern, uint32_t H, uint32_t tau,
                      const uint32_t* t_p, sdl_plan_t** out)
{
    return sdl_fragment_plan_ex(unit_numel, unit_block, n_units, n_blocks, P, pattern, H, tau, t_p, 0u, out);
}

int sdl_fragment_plan_ex(const uint64_t* unit_numel, const int32_t* unit_block, uint32_t n_units,
                         uint32_t n_blocks, uint32_t P, sdl_pattern_t pattern, uint32_t H, uint32_t tau,
                         const uint32_t* t_p, uint32_t flags, sdl_plan_t** out)
{
    if (!out || (n_units && (!unit_numel || !unit_block))) return SDL_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)(SDL_PLAN_PRE_OWN_FRAGMENT | SDL_PLAN_ALIGN_GROUPS)) return SDL_ERR_INVALID_ARG;
    // with the flag, fragment 0 holds the SDL_UNIT_PRE groups alone and the blocks use 1..P
    const uint32_t shift = (flags & SDL_PLAN_PRE_OWN_FRAGMENT) ? 1u : 0u;
    const uint32_t n_frag = P + shift;
    if (P == 0 || n_blocks == 0 || P > n_blocks || H == 0 || tau >= H) return SDL_ERR_INVALID_ARG;
    if (pattern != SDL_PATTERN_STRIDED && pattern != SDL_PATTERN_SEQUENTIAL) return SDL_ERR_INVALID_ARG;
    for (uint32_t u = 0; u < n_units; ++u) {
        int32_t b = unit_block[u];
        if (b != SDL_UNIT_PRE && b != SDL_UNIT_POST && (b < 0 || (uint32_t)b >= n_blocks))
            return SDL_ERR_INVALID_ARG;
    }
    if (t_p)
        for (uint32_t p = 0; p < n_frag; ++p)
            if (t_p[p] >= H) return SDL_ERR_INVALID_ARG;

    sdl_plan* plan = nullptr;
    try {
        plan = new sdl_plan();
        plan->P = n_frag; plan->H = H; plan->tau = tau; plan->n_blocks = n_blocks;
        plan->offset.resize(n_frag);
        for (uint32_t p = 0; p < n_frag; ++p)
            plan->offset[p] = t_p ? t_p[p] : (uint32_t)(((uint64_t)p * H) / n_frag);
        plan->block_owner.resize(n_blocks);
        for (uint32_t i = 0; i < n_blocks; ++i)
            plan->block_owner[i] = shift + owner_of_block(i, n_blocks, P, pattern);
        plan->spans.resize(n_frag);
        uint64_t pos = 0;
        for (uint32_t u = 0; u < n_units; ++u) {
            int32_t b = unit_block[u];
            uint32_t owner;
            if (b == SDL_UNIT_PRE) owner = shift ? 0u : plan->block_owner[0];
            else if (b == SDL_UNIT_POST) owner = plan->block_owner[n_blocks - 1];
            else owner = plan->block_owner[(uint32_t)b];
            if (flags & SDL_PLAN_ALIGN_GROUPS)
                pos = (pos + SDL_PLAN_GROUP_ALIGN - 1) / SDL_PLAN_GROUP_ALIGN * SDL_PLAN_GROUP_ALIGN;
            sdl_span_t s;
            s.offset = pos; s.numel = unit_numel[u]; s.unit = (int32_t)u;
            plan->spans[owner].push_back(s);
            pos += unit_numel[u];
        }
        plan->total = pos;
        plan->runs.resize(n_frag);
        for (uint32_t p = 0; p < n_frag; ++p) plan->runs[p] = join_spans(plan->spans[p]);
    } catch (const std::bad_alloc&) {
        delete plan;
        return SDL_ERR_NOMEM;
    }
    *out = plan;
    return SDL_OK;
}

void sdl_plan_destroy(sdl_plan_t* plan) { delete plan; }

uint32_t sdl_plan_num_fragments(const sdl_plan_t* plan) { return plan ? plan->P : 0; }
uint64_t sdl_plan_total_numel(const sdl_plan_t* plan) { return plan ? plan->total : 0; }

int sdl_plan_block_fragment(const sdl_plan_t* plan, uint32_t block)
{
    if (!plan || block >= plan->n_blocks) return SDL_ERR_INVALID_ARG;
    return (int)plan->block_owner[block];
}

int sdl_plan_fragment_spans(const sdl_plan_t* plan, uint32_t p, const sdl_span_t** spans,
                            uint32_t* n_spans)
{
    if (!plan || p >= plan->P || !spans || !n_spans) return SDL_ERR_INVALID_ARG;
    *spans = plan->spans[p].data();
    *n_spans = (uint32_t)plan->spans[p].size();
    return SDL_OK;
}

int sdl_plan_fragment_runs(const sdl_plan_t* plan, uint32_t p, const sdl_span_t** runs,
                           uint32_t* n_runs)
{
    if (!plan || p >= plan->P || !runs || !n_runs) return SDL_ERR_INVALID_ARG;
    *runs = plan->runs[p].data();
    *n_runs = (uint32_t)plan->runs[p].size();
    return SDL_OK;
}

int sdl_plan_offset(const sdl_plan_t* plan, uint32_t p, uint32_t* t_p)
{
    if (!plan || p >= plan->P || !t_p) return SDL_ERR_INVALID_ARG;
    *t_p = plan->offset[p];
    return SDL_OK;
}

int sdl_plan_events(const sdl_plan_t* plan, uint64_t t, uint32_t* send, uint32_t* n_send,
                    uint32_t* recv, uint32_t* n_recv)
{
    if (!plan || (send && !n_send) || (recv && !n_recv)) return SDL_ERR_INVALID_ARG;
    uint32_t ns = 0, nr = 0;
    for (uint32_t p = 0; p < plan->P; ++p) {
        // send at t_p + k*H, receive tau later, k >= 1: the step must lie strictly
        // after the offset (plus tau) and a whole number of periods away from it
        uint64_t s0 = plan->offset[p], r0 = s0 + plan->tau;
        if (t > s0 && (t - s0) % plan->H == 0) { if (send) send[ns] = p; ++ns; }
        if (t > r0 && (t - r0) % plan->H == 0) { if (recv) recv[nr] = p; ++nr; }
    }
    if (n_send) *n_send = ns;
    if (n_recv) *n_recv = nr;
    return SDL_OK;
}

size_t sdl_exchange_bytes(sdl_format_t fmt, uint64_t numel, size_t* code_bytes, size_t* scale_bytes)
{
    size_t c = 0, s = 0;
    const size_t blocks = (size_t)((numel + SDL_BLOCK - 1) / SDL_BLOCK);
    switch (fmt) {
    case SDL_FMT_FP32: c = (size_t)numel * 4; break;
    case SDL_FMT_BF16: c = (size_t)numel * 2; break;
    case SDL_FMT_E4M3: c = (size_t)numel; s = blocks; break;
    case SDL_FMT_E3M0: case SDL_FMT_E3M0_RN: c = (size_t)((numel + 1) / 2); s = blocks; break;
    case SDL_FMT_E3M0_B64: c = (size_t)((numel + 1) / 2); s = (size_t)((numel + 63) / 64); break;
    case SDL_FMT_E3M0_B128: c = (size_t)((numel + 1) / 2); s = (size_t)((numel + 127) / 128); break;
    case SDL_FMT_E3M0_SPAN: c = (size_t)((numel + 1) / 2); s = numel ? 4 : 0; break;
    default: break;
    }
    if (code_bytes) *code_bytes = c;
    if (scale_bytes) *scale_bytes = s;
    return c + s;
}

int sdl_flat_layout(uint64_t total_numel, uint32_t M, int separate_w_now, uint64_t* offsets, uint64_t* total_bytes)
{
    if (!offsets || !total_bytes || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const uint32_t n_arrays = 2u + (separate_w_now ? 2u : 1u) * M;
    uint64_t slot = 0;       // start of the next 2 MiB-aligned slot
    for (uint32_t k = 0; k < n_arrays; ++k) {
        const uint64_t bytes = total_numel * (k < 2 ? 4u : 2u);
        offsets[k] = slot + (uint64_t)k * SDL_LAYOUT_STAGGER;
        const uint64_t end = offsets[k] + bytes;
        slot = (end + SDL_LAYOUT_SLOT_ALIGN - 1) / SDL_LAYOUT_SLOT_ALIGN * SDL_LAYOUT_SLOT_ALIGN;
    }
    *total_bytes = slot;
    return SDL_OK;
}

const char* sdl_status_string(int status)
{
    switch (status) {
    case SDL_OK: return "ok";
    case SDL_ERR_INVALID_ARG: return "invalid argument";
    case SDL_ERR_UNSUPPORTED: return "unsupported";
    case SDL_ERR_ALIGNMENT: return "pointer not aligned to its element type";
    case SDL_ERR_DEVICE: return "HIP error at kernel launch";
    case SDL_ERR_NOMEM: return "out of host memory or staging slots";
    case SDL_ERR_TOO_LARGE: return "input exceeds the fixed capacity of the allocation-free entry point";
    default: return "unknown status";
    }
}

}  // extern "C"
