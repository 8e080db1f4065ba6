// Outer parameters and Nesterov state kept in host memory (Section 2.5 of the paper:
// only the fragment that is being synchronised needs its outer parameters and outer
// optimizer state in HBM, two words per parameter of the fragment, and since the schedule is
// known in advance the transfer can start early).  This file stages fragments between
// pinned host arrays and a small pool of device slots with asynchronous copies on a
// stream of their own, ordered against the compute stream with events.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "sdl.h"

namespace {
constexpr uint64_t kTile = 512;    // staged runs are padded to multiples of 512 elements (whole kernel tiles)
uint64_t pad_tile(uint64_t n) { return (n + kTile - 1) / kTile * kTile; }
}  // namespace

struct sdl_offload {
    struct Slot {
        float* g = nullptr;
        float* mom = nullptr;
        int frag = -1;               // fragment that lives here, -1 = free
        bool in_use = false;         // handed out by acquire (it may hold updates): only release frees it
        hipEvent_t ready = nullptr;  // host-to-device copy finished
        hipEvent_t done = nullptr;   // compute on the slot finished
    };
    const sdl_plan_t* plan = nullptr;
    uint32_t P = 0;
    float* g_host = nullptr;
    float* mom_host = nullptr;
    uint64_t slot_numel = 0;
    std::vector<Slot> slots;
    std::vector<int> slot_of;        // per fragment: slot index or -1
    bool bound = false;
};

extern "C" {

int sdl_offload_create(const sdl_plan_t* plan, uint32_t n_slots, sdl_offload_t** out)
{
    if (!plan || !out || n_slots == 0) return SDL_ERR_INVALID_ARG;
    sdl_offload* o = nullptr;
    try {
        o = new sdl_offload();
        o->plan = plan;
        o->P = sdl_plan_num_fragments(plan);
        o->slots.resize(n_slots);
        o->slot_of.assign(o->P, -1);
        for (uint32_t p = 0; p < o->P; ++p) {
            const uint64_t n = sdl_plan_staged_numel(plan, p);
            if (n > o->slot_numel) o->slot_numel = n;
        }
    } catch (const std::bad_alloc&) {
        delete o;
        return SDL_ERR_NOMEM;
    }
    for (auto& s : o->slots) {
        if (hipEventCreateWithFlags(&s.ready, hipEventDisableTiming) != hipSuccess ||
            hipEventCreateWithFlags(&s.done, hipEventDisableTiming) != hipSuccess) {
            sdl_offload_destroy(o);
            return SDL_ERR_DEVICE;
        }
    }
    *out = o;
    return SDL_OK;
}

void sdl_offload_destroy(sdl_offload_t* o)
{
    if (!o) return;
    for (auto& s : o->slots) {
        if (s.ready) (void)hipEventDestroy(s.ready);
        if (s.done) (void)hipEventDestroy(s.done);
    }
    delete o;
}

uint64_t sdl_offload_slot_numel(const sdl_offload_t* o) { return o ? o->slot_numel : 0; }
uint32_t sdl_offload_num_slots(const sdl_offload_t* o) { return o ? (uint32_t)o->slots.size() : 0; }

int sdl_offload_bind(sdl_offload_t* o, float* g_host, float* mom_host, float* const* slot_g, float* const* slot_mom)
{
    if (!o || !g_host || !mom_host || !slot_g || !slot_mom) return SDL_ERR_INVALID_ARG;
    for (size_t i = 0; i < o->slots.size(); ++i) {
        if (!slot_g[i] || !slot_mom[i]) return SDL_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(slot_g[i]) % 16 || reinterpret_cast<uintptr_t>(slot_mom[i]) % 16)
            return SDL_ERR_ALIGNMENT;
    }
    for (size_t i = 0; i < o->slots.size(); ++i) {
        if (o->slots[i].frag >= 0) return SDL_ERR_INVALID_ARG;     // rebinding while fragments are staged
        o->slots[i].g = slot_g[i];
        o->slots[i].mom = slot_mom[i];
    }
    o->g_host = g_host;
    o->mom_host = mom_host;
    o->bound = true;
    return SDL_OK;
}

int sdl_offload_resident(const sdl_offload_t* o, uint32_t p)
{
    if (!o || p >= o->P) return SDL_ERR_INVALID_ARG;
    return o->slot_of[p] >= 0 ? 1 : 0;
}

// Copies every run of fragment p between the host arrays (flat model layout) and a slot
// (runs back to back, each padded to whole tiles).
static int copy_fragment(sdl_offload* o, uint32_t p, sdl_offload::Slot& s, bool to_device, hipStream_t stream)
{
    const sdl_span_t* runs = nullptr;
    uint32_t n_runs = 0;
    int rc = sdl_plan_fragment_runs(o->plan, p, &runs, &n_runs);
    if (rc != SDL_OK) return rc;
    uint64_t off = 0;
    for (uint32_t i = 0; i < n_runs; ++i) {
        const size_t bytes = (size_t)runs[i].numel * sizeof(float);
        hipError_t e1, e2;
        if (to_device) {
            e1 = hipMemcpyAsync(s.g + off, o->g_host + runs[i].offset, bytes, hipMemcpyHostToDevice, stream);
            e2 = hipMemcpyAsync(s.mom + off, o->mom_host + runs[i].offset, bytes, hipMemcpyHostToDevice, stream);
        } else {
            e1 = hipMemcpyAsync(o->g_host + runs[i].offset, s.g + off, bytes, hipMemcpyDeviceToHost, stream);
            e2 = hipMemcpyAsync(o->mom_host + runs[i].offset, s.mom + off, bytes, hipMemcpyDeviceToHost, stream);
        }
        if (e1 != hipSuccess || e2 != hipSuccess) return SDL_ERR_DEVICE;
        off += pad_tile(runs[i].numel);
    }
    return SDL_OK;
}

// Starts the copy-in of fragment p into slot `slot` (free, or holding a fragment that was only prefetched).
static int stage_into(sdl_offload* o, uint32_t p, int slot, void* copy_stream)
{
    sdl_offload::Slot& s = o->slots[slot];
    if (s.frag >= 0) o->slot_of[s.frag] = -1;      // a prefetched copy that nobody used: dropped, the host arrays are current
    s.frag = -1;
    // the write-back of the slot's previous tenant and any earlier copy-in were queued on the same
    // copy stream, so this copy cannot overtake them
    int rc = copy_fragment(o, p, s, true, (hipStream_t)copy_stream);
    if (rc != SDL_OK) return rc;
    if (hipEventRecord(s.ready, (hipStream_t)copy_stream) != hipSuccess) return SDL_ERR_DEVICE;
    s.frag = (int)p;
    s.in_use = false;
    o->slot_of[p] = slot;
    return SDL_OK;
}

int sdl_offload_prefetch(sdl_offload_t* o, uint32_t p, void* copy_stream)
{
    if (!o || !o->bound || p >= o->P) return SDL_ERR_INVALID_ARG;
    if (o->slot_of[p] >= 0) return SDL_OK;
    for (size_t i = 0; i < o->slots.size(); ++i)
        if (o->slots[i].frag < 0) return stage_into(o, p, (int)i, copy_stream);
    return SDL_ERR_NOMEM;
}

int sdl_offload_acquire(sdl_offload_t* o, uint32_t p, void* compute_stream, void* copy_stream, float** g_frag,
                        float** mom_frag)
{
    if (!o || !o->bound || p >= o->P || !g_frag || !mom_frag) return SDL_ERR_INVALID_ARG;
    if (o->slot_of[p] < 0) {
        // a free slot, else the slot of a fragment that was prefetched but not acquired yet: its
        // copy holds nothing the host arrays do not, so it can give way to a fragment that is due now
        int slot = -1;
        for (size_t i = 0; i < o->slots.size() && slot < 0; ++i)
            if (o->slots[i].frag < 0) slot = (int)i;
        for (size_t i = 0; i < o->slots.size() && slot < 0; ++i)
            if (!o->slots[i].in_use) slot = (int)i;
        if (slot < 0) return SDL_ERR_NOMEM;
        int rc = stage_into(o, p, slot, copy_stream);
        if (rc != SDL_OK) return rc;
    }
    sdl_offload::Slot& s = o->slots[o->slot_of[p]];
    if (hipStreamWaitEvent((hipStream_t)compute_stream, s.ready, 0) != hipSuccess) return SDL_ERR_DEVICE;
    s.in_use = true;
    *g_frag = s.g;
    *mom_frag = s.mom;
    return SDL_OK;
}

static int write_back(sdl_offload* o, uint32_t p, void* compute_stream, void* copy_stream)
{
    sdl_offload::Slot& s = o->slots[o->slot_of[p]];
    if (hipEventRecord(s.done, (hipStream_t)compute_stream) != hipSuccess) return SDL_ERR_DEVICE;
    if (hipStreamWaitEvent((hipStream_t)copy_stream, s.done, 0) != hipSuccess) return SDL_ERR_DEVICE;
    return copy_fragment(o, p, s, false, (hipStream_t)copy_stream);
}

int sdl_offload_release(sdl_offload_t* o, uint32_t p, void* compute_stream, void* copy_stream)
{
    if (!o || !o->bound || p >= o->P || o->slot_of[p] < 0) return SDL_ERR_INVALID_ARG;
    int rc = write_back(o, p, compute_stream, copy_stream);
    if (rc != SDL_OK) return rc;
    o->slots[o->slot_of[p]].frag = -1;
    o->slots[o->slot_of[p]].in_use = false;
    o->slot_of[p] = -1;
    return SDL_OK;
}

int sdl_offload_flush(sdl_offload_t* o, void* compute_stream, void* copy_stream)
{
    if (!o || !o->bound) return SDL_ERR_INVALID_ARG;
    for (uint32_t p = 0; p < o->P; ++p) {
        if (o->slot_of[p] < 0) continue;
        int rc = write_back(o, p, compute_stream, copy_stream);
        if (rc != SDL_OK) return rc;
    }
    return SDL_OK;
}

}  // extern "C"
