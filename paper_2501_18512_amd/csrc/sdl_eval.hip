// Parameters handed to evaluation (Appendix of the paper, "Which parameters to evaluate"): the
// first replica, the fp32 average of all replicas, or the outer parameters, written in the
// model's storage type (bf16).  One streaming pass for gfx950: a workgroup is one 64-lane
// wavefront and owns a tile of 512 consecutive parameters; lane l reads and writes the eight
// parameters [8l, 8l+8) -- one 128-bit access per bf16 array, two per fp32 array, non-temporal.
// Whole tiles of arrays that start at any other element go through 128-bit accesses of element
// alignment, ragged tails element by element under the buffer range check.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "sdl.h"
#include "sdl_device.h"

namespace {

using namespace sdl_device;

constexpr int kLaneElems = 8;
constexpr int kTile = kLaneElems * kWave;

struct EvalArgs {
    const float* g;
    const uint16_t* w[SDL_MAX_WORKERS];
    uint16_t* out;
    uint64_t numel;
    uint32_t M;
    uint32_t which;
    uint32_t fast;       // every array that is touched is 16-byte aligned
};

// two fp32 -> two bf16 (round to nearest even) in one 32-bit word, first value in the low half
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi)
{
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// The lane's 8 bf16 of one array as 4 words (element 2k in the low half of word k): a 128-bit
// buffer access in a whole tile when every array is 16-byte aligned, a 128-bit access of element
// alignment in a whole tile otherwise, element by element under the buffer range check in a ragged
// last tile.
__device__ __forceinline__ u32x4 load_bf16x8(const uint16_t* p, uint64_t e0, uint32_t valid, bool fast, uint32_t lane)
{
    if (fast && valid == (uint32_t)kTile)
        return __builtin_amdgcn_raw_buffer_load_b128(rsrc(p + e0, kTile * 2), (int)(lane * 16), 0, 2);
    if (valid == (uint32_t)kTile)
        return __builtin_nontemporal_load(reinterpret_cast<const u32x4_bf16elem*>(p + e0 + lane * kLaneElems));
    const __amdgpu_buffer_rsrc_t r = rsrc(p + e0, valid * 2);
    uint32_t h[kLaneElems];
#pragma unroll
    for (int j = 0; j < kLaneElems; ++j)
        h[j] = (uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r, (int)((lane * kLaneElems + j) * 2), 0, 0) & 0xffffu;
    return u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
}

__device__ __forceinline__ void store_bf16x8(uint16_t* p, uint64_t e0, uint32_t valid, bool fast, uint32_t lane,
                                             const u32x4& x)
{
    if (fast && valid == (uint32_t)kTile) {
        __builtin_amdgcn_raw_buffer_store_b128(x, rsrc(p + e0, kTile * 2), (int)(lane * 16), 0, 2);
        return;
    }
    if (valid == (uint32_t)kTile) {
        __builtin_nontemporal_store(u32x4_bf16elem{x.x, x.y, x.z, x.w},
                                    reinterpret_cast<u32x4_bf16elem*>(p + e0 + lane * kLaneElems));
        return;
    }
    const __amdgpu_buffer_rsrc_t r = rsrc(p + e0, valid * 2);      // stores past the end are dropped
    const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
    for (int j = 0; j < kLaneElems; ++j)
        __builtin_amdgcn_raw_buffer_store_b16((uint16_t)(w[j / 2] >> (16 * (j & 1))), r,
                                              (int)((lane * kLaneElems + j) * 2), 0, 0);
}

template <int WHICH>
__global__ void __launch_bounds__(kWave) sdl_eval_kernel(const EvalArgs a)
{
    const uint32_t lane = threadIdx.x;
    const uint64_t e0 = (uint64_t)blockIdx.x * kTile;
    const uint64_t rem = a.numel - e0;
    const uint32_t valid = rem < (uint64_t)kTile ? (uint32_t)rem : (uint32_t)kTile;
    const bool fast = a.fast != 0u;
    u32x4 out;
    if constexpr (WHICH == SDL_EVAL_FIRST_REPLICA) {
        out = load_bf16x8(a.w[0], e0, valid, fast, lane);
    } else if constexpr (WHICH == SDL_EVAL_OUTER) {
        float v[kLaneElems];
        if (fast && valid == (uint32_t)kTile) {
            const __amdgpu_buffer_rsrc_t r = rsrc(a.g + e0, kTile * 4);
            const u32x4 x0 = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(lane * 32), 0, 2);
            const u32x4 x1 = __builtin_amdgcn_raw_buffer_load_b128(r, (int)(lane * 32 + 16), 0, 2);
            v[0] = u2f(x0.x); v[1] = u2f(x0.y); v[2] = u2f(x0.z); v[3] = u2f(x0.w);
            v[4] = u2f(x1.x); v[5] = u2f(x1.y); v[6] = u2f(x1.z); v[7] = u2f(x1.w);
        } else if (valid == (uint32_t)kTile) {
            const u32x4_f32elem* pg = reinterpret_cast<const u32x4_f32elem*>(a.g + e0 + lane * kLaneElems);
            const u32x4_f32elem x0 = __builtin_nontemporal_load(pg);
            const u32x4_f32elem x1 = __builtin_nontemporal_load(pg + 1);
            v[0] = u2f(x0.x); v[1] = u2f(x0.y); v[2] = u2f(x0.z); v[3] = u2f(x0.w);
            v[4] = u2f(x1.x); v[5] = u2f(x1.y); v[6] = u2f(x1.z); v[7] = u2f(x1.w);
        } else {
            const __amdgpu_buffer_rsrc_t r = rsrc(a.g + e0, valid * 4);
#pragma unroll
            for (int j = 0; j < kLaneElems; ++j)
                v[j] = u2f(__builtin_amdgcn_raw_buffer_load_b32(r, (int)((lane * kLaneElems + j) * 4), 0, 0));
        }
        out = u32x4{bf16_pack(v[0], v[1]), bf16_pack(v[2], v[3]), bf16_pack(v[4], v[5]), bf16_pack(v[6], v[7])};
    } else {
        // fp32 sum in replica order, one division, one rounding to bf16
        float acc[kLaneElems];
#pragma unroll
        for (int j = 0; j < kLaneElems; ++j) acc[j] = 0.0f;
        for (uint32_t m = 0; m < a.M; ++m) {
            const u32x4 x = load_bf16x8(a.w[m], e0, valid, fast, lane);
            const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int j = 0; j < kLaneElems; ++j)
                acc[j] = acc[j] + u2f((j & 1) ? (w[j / 2] & 0xffff0000u) : (w[j / 2] << 16));
        }
        const float fm = (float)a.M;
#pragma unroll
        for (int j = 0; j < kLaneElems; ++j) acc[j] = acc[j] / fm;
        out = u32x4{bf16_pack(acc[0], acc[1]), bf16_pack(acc[2], acc[3]), bf16_pack(acc[4], acc[5]),
                    bf16_pack(acc[6], acc[7])};
    }
    store_bf16x8(a.out, e0, valid, fast, lane, out);
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace

extern "C" {

int sdl_evaluation_params(sdl_eval_params_t which, const float* g, const void* const* w, uint32_t M, uint64_t numel,
                          void* out_bf16, void* stream)
{
    if (which != SDL_EVAL_FIRST_REPLICA && which != SDL_EVAL_REPLICA_MEAN && which != SDL_EVAL_OUTER)
        return SDL_ERR_INVALID_ARG;
    const bool needs_w = which != SDL_EVAL_OUTER;
    if (needs_w && (M == 0 || M > SDL_MAX_WORKERS)) return SDL_ERR_INVALID_ARG;
    if (numel == 0) return SDL_OK;
    if (!out_bf16 || (needs_w && !w) || (!needs_w && !g)) return SDL_ERR_INVALID_ARG;
    if (!aligned(out_bf16, 2) || (!needs_w && !aligned(g, 4))) return SDL_ERR_ALIGNMENT;
    if (numel > (uint64_t)0x7fffffff * (uint64_t)kTile) return SDL_ERR_UNSUPPORTED;
    EvalArgs a{};
    a.g = g;
    a.out = static_cast<uint16_t*>(out_bf16);
    a.numel = numel;
    a.M = needs_w ? (which == SDL_EVAL_FIRST_REPLICA ? 1u : M) : 0u;
    a.which = (uint32_t)which;
    bool fast = aligned(out_bf16, 16) && (needs_w || aligned(g, 16));
    for (uint32_t m = 0; m < a.M; ++m) {
        if (!w[m]) return SDL_ERR_INVALID_ARG;
        if (!aligned(w[m], 2)) return SDL_ERR_ALIGNMENT;
        fast = fast && aligned(w[m], 16);
        a.w[m] = static_cast<const uint16_t*>(w[m]);
    }
    a.fast = fast ? 1u : 0u;
    const dim3 grid((uint32_t)((numel + kTile - 1) / kTile)), block(kWave);
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (which) {
    case SDL_EVAL_FIRST_REPLICA: hipLaunchKernelGGL((sdl_eval_kernel<SDL_EVAL_FIRST_REPLICA>), grid, block, 0, st, a); break;
    case SDL_EVAL_REPLICA_MEAN: hipLaunchKernelGGL((sdl_eval_kernel<SDL_EVAL_REPLICA_MEAN>), grid, block, 0, st, a); break;
    default: hipLaunchKernelGGL((sdl_eval_kernel<SDL_EVAL_OUTER>), grid, block, 0, st, a); break;
    }
    return hipGetLastError() == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

}  // extern "C"
