// Device side of the library: the streaming kernels of the fragment outer step for
// gfx950 (MI355X), and the C entry points that launch them.
//
// Work decomposition (all four kernels): one lane owns 8 consecutive parameters, so a
// quad of lanes owns one 32-element scale block and a 256-lane workgroup owns 2048
// parameters.  Per replica a lane moves one 128-bit word of bf16, per fp32 array two.
// The block maximum is a 2-step DPP exchange inside the quad; nothing goes through
// LDS.  A launch covers up to kMaxRuns contiguous runs of the flat model; every
// workgroup belongs to exactly one run, so scale blocks never straddle runs.
//
// Arithmetic contract (Algorithm 2 and Sections 2.1, 2.3, 2.4 of the paper, with the
// exchange formats documented in sdl.h): every fp32 operation is a single IEEE
// operation in the documented order; this file must be compiled with
// -ffp-contract=off and with fp32 denormals enabled (the hipcc default).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>

#include "sdl.h"

namespace {

constexpr int kLane = 8;                      // parameters per lane
constexpr int kThreads = 256;                 // lanes per workgroup
constexpr int kGroup = kLane * kThreads;      // parameters per workgroup
constexpr int kMaxRuns = 16;                  // runs per launch

enum Mode { kQuantize = 0, kReduce = 1, kMerge = 2, kFused = 3 };

struct Run {
    uint64_t offset;     // first element of the run in the flat arrays
    uint64_t numel;
    uint32_t first_wg;   // first workgroup of the launch that works on this run
    uint32_t vec;        // 1: every array of this run is 16-byte aligned at its start
};

struct Args {
    float* g;
    float* mom;
    const uint16_t* w_send[SDL_MAX_WORKERS];
    uint16_t* w_now[SDL_MAX_WORKERS];
    uint8_t* codes[SDL_MAX_WORKERS];
    uint8_t* scales[SDL_MAX_WORKERS];
    Run runs[kMaxRuns];
    uint32_t n_runs;
    uint32_t M;
    float lr, mu, alpha, one_minus_alpha;
    uint32_t aliased;    // w_send[m] == w_now[m]
    uint32_t emit;       // fused kernel: also write the messages
};

// ------------------------------------------------------------------ bit helpers

__device__ __forceinline__ uint32_t f2u(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// bf16 pair packed in one dword: element 0 in the low half.
__device__ __forceinline__ float bf16_lo(uint32_t u) { return u2f(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return u2f(u & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even, NaN kept quiet.
__device__ __forceinline__ uint32_t bf16_rne(float x)
{
    uint32_t u = f2u(x);
    uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    return ((u & 0x7fffffffu) > 0x7f800000u) ? ((u >> 16) | 0x40u) : r;
}
__device__ __forceinline__ uint32_t bf16_pack(float lo, float hi)
{
    return bf16_rne(lo) | (bf16_rne(hi) << 16);
}

// Maximum over the four lanes of a quad (two DPP quad-permute exchanges).
__device__ __forceinline__ uint32_t quad_max(uint32_t v)
{
    uint32_t t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);   // lanes 1,0,3,2
    v = v > t ? v : t;
    t = (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);            // lanes 2,3,0,1
    return v > t ? v : t;
}

// ------------------------------------------------------------------ tile loads / stores
// fast: the lane's 8 elements are all valid and the arrays are 16-byte aligned.

__device__ __forceinline__ void load_f32(const float* p, int valid, bool fast, float (&v)[kLane])
{
    if (fast) {
        const float4 a = reinterpret_cast<const float4*>(p)[0];
        const float4 b = reinterpret_cast<const float4*>(p)[1];
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
        v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
#pragma unroll
        for (int j = 0; j < kLane; ++j) v[j] = j < valid ? p[j] : 0.0f;
    }
}

__device__ __forceinline__ void store_f32(float* p, int valid, bool fast, const float (&v)[kLane])
{
    if (fast) {
        reinterpret_cast<float4*>(p)[0] = make_float4(v[0], v[1], v[2], v[3]);
        reinterpret_cast<float4*>(p)[1] = make_float4(v[4], v[5], v[6], v[7]);
    } else {
#pragma unroll
        for (int j = 0; j < kLane; ++j)
            if (j < valid) p[j] = v[j];
    }
}

__device__ __forceinline__ void load_bf16(const uint16_t* p, int valid, bool fast, uint32_t (&u)[4])
{
    if (fast) {
        const uint4 a = reinterpret_cast<const uint4*>(p)[0];
        u[0] = a.x; u[1] = a.y; u[2] = a.z; u[3] = a.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            uint32_t lo = 2 * k < valid ? p[2 * k] : 0u;
            uint32_t hi = 2 * k + 1 < valid ? p[2 * k + 1] : 0u;
            u[k] = lo | (hi << 16);
        }
    }
}

__device__ __forceinline__ void store_bf16(uint16_t* p, int valid, bool fast, const uint32_t (&u)[4])
{
    if (fast) {
        reinterpret_cast<uint4*>(p)[0] = make_uint4(u[0], u[1], u[2], u[3]);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (2 * k < valid) p[2 * k] = (uint16_t)(u[k] & 0xffffu);
            if (2 * k + 1 < valid) p[2 * k + 1] = (uint16_t)(u[k] >> 16);
        }
    }
}

__device__ __forceinline__ void unpack_bf16(const uint32_t (&u)[4], float (&v)[kLane])
{
#pragma unroll
    for (int k = 0; k < 4; ++k) { v[2 * k] = bf16_lo(u[k]); v[2 * k + 1] = bf16_hi(u[k]); }
}

// ------------------------------------------------------------------ exchange formats
// A message element is produced in two forms: its decoded fp32 value dq (what the
// receiver accumulates) and, when asked for, its code.

template <int FMT> struct BlockScale {       // per quad (32-element block) quantities
    uint32_t sb;      // scale byte
    float inv;        // 2^(127-sb), or 0 for a degenerate block
    float scale;      // 2^(sb-127), NaN for a block that holds Inf/NaN
    bool degenerate;  // block maximum is zero, subnormal, Inf or NaN
};

template <int FMT>
__device__ __forceinline__ BlockScale<FMT> block_scale_from_exponent(uint32_t e_a)
{
    constexpr uint32_t emax = (FMT == SDL_FMT_E3M0) ? 4u : 8u;
    BlockScale<FMT> b;
    b.sb = e_a > emax ? e_a - emax : 0u;
    b.degenerate = (e_a == 0u) || (e_a == 255u);
    b.inv = b.degenerate ? 0.0f : u2f((254u - b.sb) << 23);
    b.scale = b.sb ? u2f(b.sb << 23) : u2f(0x00400000u);       // 2^-127 is an fp32 subnormal
    if (e_a == 255u) { b.sb = 255u; b.scale = u2f(0x7fc00000u); }
    return b;
}

__device__ __forceinline__ float scale_from_byte(uint32_t sb)
{
    float s = sb ? u2f(sb << 23) : u2f(0x00400000u);
    return sb == 255u ? u2f(0x7fc00000u) : s;
}

// Encode the lane's 8 outer gradients d of one replica.  dq = decoded values.  codes:
// E3M0 -> c[0] holds 8 nibbles; E4M3 -> c[0..1] hold 8 bytes; BF16 -> c[0..3];
// FP32 -> the bits of d.  sb = scale byte of the lane's block (scaled formats).
template <int FMT>
__device__ __forceinline__ void encode(const float (&d)[kLane], float (&dq)[kLane], uint32_t (&c)[kLane],
                                       uint32_t& sb, bool want_codes)
{
    if constexpr (FMT == SDL_FMT_FP32) {
#pragma unroll
        for (int j = 0; j < kLane; ++j) { dq[j] = d[j]; c[j] = f2u(d[j]); }
        sb = 0;
    } else if constexpr (FMT == SDL_FMT_BF16) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[k] = bf16_pack(d[2 * k], d[2 * k + 1]);
            dq[2 * k] = bf16_lo(c[k]);
            dq[2 * k + 1] = bf16_hi(c[k]);
        }
        sb = 0;
    } else {
        uint32_t amax = 0;
#pragma unroll
        for (int j = 0; j < kLane; ++j) {
            uint32_t m = f2u(d[j]) & 0x7fffffffu;
            amax = m > amax ? m : amax;
        }
        amax = quad_max(amax);
        const BlockScale<FMT> b = block_scale_from_exponent<FMT>(amax >> 23);
        sb = b.sb;
        uint32_t packed0 = 0, packed1 = 0;
#pragma unroll
        for (int j = 0; j < kLane; ++j) {
            const float y = __builtin_fabsf(d[j]) * b.inv;     // exact power-of-two scaling
            const uint32_t yb = f2u(y);
            const uint32_t sign = f2u(d[j]) & 0x80000000u;
            float val;
            if constexpr (FMT == SDL_FMT_E3M0) {
                // nearest power of two in the linear domain; a tie (mantissa exactly
                // 1.5) goes to the even exponent code, whose parity is that of the
                // biased fp32 exponent because the re-bias (124) is even
                const uint32_t r = (yb + 0x3fffffu + ((yb >> 23) & 1u)) & 0x7f800000u;
                const float pw = __builtin_amdgcn_fmed3f(u2f(r), 0.25f, 16.0f);
                val = y > 0.125f ? pw : 0.0f;                  // half of the smallest magnitude
            } else {
                // E4M3: 3 mantissa bits above 2^-6, multiples of 2^-9 below, max 448
                const uint32_t r = (yb + 0x7ffffu + ((yb >> 20) & 1u)) & 0xfff00000u;
                const float vs = __builtin_rintf(y * 512.0f) * 0.001953125f;
                val = y < 0.015625f ? vs : u2f(r);
                val = __builtin_fminf(val, 448.0f);
                val = b.degenerate ? 0.0f : val;
            }
            dq[j] = u2f(sign | f2u(val * b.scale));
            if (want_codes) {
                if constexpr (FMT == SDL_FMT_E3M0) {
                    const uint32_t E = val == 0.0f ? 0u : (f2u(val) >> 23) - 124u;
                    packed0 |= ((sign >> 28) | E) << (4 * j);
                } else {
                    const uint32_t mag = val < 0.015625f ? (uint32_t)(val * 512.0f)
                                                         : (f2u(val) >> 20) - 960u;
                    const uint32_t byte = (sign >> 24) | mag;
                    if (j < 4) packed0 |= byte << (8 * j); else packed1 |= byte << (8 * (j - 4));
                }
            }
        }
        c[0] = packed0; c[1] = packed1;
    }
}

// Decode the lane's 8 message elements of one replica from memory.
template <int FMT>
__device__ __forceinline__ void load_decode(const uint8_t* codes, const uint8_t* scales, uint64_t base,
                                            int valid, bool fast, float (&dq)[kLane])
{
    if constexpr (FMT == SDL_FMT_FP32) {
        load_f32(reinterpret_cast<const float*>(codes) + base, valid, fast, dq);
    } else if constexpr (FMT == SDL_FMT_BF16) {
        uint32_t u[4];
        load_bf16(reinterpret_cast<const uint16_t*>(codes) + base, valid, fast, u);
        unpack_bf16(u, dq);
    } else {
        const uint32_t sb = valid > 0 ? scales[base / SDL_BLOCK] : 127u;
        const float scale = scale_from_byte(sb);
        uint32_t c0 = 0, c1 = 0;
        if constexpr (FMT == SDL_FMT_E3M0) {
            if (fast) {
                c0 = *reinterpret_cast<const uint32_t*>(codes + base / 2);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (2 * k < valid) c0 |= (uint32_t)codes[base / 2 + k] << (8 * k);
            }
#pragma unroll
            for (int j = 0; j < kLane; ++j) {
                const uint32_t nib = (c0 >> (4 * j)) & 15u;
                const uint32_t E = nib & 7u;
                const float val = E ? u2f((E + 124u) << 23) : 0.0f;
                dq[j] = u2f(((nib & 8u) << 28) | f2u(val * scale));
            }
        } else {
            if (fast) {
                const uint2 w = *reinterpret_cast<const uint2*>(codes + base);
                c0 = w.x; c1 = w.y;
            } else {
#pragma unroll
                for (int j = 0; j < kLane; ++j) {
                    uint32_t byte = j < valid ? codes[base + j] : 0u;
                    if (j < 4) c0 |= byte << (8 * j); else c1 |= byte << (8 * (j - 4));
                }
            }
#pragma unroll
            for (int j = 0; j < kLane; ++j) {
                const uint32_t byte = ((j < 4 ? c0 : c1) >> (8 * (j & 3))) & 255u;
                const uint32_t mag = byte & 0x7fu;
                const float val = mag >= 8u ? u2f((mag + 960u) << 20) : (float)mag * 0.001953125f;
                dq[j] = u2f(((byte & 0x80u) << 24) | f2u(val * scale));
            }
        }
    }
}

// Write the lane's part of one replica's message.
template <int FMT>
__device__ __forceinline__ void store_codes(uint8_t* codes, uint8_t* scales, uint64_t base, int valid,
                                            bool fast, const uint32_t (&c)[kLane], uint32_t sb)
{
    if constexpr (FMT == SDL_FMT_FP32) {
        float v[kLane];
#pragma unroll
        for (int j = 0; j < kLane; ++j) v[j] = u2f(c[j]);
        store_f32(reinterpret_cast<float*>(codes) + base, valid, fast, v);
    } else if constexpr (FMT == SDL_FMT_BF16) {
        const uint32_t u[4] = {c[0], c[1], c[2], c[3]};
        store_bf16(reinterpret_cast<uint16_t*>(codes) + base, valid, fast, u);
    } else {
        if ((threadIdx.x & 3u) == 0u && valid > 0) scales[base / SDL_BLOCK] = (uint8_t)sb;
        if constexpr (FMT == SDL_FMT_E3M0) {
            if (fast) {
                *reinterpret_cast<uint32_t*>(codes + base / 2) = c[0];
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (2 * k < valid) codes[base / 2 + k] = (uint8_t)(c[0] >> (8 * k));
            }
        } else {
            if (fast) {
                *reinterpret_cast<uint2*>(codes + base) = make_uint2(c[0], c[1]);
            } else {
#pragma unroll
                for (int j = 0; j < kLane; ++j)
                    if (j < valid) codes[base + j] = (uint8_t)((j < 4 ? c[0] : c[1]) >> (8 * (j & 3)));
            }
        }
    }
}

// ------------------------------------------------------------------ the kernel
// MT > 0: number of replicas known at compile time, all loads issued up front.
// MT == 0: any M, replicas visited in a run-time loop.

template <int MODE, int FMT, int MT>
__global__ __launch_bounds__(kThreads) void sdl_kernel(const Args a)
{
    // which run does this workgroup work on (uniform scan of at most kMaxRuns entries)
    const uint32_t wg = blockIdx.x;
    uint32_t r = 0;
    for (uint32_t i = 1; i < a.n_runs; ++i)
        if (wg >= a.runs[i].first_wg) r = i;
    const uint64_t run_off = a.runs[r].offset;
    const uint64_t run_n = a.runs[r].numel;
    const uint64_t base = ((uint64_t)(wg - a.runs[r].first_wg) * kThreads + threadIdx.x) * kLane;
    const int valid = base >= run_n ? 0 : (run_n - base >= (uint64_t)kLane ? kLane : (int)(run_n - base));
    const bool fast = a.runs[r].vec && valid == kLane;
    const uint64_t e0 = run_off + base;           // index into the flat model arrays
    const uint32_t M = MT > 0 ? (uint32_t)MT : a.M;
    constexpr int MU = MT > 0 ? MT : 1;

    float g[kLane], mom[kLane], acc[kLane];
    uint32_t ws[MU][4], wn[MU][4];

    // ---- loads that do not depend on anything
    load_f32(a.g + e0, valid, fast, g);
    if constexpr (MODE == kReduce || MODE == kFused) load_f32(a.mom + e0, valid, fast, mom);
    if constexpr (MT > 0) {
        if constexpr (MODE == kQuantize || MODE == kFused) {
#pragma unroll
            for (int m = 0; m < MT; ++m) load_bf16(a.w_send[m] + e0, valid, fast, ws[m]);
        }
        if constexpr (MODE == kMerge) {
#pragma unroll
            for (int m = 0; m < MT; ++m) load_bf16(a.w_now[m] + e0, valid, fast, wn[m]);
        }
        if constexpr (MODE == kFused) {
            if (!a.aliased) {
#pragma unroll
                for (int m = 0; m < MT; ++m) load_bf16(a.w_now[m] + e0, valid, fast, wn[m]);
            }
        }
    }

    // ---- outer gradients, messages, fp32 sum over replicas in ascending order
    if constexpr (MODE != kMerge) {
#pragma unroll
        for (int j = 0; j < kLane; ++j) acc[j] = 0.0f;
#pragma unroll
        for (uint32_t m = 0; m < M; ++m) {
            float dq[kLane];
            if constexpr (MODE == kReduce) {
                load_decode<FMT>(a.codes[m], a.scales[m], base, valid, fast, dq);
            } else {
                const int mi = MT > 0 ? (int)m : 0;
                if constexpr (MT == 0) load_bf16(a.w_send[m] + e0, valid, fast, ws[0]);
                float w[kLane], d[kLane];
                uint32_t c[kLane], sb;
                unpack_bf16(ws[mi], w);
#pragma unroll
                for (int j = 0; j < kLane; ++j) d[j] = g[j] - w[j];
                const bool want = MODE == kQuantize || a.emit;
                encode<FMT>(d, dq, c, sb, want);
                if (want) store_codes<FMT>(a.codes[m], a.scales[m], base, valid, fast, c, sb);
            }
#pragma unroll
            for (int j = 0; j < kLane; ++j) acc[j] = acc[j] + dq[j];
        }
    }

    // ---- mean and Nesterov outer step
    if constexpr (MODE == kReduce || MODE == kFused) {
        const float fm = (float)M;
#pragma unroll
        for (int j = 0; j < kLane; ++j) {
            const float dbar = acc[j] / fm;
            const float m_new = a.mu * mom[j] + dbar;
            const float look = dbar + a.mu * m_new;
            mom[j] = m_new;
            g[j] = g[j] - a.lr * look;
        }
        store_f32(a.g + e0, valid, fast, g);
        store_f32(a.mom + e0, valid, fast, mom);
    }

    // ---- alpha-merge into every replica
    if constexpr (MODE == kMerge || MODE == kFused) {
        float gpart[kLane];
#pragma unroll
        for (int j = 0; j < kLane; ++j) gpart[j] = a.one_minus_alpha * g[j];
#pragma unroll
        for (uint32_t m = 0; m < M; ++m) {
            const int mi = MT > 0 ? (int)m : 0;
            if constexpr (MT == 0) load_bf16(a.w_now[m] + e0, valid, fast, wn[0]);
            float w[kLane];
            if (MT > 0 && MODE == kFused && a.aliased) unpack_bf16(ws[mi], w);
            else unpack_bf16(wn[mi], w);
            uint32_t out[4];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                out[k] = bf16_pack(a.alpha * w[2 * k] + gpart[2 * k],
                                   a.alpha * w[2 * k + 1] + gpart[2 * k + 1]);
            store_bf16(a.w_now[m] + e0, valid, fast, out);
        }
    }
}

// Plain streaming copy, 16 bytes per lane: the yardstick for the HBM roofline.
__global__ __launch_bounds__(kThreads) void sdl_copy_kernel(uint4* __restrict__ dst,
                                                            const uint4* __restrict__ src, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n16) dst[i] = src[i];
}

// ------------------------------------------------------------------ host side

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

size_t code_align(sdl_format_t fmt)
{
    return fmt == SDL_FMT_FP32 ? 4 : fmt == SDL_FMT_BF16 ? 2 : 1;
}
// bytes of code per element (x2 for E3M0, which holds half a byte)
size_t code_bytes_at(sdl_format_t fmt, uint64_t elem)
{
    switch (fmt) {
    case SDL_FMT_FP32: return (size_t)elem * 4;
    case SDL_FMT_BF16: return (size_t)elem * 2;
    case SDL_FMT_E4M3: return (size_t)elem;
    default: return (size_t)(elem / 2);
    }
}

template <int MODE, int FMT>
hipError_t launch_m(const Args& a, uint32_t n_wg, hipStream_t s)
{
    const dim3 grid(n_wg), block(kThreads);
    switch (a.M) {
    case 1: hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 1>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 2>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 4>), grid, block, 0, s, a); break;
    case 8: hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 8>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((sdl_kernel<MODE, FMT, 0>), grid, block, 0, s, a); break;
    }
    return hipGetLastError();
}

template <int MODE>
hipError_t launch(const Args& a, sdl_format_t fmt, uint32_t n_wg, hipStream_t s)
{
    if constexpr (MODE == kMerge) return launch_m<MODE, SDL_FMT_FP32>(a, n_wg, s);
    switch (fmt) {
    case SDL_FMT_FP32: return launch_m<MODE, SDL_FMT_FP32>(a, n_wg, s);
    case SDL_FMT_BF16: return launch_m<MODE, SDL_FMT_BF16>(a, n_wg, s);
    case SDL_FMT_E4M3: return launch_m<MODE, SDL_FMT_E4M3>(a, n_wg, s);
    default: return launch_m<MODE, SDL_FMT_E3M0>(a, n_wg, s);
    }
}

bool valid_format(sdl_format_t fmt) { return fmt >= SDL_FMT_FP32 && fmt <= SDL_FMT_E3M0; }

// Fill a.runs from a list of (offset, numel); returns the number of workgroups.  vec is
// set per run when every array used by the call is 16-byte aligned at the run start.
struct RunBuilder {
    Args* a;
    uint64_t n_wg = 0;
    explicit RunBuilder(Args* args) : a(args) { a->n_runs = 0; }
    bool full() const { return a->n_runs == kMaxRuns; }
    void add(uint64_t offset, uint64_t numel, bool vec)
    {
        Run& r = a->runs[a->n_runs++];
        r.offset = offset; r.numel = numel; r.first_wg = (uint32_t)n_wg; r.vec = vec ? 1u : 0u;
        n_wg += (numel + kGroup - 1) / kGroup;
    }
};

// One span starting at the given pointers (offset 0).
template <int MODE>
int run_single_span(Args& a, uint64_t n, sdl_format_t fmt, bool vec, void* stream)
{
    if (n == 0) return SDL_OK;
    if (n > (uint64_t)0x7fffffff * (uint64_t)kGroup) return SDL_ERR_UNSUPPORTED;
    RunBuilder rb(&a);
    rb.add(0, n, vec);
    hipError_t e = launch<MODE>(a, fmt, (uint32_t)rb.n_wg, (hipStream_t)stream);
    return e == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

}  // namespace

extern "C" {

int sdl_quantize_outer_grad(const float* g, const void* const* w_send, uint32_t M, uint64_t n,
                            sdl_format_t fmt, void* const* codes, void* const* scales, void* stream)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = fmt == SDL_FMT_E4M3 || fmt == SDL_FMT_E3M0;
    if (n && (!g || !w_send || !codes || (scaled && !scales))) return SDL_ERR_INVALID_ARG;
    if (n == 0) return SDL_OK;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = const_cast<float*>(g);
    a.M = M;
    bool vec = aligned(g, 16);
    if (!aligned(g, 4)) return SDL_ERR_ALIGNMENT;
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_send[m] || !codes[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_send[m], 2) || !aligned(codes[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
        vec = vec && aligned(w_send[m], 16) && aligned(codes[m], 16);
        a.w_send[m] = static_cast<const uint16_t*>(w_send[m]);
        a.codes[m] = static_cast<uint8_t*>(codes[m]);
        a.scales[m] = scaled ? static_cast<uint8_t*>(scales[m]) : nullptr;
    }
    return run_single_span<kQuantize>(a, n, fmt, vec, stream);
}

int sdl_dequant_reduce_nesterov(float* g, float* mom, const void* const* codes,
                                const void* const* scales, uint32_t M, uint64_t n, sdl_format_t fmt,
                                float lr, float mu, void* stream)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    const bool scaled = fmt == SDL_FMT_E4M3 || fmt == SDL_FMT_E3M0;
    if (n && (!g || !mom || !codes || (scaled && !scales))) return SDL_ERR_INVALID_ARG;
    if (n == 0) return SDL_OK;
    if (!aligned(g, 4) || !aligned(mom, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = g; a.mom = mom; a.M = M; a.lr = lr; a.mu = mu;
    bool vec = aligned(g, 16) && aligned(mom, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!codes[m] || (scaled && !scales[m])) return SDL_ERR_INVALID_ARG;
        if (!aligned(codes[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
        vec = vec && aligned(codes[m], 16);
        a.codes[m] = static_cast<uint8_t*>(const_cast<void*>(codes[m]));
        a.scales[m] = scaled ? static_cast<uint8_t*>(const_cast<void*>(scales[m])) : nullptr;
    }
    return run_single_span<kReduce>(a, n, fmt, vec, stream);
}

int sdl_merge_overlap(const float* g_new, void* const* w_now, uint32_t M, uint64_t n, float alpha,
                      void* stream)
{
    if (M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    if (n && (!g_new || !w_now)) return SDL_ERR_INVALID_ARG;
    if (n == 0) return SDL_OK;
    if (!aligned(g_new, 4)) return SDL_ERR_ALIGNMENT;
    Args a;
    std::memset(&a, 0, sizeof(a));
    a.g = const_cast<float*>(g_new); a.M = M; a.alpha = alpha; a.one_minus_alpha = 1.0f - alpha;
    bool vec = aligned(g_new, 16);
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_now[m]) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_now[m], 2)) return SDL_ERR_ALIGNMENT;
        vec = vec && aligned(w_now[m], 16);
        a.w_now[m] = static_cast<uint16_t*>(w_now[m]);
    }
    return run_single_span<kMerge>(a, n, SDL_FMT_FP32, vec, stream);
}

// Shared argument marshalling of the two fused entry points.
static int fill_fused_args(Args& a, float* g, float* mom, const void* const* w_send, void* const* w_now,
                           uint32_t M, sdl_format_t fmt, float lr, float mu, float alpha, bool* vec)
{
    if (!valid_format(fmt) || M == 0 || M > SDL_MAX_WORKERS) return SDL_ERR_INVALID_ARG;
    if (!g || !mom || !w_send || !w_now) return SDL_ERR_INVALID_ARG;
    if (!aligned(g, 4) || !aligned(mom, 4)) return SDL_ERR_ALIGNMENT;
    std::memset(&a, 0, sizeof(a));
    a.g = g; a.mom = mom; a.M = M; a.lr = lr; a.mu = mu; a.alpha = alpha;
    a.one_minus_alpha = 1.0f - alpha;
    *vec = aligned(g, 16) && aligned(mom, 16);
    uint32_t same = 0;
    for (uint32_t m = 0; m < M; ++m) {
        if (!w_send[m] || !w_now[m]) return SDL_ERR_INVALID_ARG;
        if (!aligned(w_send[m], 2) || !aligned(w_now[m], 2)) return SDL_ERR_ALIGNMENT;
        *vec = *vec && aligned(w_send[m], 16) && aligned(w_now[m], 16);
        same += (w_send[m] == w_now[m]);
        a.w_send[m] = static_cast<const uint16_t*>(w_send[m]);
        a.w_now[m] = static_cast<uint16_t*>(w_now[m]);
    }
    if (same != 0 && same != M) return SDL_ERR_INVALID_ARG;   // alias all replicas or none
    a.aliased = same == M;
    return SDL_OK;
}

int sdl_fragment_outer_step(float* g, float* mom, const void* const* w_send, void* const* w_now,
                            uint32_t M, uint64_t n, sdl_format_t fmt, float lr, float mu, float alpha,
                            void* const* codes_or_null, void* const* scales_or_null, void* stream)
{
    if (n == 0) return (valid_format(fmt) && M >= 1 && M <= SDL_MAX_WORKERS) ? SDL_OK : SDL_ERR_INVALID_ARG;
    Args a;
    bool vec = false;
    int rc = fill_fused_args(a, g, mom, w_send, w_now, M, fmt, lr, mu, alpha, &vec);
    if (rc != SDL_OK) return rc;
    if (codes_or_null) {
        const bool scaled = fmt == SDL_FMT_E4M3 || fmt == SDL_FMT_E3M0;
        if (scaled && !scales_or_null) return SDL_ERR_INVALID_ARG;
        for (uint32_t m = 0; m < M; ++m) {
            if (!codes_or_null[m] || (scaled && !scales_or_null[m])) return SDL_ERR_INVALID_ARG;
            if (!aligned(codes_or_null[m], code_align(fmt))) return SDL_ERR_ALIGNMENT;
            vec = vec && aligned(codes_or_null[m], 16);
            a.codes[m] = static_cast<uint8_t*>(codes_or_null[m]);
            a.scales[m] = scaled ? static_cast<uint8_t*>(scales_or_null[m]) : nullptr;
        }
        a.emit = 1;
    }
    return run_single_span<kFused>(a, n, fmt, vec, stream);
}

int sdl_fragment_outer_step_plan(const sdl_plan_t* plan, uint32_t p, float* g_base, float* mom_base,
                                 const void* const* w_send_base, void* const* w_now_base, uint32_t M,
                                 sdl_format_t fmt, float lr, float mu, float alpha, void* stream)
{
    const sdl_span_t* runs = nullptr;
    uint32_t n_runs = 0;
    int rc = sdl_plan_fragment_runs(plan, p, &runs, &n_runs);
    if (rc != SDL_OK) return rc;
    Args a;
    bool vec = false;
    rc = fill_fused_args(a, g_base, mom_base, w_send_base, w_now_base, M, fmt, lr, mu, alpha, &vec);
    if (rc != SDL_OK) return rc;
    for (uint32_t first = 0; first < n_runs; first += kMaxRuns) {
        RunBuilder rb(&a);
        for (uint32_t i = first; i < n_runs && i < first + kMaxRuns; ++i) {
            // a run keeps the 16-byte alignment of the bases when it starts on a multiple of 8 elements
            rb.add(runs[i].offset, runs[i].numel, vec && (runs[i].offset % 8 == 0));
        }
        if (rb.n_wg > 0x7fffffffull) return SDL_ERR_UNSUPPORTED;
        hipError_t e = launch<kFused>(a, fmt, (uint32_t)rb.n_wg, (hipStream_t)stream);
        if (e != hipSuccess) return SDL_ERR_DEVICE;
    }
    return SDL_OK;
}

int sdl_copy_bytes(void* dst, const void* src, uint64_t nbytes, void* stream)
{
    if (nbytes == 0) return SDL_OK;
    if (!dst || !src || nbytes % 16 != 0) return SDL_ERR_INVALID_ARG;
    if (!aligned(dst, 16) || !aligned(src, 16)) return SDL_ERR_ALIGNMENT;
    const uint64_t n16 = nbytes / 16, n_wg = (n16 + kThreads - 1) / kThreads;
    if (n_wg > 0x7fffffffull) return SDL_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(sdl_copy_kernel, dim3((uint32_t)n_wg), dim3(kThreads), 0, (hipStream_t)stream,
                       static_cast<uint4*>(dst), static_cast<const uint4*>(src), n16);
    return hipGetLastError() == hipSuccess ? SDL_OK : SDL_ERR_DEVICE;
}

}  // extern "C"
