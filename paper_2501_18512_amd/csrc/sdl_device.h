// Device-side helpers shared by the kernels of this library (gfx950): bit casts, vector types,
// buffer resources.  Internal to csrc/; nothing here is part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sdl_device {

constexpr int kWave = 64;   // lanes of a wavefront

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Vectors at the alignment of one fp32 / bf16 element, for tiles that start at any element of an
// array: the compiler picks the widest access the target allows (64- and 128-bit ones here, gfx950
// under ROCm runs in unaligned-access mode).
typedef uint32_t u32x4_f32elem __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x4_bf16elem __attribute__((ext_vector_type(4), aligned(2)));
typedef float f32x4_elem __attribute__((ext_vector_type(4), aligned(4)));
typedef uint32_t u32x2_elem __attribute__((ext_vector_type(2), aligned(2)));

__device__ __forceinline__ uint32_t f2u(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float u2f(uint32_t u) { return __builtin_bit_cast(float, u); }

// Raw buffer resource over [p, p + bytes): loads past the end return 0, stores past the end are
// dropped (the range check of the buffer instructions).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t rsrc(const void* p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}

}  // namespace sdl_device
