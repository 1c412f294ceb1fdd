// Device helpers shared by the kernels of libdemon_vae.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "internal.h"

namespace demon {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    __bf16 b = (__bf16)f;                          // round to nearest even
    return __builtin_bit_cast(uint16_t, b);
}

// snake(x) = x + sin(alpha x)^2 / (beta + 1e-9); inv_beta = 1 / (beta + 1e-9) is prepared on the host.
__device__ __forceinline__ float snake_precise(float x, float alpha, float inv_beta)
{
    const float s = sinf(alpha * x);
    return fmaf(s * s, inv_beta, x);
}

// Fast variant for the bf16 path: alpha_rev = alpha / (2 pi), the hardware sine takes revolutions.
__device__ __forceinline__ float snake_fast(float x, float alpha_rev, float inv_beta)
{
    const float s = __builtin_amdgcn_sinf(__builtin_amdgcn_fractf(alpha_rev * x));
    return fmaf(s * s, inv_beta, x);
}

// Raw buffer descriptor over [base, base + bytes): loads outside return zero, stores outside are dropped.
// Dword 3 selects 32-bit raw addressing on gfx9-family parts.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

}  // namespace demon
