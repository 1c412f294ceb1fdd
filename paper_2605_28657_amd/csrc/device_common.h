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

// two fp32 values -> one dword of two bf16 (lo in bits 0..15), one packed conversion (round to nearest even)
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// snake(x) = x + sin(alpha x)^2 / (beta + 1e-9); inv_beta = 1 / (beta + 1e-9) is prepared on the host.
__device__ __forceinline__ float snake_precise(float x, float alpha, float inv_beta)
{
    const float s = sinf(alpha * x);
    return fmaf(s * s, inv_beta, x);
}

// Fast variant for the bf16 path: alpha_rev = alpha / (2 pi), the hardware sine takes revolutions.  It is
// defined for |alpha_rev x| <= 256 and returns 0 beyond, where snake(x) = x is exact to far below the bf16
// rounding of the operand it feeds (sin^2/beta <= 1/beta against |x| > 1600/alpha), so no range reduction.
__device__ __forceinline__ float snake_fast(float x, float alpha_rev, float inv_beta)
{
    const float s = __builtin_amdgcn_sinf(alpha_rev * x);
    return fmaf(s * s, inv_beta, x);
}

// Raw buffer descriptor over [base, base + bytes): loads outside return zero, stores outside are dropped.
// Dword 3 selects 32-bit raw addressing on gfx9-family parts.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, unsigned bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// Residual stream h of the bf16 path in HBM: IEEE half.  bf16 storage of h (one rounding of 2^-9 per layer, at
// full strength on the main path) would by itself exceed the error budget; half has 3 more mantissa bits, its
// roundings are an order of magnitude below those of the bf16 MFMA operands, and it halves the traffic of the
// HBM-bound layers compared to fp32.  All arithmetic on h is fp32.
typedef _Float16 hres_t;
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Pins a value to its fp32 rounding.  Without it the compiler may fuse the arithmetic that produced v with a following
// conversion to half into one mixed-precision instruction that rounds once; it does so in some unrolled iterations and
// not in others, and the result of an element would then depend on its position in the tile.
__device__ __forceinline__ float keep_f32(float v)
{
    asm("" : "+v"(v));
    return v;
}

// Conversions to half saturate instead of overflowing: with the FP16_OVFL bit of the wave's MODE register set, a
// result beyond the half range is clamped to +-65504 (true infinities stay).  The residual stream and the operands of
// the wide levels are IEEE half; a trained decoder whose activations leave that range then clips instead of turning
// into infinities and, through Snake's sine, NaNs.  Called once at the start of every kernel that converts to half.
__device__ __forceinline__ void fp16_saturate_on()
{
    // hwreg(HW_REG_MODE = 1, offset 23, size 1): simm16 = ((size - 1) << 11) | (offset << 6) | id
    __builtin_amdgcn_s_setreg((0 << 11) | (23 << 6) | 1, 1);
}

// two fp32 values -> one dword of two halves (lo in bits 0..15), round to nearest even
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi)
{
    const f16x2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
}

}  // namespace demon
