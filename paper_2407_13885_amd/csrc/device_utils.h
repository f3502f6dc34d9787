// Small device-side helpers shared by the attnw kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace attnw {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr float kLog2e = 1.4426950408889634f;
// Sentinel for "no score seen yet" / masked keys in running maxima.  Finite on
// purpose: differences of two sentinels are 0, never NaN.
constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Two fp32 -> packed bf16 pair (lo in bits 0..15), round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// 2^x on the transcendental unit (v_exp_f32); exp2(-inf) = 0, exp2(0) = 1.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

__device__ __forceinline__ float wave_reduce_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ float wave_reduce_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Blocks are dealt round-robin to the 8 XCDs (each with its own L2).  Remap the
// hardware block index so that every XCD works on one contiguous range of
// logical tiles (the same heads, hence the same K in its L2).  `padded` is the
// launched grid size, a multiple of 8; logical ids >= the real tile count are
// the caller's to discard.
__device__ __forceinline__ uint32_t xcd_contiguous_block_id(uint32_t bid, uint32_t padded)
{
    const uint32_t per_xcd = padded >> 3;
    return (bid & 7u) * per_xcd + (bid >> 3);
}

}  // namespace attnw
