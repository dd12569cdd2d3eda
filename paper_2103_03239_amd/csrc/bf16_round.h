// binary32 -> bfloat16, round to nearest, ties to even (the storage rounding of bfloat16
// states), for gfx950.
//
// The kernels use the hardware conversion (v_cvt_pk_bf16_f32, two values per instruction).
// bf16_bits_reference is the same rounding written with integer operations: add 0x7fff plus
// the lowest kept bit, keep the upper 16 bits; a NaN stays a NaN (upper 16 bits with the
// quiet bit set).  The two agree on all 2^32 inputs (moshpit_check_bf16_rounding compares
// them exhaustively on the GPU), so which one a kernel uses never shows in a result.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moshpit {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float bf16_src2_t __attribute__((ext_vector_type(2)));

// lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t bf16_pair(float lo, float hi)
{
    const bf16_src2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

__device__ __forceinline__ uint16_t bf16_one(float f)
{
    return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));
}

__device__ __forceinline__ uint32_t bf16_bits_reference(float f)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;   // keep NaN a NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace moshpit
