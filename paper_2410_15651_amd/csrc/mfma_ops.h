// Matrix-core (MFMA) building blocks for gfx950: 16x16 tiles with 16-bit
// operands and fp32 accumulation, and the two-part split that lets fp32
// probabilities go through 16-bit operands without losing accuracy.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "rlhf_rollout.h"

namespace rlhf {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

// D[16x16] += A[16x32] * B[32x16]; lane l supplies row (A) / column (B) l%16 and
// the 8 contraction entries of group l/16; it receives D[4*(l/16)+j][l%16].
template <int DT>
__device__ __forceinline__ f32x4_t mfma_k32(const uint4 &a, const uint4 &b, f32x4_t c)
{
    if constexpr (DT == RLHF_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// D[32x32] += A[32x16] * B[16x32]; lane l supplies row (A) / column (B) l%32 and
// the 8 contraction entries of half l/32; it receives, in register r, the
// element D[8*(r/4) + 4*(l/32) + r%4][l%32].  One wavefront issues these at the
// matrix cores' full rate, which the 16x16 shapes do not reach.
template <int DT>
__device__ __forceinline__ f32x16_t mfma_32x32(const uint4 &a, const uint4 &b, f32x16_t c)
{
    if constexpr (DT == RLHF_BF16)
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a),
                                                      __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
}

// Same with 16 contraction entries, 4 per lane (entries 4*(l/16) .. +3).
template <int DT>
__device__ __forceinline__ f32x4_t mfma_k16(const uint2 &a, const uint2 &b, f32x4_t c)
{
    if constexpr (DT == RLHF_BF16)
        return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a),
                                                         __builtin_bit_cast(s16x4_t, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x16f16(__builtin_bit_cast(f16x4_t, a),
                                                     __builtin_bit_cast(f16x4_t, b), c, 0, 0, 0);
}

// Splits two fp32 probabilities into packed 16-bit high parts and packed 16-bit
// remainders: p ~= hi + lo with relative error about 2^-16 (bf16) or better.
template <int DT>
__device__ __forceinline__ void split_pair(float p0, float p1, uint32_t &hi, uint32_t &lo)
{
    if constexpr (DT == RLHF_BF16) {
        const uint32_t u0 = __float_as_uint(p0), u1 = __float_as_uint(p1);
        hi = (u0 >> 16) | (u1 & 0xffff0000u);
        const float r0 = p0 - __uint_as_float(u0 & 0xffff0000u);  // exact
        const float r1 = p1 - __uint_as_float(u1 & 0xffff0000u);
        lo = (__float_as_uint(r0) >> 16) | (__float_as_uint(r1) & 0xffff0000u);
    } else {
        const _Float16 h0 = (_Float16)p0, h1 = (_Float16)p1;
        const _Float16 l0 = (_Float16)(p0 - (float)h0), l1 = (_Float16)(p1 - (float)h1);
        hi = (uint32_t)__builtin_bit_cast(uint16_t, h0) | ((uint32_t)__builtin_bit_cast(uint16_t, h1) << 16);
        lo = (uint32_t)__builtin_bit_cast(uint16_t, l0) | ((uint32_t)__builtin_bit_cast(uint16_t, l1) << 16);
    }
}

}  // namespace rlhf
