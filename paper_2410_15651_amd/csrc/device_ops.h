// Device-side building blocks for gfx950 (wave64): 16-bit float unpacking,
// DPP row reductions, packed dot products.  Everything here is inline.
#pragma once

#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

#include "rlhf_rollout.h"

namespace rlhf {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

__device__ __forceinline__ float fast_exp2(float x)
{
    return __builtin_amdgcn_exp2f(x);  // v_exp_f32: exp2(-inf) = 0, no range fix-up code
}

// ---- 16-bit storage -> fp32 ------------------------------------------------
// A dword holds two 16-bit elements; `lo` is the element at the lower address.
template <int DT>
__device__ __forceinline__ float unpack_lo(uint32_t w)
{
    if constexpr (DT == RLHF_BF16) {
        return __uint_as_float(w << 16);
    } else {
        return (float)__builtin_bit_cast(f16x2_t, w)[0];
    }
}

template <int DT>
__device__ __forceinline__ float unpack_hi(uint32_t w)
{
    if constexpr (DT == RLHF_BF16) {
        return __uint_as_float(w & 0xffff0000u);
    } else {
        return (float)__builtin_bit_cast(f16x2_t, w)[1];
    }
}

template <int DT>
__device__ __forceinline__ float load_scalar(const void *base, int64_t idx)
{
    if constexpr (DT == RLHF_F32) {
        return ((const float *)base)[idx];
    } else if constexpr (DT == RLHF_BF16) {
        return __uint_as_float((uint32_t)((const uint16_t *)base)[idx] << 16);
    } else {
        return (float)((const _Float16 *)base)[idx];
    }
}

// fp32 -> 16-bit storage, round to nearest even (one conversion instruction, no branch: bf16 has its
// own on this device; NaN stays NaN, quiet).
template <int DT>
__device__ __forceinline__ uint16_t pack16(float x)
{
    if constexpr (DT == RLHF_BF16) {
        return __builtin_bit_cast(uint16_t, (__bf16)x);  // v_cvt_pk_bf16_f32
    } else {
        // The value is rounded to fp32 first and to fp16 second, always: the empty
        // statement keeps the compiler from folding the caller's last multiply into a
        // mixed-precision instruction that rounds once (the two can differ in the last
        // bit, and one call site may get the fold while another does not).
        asm volatile("" : "+v"(x));
        _Float16 h = (_Float16)x;  // v_cvt_f16_f32, RNE
        return __builtin_bit_cast(uint16_t, h);
    }
}

// Two fp32 -> two 16-bit values in one word, `first` in the low half, with one packed conversion.
template <int DT>
__device__ __forceinline__ uint32_t pack16x2(float first, float second)
{
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    if constexpr (DT == RLHF_BF16) {
        const f32x2_t v = {first, second};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));  // v_cvt_pk_bf16_f32
    } else {
        asm volatile("" : "+v"(first), "+v"(second));  // see pack16
        const f32x2_t v = {first, second};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));  // v_cvt_pk_f16_f32
    }
}

// c + a.lo*b.lo + a.hi*b.hi with fp32 accumulation (v_dot2_f32_bf16 / v_dot2_f32_f16).
template <int DT>
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c)
{
    if constexpr (DT == RLHF_BF16) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a),
                                               __builtin_bit_cast(bf16x2_t, b), c, false);
    } else {
        return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a),
                                      __builtin_bit_cast(f16x2_t, b), c, false);
    }
}

// ---- DPP moves within a row of 16 lanes -------------------------------------
constexpr int kDppQuadXor1 = 0xB1;       // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm [2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppRowMirror = 0x140;     // lane i <-> 15-i inside each 16

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum / max over each row of 16 lanes; every lane of the row gets the result.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_move<kDppQuadXor1>(v);
    v += dpp_move<kDppQuadXor2>(v);
    v += dpp_move<kDppRowHalfMirror>(v);
    v += dpp_move<kDppRowMirror>(v);
    return v;
}

__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, dpp_move<kDppQuadXor1>(v));
    v = fmaxf(v, dpp_move<kDppQuadXor2>(v));
    v = fmaxf(v, dpp_move<kDppRowHalfMirror>(v));
    v = fmaxf(v, dpp_move<kDppRowMirror>(v));
    return v;
}

// Whole-wavefront reductions; the result is wave-uniform (read out of lanes
// 0, 16, 32, 48 after the row step).
__device__ __forceinline__ float wave_sum(float v)
{
    v = row16_sum(v);
    float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return (a + b) + (c + d);
}

__device__ __forceinline__ float wave_max(float v)
{
    v = row16_max(v);
    float a = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float b = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float c = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float d = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return fmaxf(fmaxf(a, b), fmaxf(c, d));
}

__device__ __forceinline__ float lane_bcast(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// 16-byte streaming load.  Every byte of K, V and the logits is used exactly
// once per call, so the loads are marked non-temporal: on MI355X a plain
// 128-bit read stream tops out near 6.3 TB/s, the same stream with the
// non-temporal hint near 7.1 TB/s.  Kept in one place so that the cache policy
// of all streaming reads changes together.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 load16(const void *p)
{
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

}  // namespace rlhf
