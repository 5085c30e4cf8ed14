// Device helpers: element conversion and the float32 quantiser steps.
#pragma once

#include "bq_internal.h"

namespace bq {

struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(__half v) { return __half2float(v); }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float((uint32_t)v.bits << 16); }

template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v)
{
    return v;
}
template <>
__device__ __forceinline__ __half from_float<__half>(float v)
{
    return __float2half_rn(v);
}
// float32 -> bfloat16, round to nearest even: the hardware conversion (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float v) { return __builtin_bit_cast(uint16_t, (__bf16)v); }
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_bits(float lo, float hi)
{
    typedef float float2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const float2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
// two float32 -> two binary16 in one register, round to nearest even: one v_cvt_pk_f16_f32
__device__ __forceinline__ uint32_t f32x2_to_f16x2_bits(float lo, float hi)
{
    typedef float float2_t __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
    const float2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
}
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float v)
{
    bf16_t r;
    r.bits = f32_to_bf16_bits(v);
    return r;
}

// Scale of one quantisation group from its abs-max; every step is one correctly rounded float32
// operation (the contract stated in bq.h).  Returns the stored scale; *inv receives 1/s (0 if s == 0).
__device__ __forceinline__ float group_scale(float amax, float qmax, bool scale_f16, float *inv)
{
    float s = amax / qmax;
    if (scale_f16) {
        s = fminf(s, 65504.0f);
        s = __half2float(__float2half_rn(s));
    }
    *inv = (s == 0.0f) ? 0.0f : 1.0f / s;
    return s;
}

__device__ __forceinline__ int quant_code(float v, float inv, float qmin, float qmax)
{
    float q = rintf(v * inv);
    q = fminf(fmaxf(q, qmin), qmax);
    return (int)q;
}

}  // namespace bq
