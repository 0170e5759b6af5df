// Internal helpers shared by the translation units of libmkq (host side checks,
// launch plumbing, small device utilities).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "mkq.h"

namespace mkq {

constexpr int QMIN = -8;
constexpr int QMAX = 7;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool scale_ok(float s) { return s > 0.0f && s < __builtin_inff(); }
inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }
inline int launch_status() { return hipGetLastError() == hipSuccess ? MKQ_OK : MKQ_ERR_HIP; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- device utilities ------------------------------------------------------

// Eq. 1, integer part, for one value: binary32 divide, clamp to the signed
// 4-bit range, round half to even.  NaN -> 0.
__device__ __forceinline__ int quantize_code(float x, float s)
{
    float v = x / s;                    // correctly rounded (no fast-math)
    v = (v != v) ? 0.0f : v;
    v = fminf(fmaxf(v, (float)QMIN), (float)QMAX);
    return (int)__builtin_rintf(v);     // v_rndne_f32
}

// Eq. 1 at 8 bits: clamp to [-128, 127]; 8 codes as 8 bytes, element 0 lowest.
__device__ __forceinline__ int quantize_code8(float x, float s)
{
    float v = x / s;
    v = (v != v) ? 0.0f : v;
    v = fminf(fmaxf(v, -128.0f), 127.0f);
    return (int)__builtin_rintf(v);
}

__device__ __forceinline__ uint2 bytes8(const int (&c)[8])
{
    uint32_t lo = 0, hi = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        lo |= ((uint32_t)c[i] & 0xFFu) << (8 * i);
        hi |= ((uint32_t)c[4 + i] & 0xFFu) << (8 * i);
    }
    return make_uint2(lo, hi);
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h)
{
    return __half2float(__ushort_as_half(h));
}

__device__ __forceinline__ uint16_t float_to_half_bits(float f)
{
    return __half_as_ushort(__float2half_rn(f));
}

// binary32 -> bfloat16, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7F800000u) == 0x7F800000u) {
        if (u & 0x007FFFFFu) u |= 0x00400000u;
        return (uint16_t)(u >> 16);
    }
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// 8 consecutive elements of a binary32 / binary16 row as binary32 (16-byte aligned address).
template <typename T>
__device__ __forceinline__ void load8(const T *p, float (&v)[8]);

template <>
__device__ __forceinline__ void load8<float>(const float *p, float (&v)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
    v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}

template <>
__device__ __forceinline__ void load8<__half>(const __half *p, float (&v)[8])
{
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = half_bits_to_float((uint16_t)(w[i] & 0xFFFFu));
        v[2 * i + 1] = half_bits_to_float((uint16_t)(w[i] >> 16));
    }
}

// Two binary32 values -> two 16-bit floats in one word (low half = a), round to
// nearest even, one v_cvt_pk_* instruction each on gfx950.
typedef float mkq_f2 __attribute__((ext_vector_type(2)));
typedef __bf16 mkq_bf2 __attribute__((ext_vector_type(2)));
typedef _Float16 mkq_h2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack2_bf16(float a, float b)
{
    const mkq_f2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, mkq_bf2));
}
__device__ __forceinline__ uint32_t pack2_f16(float a, float b)
{
    const mkq_f2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, mkq_h2));
}

// erf in binary32 without branches: the exponential-times-polynomial form of Abramowitz &
// Stegun 7.1.26, erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x) for x >= 0
// (absolute error of the formula <= 1.5e-7; v_rcp_f32 and v_exp_f32 add about 1e-7).
__device__ __forceinline__ float erf_as(float x)
{
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, ax, 1.0f));
    float p = __builtin_fmaf(1.061405429f, t, -1.453152027f);
    p = __builtin_fmaf(p, t, 1.421413741f);
    p = __builtin_fmaf(p, t, -0.284496736f);
    p = __builtin_fmaf(p, t, 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f(ax * ax * -1.4426950408889634f);
    return __builtin_copysignf(__builtin_fmaf(-p, e, 1.0f), x);
}

// GELU, erf form, binary32 (activation functions stay in float32, section 5).
__device__ __forceinline__ float gelu_erf(float x)
{
    return 0.5f * x * (1.0f + erf_as(x * 0.70710678118654752440f));
}

}  // namespace mkq
