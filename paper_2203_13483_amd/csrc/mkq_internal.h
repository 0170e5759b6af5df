// Internal helpers shared by the translation units of libmkq (host side checks,
// launch plumbing, small device utilities).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include <mutex>

#include "mkq.h"

namespace mkq {

constexpr int QMIN = -8;
constexpr int QMAX = 7;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool scale_ok(float s) { return s > 0.0f && s < __builtin_inff(); }
// Every entry point converts its stream argument here before it launches anything.  The runtime keeps the
// last error of the thread until somebody reads it: one left behind by an earlier call of the process (not
// ours, and handled or ignored there) must not be taken for a failure of our launch, so it is read away here.
inline hipStream_t as_stream(void *s)
{
    (void)hipGetLastError();
    return reinterpret_cast<hipStream_t>(s);
}
inline int launch_status() { return hipGetLastError() == hipSuccess ? MKQ_OK : MKQ_ERR_HIP; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Per-device, once-only setup values (dynamic LDS limits, resident workgroups per CU, CU counts).
// One object per kernel instantiation; get() runs `init` the first time it is called with a given
// device current and returns its (positive) result from then on; a result <= 0 is an error and is
// not cached.  Safe to call from several threads.
constexpr int MAX_DEVICES = 64;
struct PerDeviceOnce {
    std::mutex mu;
    int val[MAX_DEVICES] = {};
    template <class F>
    int get(F &&init)
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return -1;
        std::lock_guard<std::mutex> lock(mu);
        if (val[dev] <= 0) {
            const int v = init();
            if (v <= 0) return v < 0 ? v : -1;
            val[dev] = v;
        }
        return val[dev];
    }
};

// Compute units of the current device; false if the runtime cannot say.
inline bool device_cus(int *cus)
{
    static PerDeviceOnce once;
    const int v = once.get([]() -> int {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return -1;
        return n;
    });
    if (v <= 0) return false;
    *cus = v;
    return true;
}

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

// The same code for many values under one step, without a division per value.  With rs = RN(1/s),
// q = RN(x * rs) differs from the exact quotient x/s by at most |x/s| * 2^-23 (two roundings), and the
// correctly rounded quotient differs from it by at most |x/s| * 2^-24; inside the clamp range that is
// less than `margin` in all.  So unless q lies within `margin` of a rounding boundary k + 1/2, the
// correctly rounded quotient rounds to the same integer (values beyond the clamp range clamp alike);
// the rare value that does lie that close takes the division.  For steps outside [2^-100, 2^100]
// (where 1/s could lose precision) the threshold is negative and every value takes the division.
struct QuantStep {
    float s, rs, thr;
};
template <int BITS>
__device__ __forceinline__ QuantStep quant_step(float s)
{
    // (covers both forms below: 1.5 * 2^-23 * 9 resp. * 129 for the plain product, 33.5 * 2^-24 resp.
    // 513.5 * 2^-24 for the biased one; rounded up)
    constexpr float margin = (BITS == 4) ? 4.0e-6f : 5.0e-5f;
    QuantStep q;
    q.s = s;
    q.rs = 1.0f / s;
    q.thr = (s >= 0x1p-100f && s <= 0x1p100f) ? 0.5f - margin : -1.0f;
    return q;
}
template <int BITS>
__device__ __forceinline__ int quantize_code_rs(float x, const QuantStep &q)
{
    constexpr float lo = (BITS == 4) ? (float)QMIN : -128.0f, hi = (BITS == 4) ? (float)QMAX : 127.0f;
    float v = x * q.rs;
    v = (v != v) ? 0.0f : v;
    v = fminf(fmaxf(v, lo), hi);
    const float r = __builtin_rintf(v);
    if (__builtin_expect(fabsf(v - r) > q.thr, 0)) {
        float w = x / q.s;
        w = (w != w) ? 0.0f : w;
        w = fminf(fmaxf(w, lo), hi);
        return (int)__builtin_rintf(w);
    }
    return (int)r;
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

// Eq. 1 for eight values under one step, packed as they are stored: BITS = 4 -> eight nibbles in .x (value 0
// lowest), BITS = 8 -> eight bytes in .x, .y.  Division-free as above, in a form that takes six vector
// operations per value: v = fma(x, rs, 2^(BITS-1)) is the quotient moved to [0, 2^BITS - 1] (one rounding;
// for quotients inside the clamp range it differs from the correctly rounded x / s plus the bias by less
// than `margin`), it is rounded, clamped and written into its byte by one conversion instruction, and the
// bias comes off all codes at once as a flip of their sign bits.  If any of the eight lies within `margin`
// of a rounding boundary, or is NaN or infinite (v - rint(v) is then NaN), all eight take the division.
template <int BITS>
__device__ __forceinline__ uint2 quantize8(const float (&x)[8], const QuantStep &q)
{
    constexpr float bias = (BITS == 4) ? 8.0f : 128.0f, top = (BITS == 4) ? 15.0f : 255.0f;
    uint32_t a = 0, b = 0;
    bool divide = false;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float v = __builtin_fmaf(x[e], q.rs, bias);
        const float r = __builtin_rintf(v);
        divide |= !(fabsf(v - r) <= q.thr);
        const float c = __builtin_amdgcn_fmed3f(r, 0.0f, top);
        // 4 bits: even values in the bytes of a, odd ones in b; 8 bits: values 0..3 in a, 4..7 in b
        const bool to_b = (BITS == 4) ? (e & 1) : (e >= 4);
        const unsigned at = (BITS == 4) ? (e >> 1) : (e & 3);
        if (to_b) b = __builtin_amdgcn_cvt_pk_u8_f32(c, at, b);
        else a = __builtin_amdgcn_cvt_pk_u8_f32(c, at, a);
    }
    uint2 out = (BITS == 4) ? make_uint2((a | (b << 4)) ^ 0x88888888u, 0u)
                            : make_uint2(a ^ 0x80808080u, b ^ 0x80808080u);
    if (__builtin_expect(divide, 0)) {
        int cd[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) cd[e] = (BITS == 4) ? quantize_code(x[e], q.s) : quantize_code8(x[e], q.s);
        if (BITS == 4) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) packed |= ((uint32_t)cd[e] & 0xFu) << (4 * e);
            out = make_uint2(packed, 0u);
        } else {
            out = bytes8(cd);
        }
    }
    return out;
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

// GELU, erf form, binary32 (activation functions stay in float32, section 5), without branches.
// erf comes from the exponential-times-polynomial form of Abramowitz & Stegun 7.1.26,
// erf(z) = 1 - (a1 t + ... + a5 t^5) exp(-z^2), t = 1 / (1 + p z) for z >= 0 (absolute error of the
// formula <= 1.5e-7; v_rcp_f32 and v_exp_f32 add about 1e-7).  With z = |x| / sqrt(2) folded into the
// constants, Phi(x) = 1 - u for x >= 0 and u for x < 0, u = (a1 t + ... + a5 t^5) exp(-x^2 / 2) / 2,
// so  gelu(x) = x Phi(x) = max(x, 0) - |x| u.
__device__ __forceinline__ float gelu_erf(float x)
{
    const float ax = fabsf(x);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f * 0.70710678118654752440f, ax, 1.0f));
    float p = __builtin_fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
    p = __builtin_fmaf(p, t, 0.5f * 1.421413741f);
    p = __builtin_fmaf(p, t, 0.5f * -0.284496736f);
    p = __builtin_fmaf(p, t, 0.5f * 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f(x * x * (-0.5f * 1.4426950408889634f));
    // max(x, 0) as a median of three: one instruction (fmaxf first quiets its operand with a second one); a
    // NaN still reaches the result through the product
    return __builtin_fmaf(-ax, p * e, __builtin_amdgcn_fmed3f(x, 0.0f, __builtin_inff()));
}

}  // namespace mkq
