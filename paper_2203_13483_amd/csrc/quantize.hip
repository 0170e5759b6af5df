// Quantizer kernels: activation quantize + pack, abs-max calibration, offline
// weight quantize + pack, code pack / unpack.  All are streaming kernels bound by
// HBM bandwidth; each thread produces one 32-bit word (8 codes) per step so that
// a wavefront reads 2 KiB (binary32 input) and writes 256 B, both contiguous.
#include "mkq_internal.h"

namespace mkq {

// Packs 8 codes (element k in bits [4k, 4k+4)) -- this is the canonical layout:
// byte k/2 holds element k in its low nibble for even k, high nibble for odd k.
__device__ __forceinline__ uint32_t pack8(const int (&c)[8])
{
    uint32_t w = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) w |= ((uint32_t)c[i] & 0xFu) << (4 * i);
    return w;
}

// Eq. 1 with a per-tensor step: x [M,K] (row stride ldx) -> packed codes [M,Kp/2]; codes K .. Kp-1 of a
// row are zero (Kp >= K: a row padded to the GEMM's granularity of k adds nothing to any dot product).
template <typename T>
__global__ __launch_bounds__(256) void quantize_kernel(const T *__restrict__ x, int64_t M, int64_t K,
                                                       int64_t ldx, float s,
                                                       uint32_t *__restrict__ q, int64_t Kp)
{
    const int64_t words_per_row = Kp / 8;
    const int64_t total = M * words_per_row;
    const QuantStep qs = quant_step<4>(s);  // the division's decision without dividing every value
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total;
         w += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = w / words_per_row;
        const int64_t kw = w - m * words_per_row;
        if (kw * 8 >= K) {
            q[w] = 0u;
            continue;
        }
        float v[8];
        load8<T>(x + m * ldx + kw * 8, v);
        int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = quantize_code_rs<4>(v[i], qs);
        q[w] = pack8(c);
    }
}

// The same for contiguous rows (ldx == K) and fewer than 2^31 words: no row/column split
// (a 64-bit division per word in the general kernel), two words per thread with both loads
// in flight before the arithmetic starts.
template <typename T>
__global__ __launch_bounds__(256) void quantize_contig_kernel(const T *__restrict__ x, int total_words, float s,
                                                              uint32_t *__restrict__ q)
{
    const int stride = (int)(gridDim.x * blockDim.x);
    const int w0 = (int)(blockIdx.x * blockDim.x + threadIdx.x);
    const int w1 = w0 + stride;
    if (w0 >= total_words) return;
    const bool two = w1 < total_words;
    float v0[8], v1[8];
    load8<T>(x + (int64_t)w0 * 8, v0);
    load8<T>(x + (int64_t)(two ? w1 : w0) * 8, v1);
    const QuantStep qs = quant_step<4>(s);
    int c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = quantize_code_rs<4>(v0[i], qs);
    q[w0] = pack8(c);
    if (two) {
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = quantize_code_rs<4>(v1[i], qs);
        q[w1] = pack8(c);
    }
}

// max |x| over a block's share, combined with an atomic max on the bit pattern
// (non-negative floats order like unsigned integers).  *acc_bits must be 0 on entry.
template <typename T>
__global__ __launch_bounds__(256) void absmax_tensor_kernel(const T *__restrict__ x, int64_t M,
                                                            int64_t K, int64_t ldx,
                                                            uint32_t *__restrict__ acc_bits)
{
    __shared__ float part[4];
    const int64_t groups_per_row = K / 8;
    const int64_t total = M * groups_per_row;
    float mx = 0.0f;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total;
         w += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = w / groups_per_row;
        const int64_t kw = w - m * groups_per_row;
        float v[8];
        load8<T>(x + m * ldx + kw * 8, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(v[i]));  // fmaxf drops NaN
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        mx = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        atomicMax(acc_bits, __float_as_uint(mx));
    }
}

__global__ void fill_zero_kernel(uint32_t *p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// In place: bits of max|x|  ->  step  max|x| / 7  (1 when the maximum is 0).
__global__ void finalize_scale_kernel(float *s, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        const float mx = s[i];
        s[i] = (mx > 0.0f) ? mx / (float)QMAX : 1.0f;
    }
}

// One workgroup per row: block max of |x| (used for per-row calibration and for
// weight rows).  Returns the row maximum to every thread.
template <typename T>
__device__ __forceinline__ float row_absmax(const T *__restrict__ row, int64_t K, float *part)
{
    float mx = 0.0f;
    for (int64_t k = (int64_t)threadIdx.x * 8; k < K; k += (int64_t)blockDim.x * 8) {
        float v[8];
        load8<T>(row + k, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(v[i]));
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    __syncthreads();
    return mx;
}

template <typename T>
__global__ __launch_bounds__(256) void absmax_rows_kernel(const T *__restrict__ x, int64_t K,
                                                          int64_t ldx, float *__restrict__ s_out)
{
    __shared__ float part[4];
    const float mx = row_absmax<T>(x + (int64_t)blockIdx.x * ldx, K, part);
    if (threadIdx.x == 0) s_out[blockIdx.x] = (mx > 0.0f) ? mx / (float)QMAX : 1.0f;
}

// Offline weight preparation, one workgroup per output channel: calibrate (or
// take) the row's step, then Eq. 1 and pack.
__global__ __launch_bounds__(256) void pack_weights_kernel(const float *__restrict__ W, int64_t K,
                                                           const float *__restrict__ s_in,
                                                           float *__restrict__ s_out,
                                                           uint32_t *__restrict__ q, int64_t Kp)
{
    __shared__ float part[4];
    const int64_t n = blockIdx.x;
    const float *row = W + n * K;
    float s;
    if (s_in) {
        s = s_in[n];
    } else {
        const float mx = row_absmax<float>(row, K, part);
        s = (mx > 0.0f) ? mx / (float)QMAX : 1.0f;
    }
    if (threadIdx.x == 0) s_out[n] = s;
    uint32_t *qrow = q + n * (Kp / 8);  // codes K .. Kp-1 are zero
    for (int64_t k = (int64_t)threadIdx.x * 8; k < Kp; k += (int64_t)blockDim.x * 8) {
        if (k >= K) {
            qrow[k / 8] = 0u;
            continue;
        }
        float v[8];
        load8<float>(row + k, v);
        int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = quantize_code(v[i], s);
        qrow[k / 8] = pack8(c);
    }
}

__global__ __launch_bounds__(256) void pack_codes_kernel(const int8_t *__restrict__ codes,
                                                         int64_t total_words,
                                                         uint32_t *__restrict__ q)
{
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total_words;
         w += (int64_t)gridDim.x * blockDim.x) {
        const uint2 raw = *reinterpret_cast<const uint2 *>(codes + w * 8);
        int c[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            c[i] = (int)((raw.x >> (8 * i)) & 0xFFu);
            c[4 + i] = (int)((raw.y >> (8 * i)) & 0xFFu);
        }
        q[w] = pack8(c);
    }
}

__global__ __launch_bounds__(256) void unpack_codes_kernel(const uint32_t *__restrict__ q,
                                                           int64_t total_words,
                                                           int8_t *__restrict__ codes)
{
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total_words;
         w += (int64_t)gridDim.x * blockDim.x) {
        const uint32_t v = q[w];
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            // sign-extend each nibble to a byte
            const int a = ((int)(v << (28 - 4 * i))) >> 28;
            const int b = ((int)(v << (12 - 4 * i))) >> 28;
            lo |= ((uint32_t)a & 0xFFu) << (8 * i);
            hi |= ((uint32_t)b & 0xFFu) << (8 * i);
        }
        *reinterpret_cast<uint2 *>(codes + w * 8) = make_uint2(lo, hi);
    }
}

// ---- 8-bit range (the comparison column of Table 2; mixed 4/8-bit models of section 4.2) ----
// Eq. 1 with k = 8: clamp to [-128, 127], one byte per code, no packing.

// x [M,K] (row stride ldx) -> int8 codes [M,K]; each thread turns 8 values into 8 bytes.
template <typename T>
__global__ __launch_bounds__(256) void quantize8_kernel(const T *__restrict__ x, int64_t M, int64_t K,
                                                        int64_t ldx, float s, uint2 *__restrict__ q)
{
    const int64_t groups_per_row = K / 8;
    const int64_t total = M * groups_per_row;
    const QuantStep qs = quant_step<8>(s);
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total;
         g += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = g / groups_per_row;
        const int64_t kg = g - m * groups_per_row;
        float v[8];
        load8<T>(x + m * ldx + kg * 8, v);
        int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = quantize_code_rs<8>(v[i], qs);
        q[g] = bytes8(c);
    }
}

// One workgroup per output channel: step = max|row| / 127 (or the given one), then codes.
__global__ __launch_bounds__(256) void pack_weights8_kernel(const float *__restrict__ W, int64_t K,
                                                            const float *__restrict__ s_in,
                                                            float *__restrict__ s_out,
                                                            uint2 *__restrict__ q)
{
    __shared__ float part[4];
    const int64_t n = blockIdx.x;
    const float *row = W + n * K;
    float s;
    if (s_in) {
        s = s_in[n];
    } else {
        const float mx = row_absmax<float>(row, K, part);
        s = (mx > 0.0f) ? mx / 127.0f : 1.0f;
    }
    if (threadIdx.x == 0) s_out[n] = s;
    uint2 *qrow = q + n * (K / 8);
    for (int64_t k = (int64_t)threadIdx.x * 8; k < K; k += (int64_t)blockDim.x * 8) {
        float v[8];
        load8<float>(row + k, v);
        int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = quantize_code8(v[i], s);
        qrow[k / 8] = bytes8(c);
    }
}

// ---- E3M2 containers (experimental 6-bit float path of the GEMM) ------------------------------
// A code c in [-8, 8] as a 6-bit float: sign, 3 exponent bits (bias 3), 2 mantissa bits.  The nine
// magnitudes, 6 bits each, sit in one 64-bit constant.
__device__ __forceinline__ uint32_t e3m2_of_code(int c)
{
    constexpr unsigned long long MAG = 0x00ull | (0x0Cull << 6) | (0x10ull << 12) | (0x12ull << 18) | (0x14ull << 24) |
                                       (0x15ull << 30) | (0x16ull << 36) | (0x17ull << 42) | (0x18ull << 48);
    const int m = c < 0 ? -c : c;
    return (uint32_t)((MAG >> (6 * m)) & 0x3Full) | (c < 0 ? 0x20u : 0u);
}

// 16 codes -> 96 bits, code i in bits [6i, 6i + 6)
__device__ __forceinline__ void pack16_e3m2(const int (&c)[16], uint32_t (&w)[3])
{
    uint32_t e[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) e[i] = e3m2_of_code(c[i]);
    w[0] = e[0] | (e[1] << 6) | (e[2] << 12) | (e[3] << 18) | (e[4] << 24) | (e[5] << 30);
    w[1] = (e[5] >> 2) | (e[6] << 4) | (e[7] << 10) | (e[8] << 16) | (e[9] << 22) | (e[10] << 28);
    w[2] = (e[10] >> 4) | (e[11] << 2) | (e[12] << 8) | (e[13] << 14) | (e[14] << 20) | (e[15] << 26);
}

// Container layout: a row is groups of 64 codes = 48 bytes.  The 32 codes of half h of a group form a
// 192-bit little-endian stream (code i in bits [6i, 6i + 6)) -- one matrix-core operand of a lane --
// stored as bytes [16h, 16h + 16) then [32 + 8h, 32 + 8h + 8) of the group, so that a lane fetches its
// operand with one aligned 16-byte and one 8-byte read.  This writes half `half` (0 / 1) of group `g`.
__device__ __forceinline__ void store_half_e3m2(uint8_t *group, int half, const int (&c)[32])
{
    int lo[16], hi[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        lo[i] = c[i];
        hi[i] = c[16 + i];
    }
    uint32_t a[3], b[3];
    pack16_e3m2(lo, a);
    pack16_e3m2(hi, b);
    *reinterpret_cast<uint4 *>(group + 16 * half) = make_uint4(a[0], a[1], a[2], b[0]);
    *reinterpret_cast<uint2 *>(group + 32 + 8 * half) = make_uint2(b[1], b[2]);
}

// Eq. 1 then the container: x [M, K] -> [M, 3K/4] bytes; one thread per 32 values (half a group)
template <typename T>
__global__ __launch_bounds__(256) void quantize_e3m2_kernel(const T *__restrict__ x, int64_t M, int64_t K, int64_t ldx,
                                                            float s, uint8_t *__restrict__ q)
{
    const int64_t halves_per_row = K / 32;
    const int64_t total = M * halves_per_row;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total;
         g += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = g / halves_per_row;
        const int64_t kh = g - m * halves_per_row;
        int c[32];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v[8];
            load8<T>(x + m * ldx + kh * 32 + j * 8, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) c[8 * j + i] = quantize_code(v[i], s);
        }
        store_half_e3m2(q + m * (K / 4 * 3) + (kh >> 1) * 48, (int)(kh & 1), c);
    }
}

// int8 codes [rows, K] (values in [-8, 8]) -> containers
__global__ __launch_bounds__(256) void pack_codes_e3m2_kernel(const int8_t *__restrict__ codes, int64_t total_halves,
                                                              uint8_t *__restrict__ q)
{
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total_halves;
         g += (int64_t)gridDim.x * blockDim.x) {
        int c[32];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(codes + g * 32 + j * 16);
            const uint32_t rw[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int i = 0; i < 16; ++i) c[16 * j + i] = (int)(int8_t)(rw[i >> 2] >> (8 * (i & 3)));
        }
        // rows are whole groups, so half g of the flat array is half g % 2 of group g / 2
        store_half_e3m2(q + (g >> 1) * 48, (int)(g & 1), c);
    }
}

// Offline weight preparation into containers, one workgroup per output channel
__global__ __launch_bounds__(256) void pack_weights_e3m2_kernel(const float *__restrict__ W, int64_t K,
                                                                const float *__restrict__ s_in,
                                                                float *__restrict__ s_out, uint8_t *__restrict__ q)
{
    __shared__ float part[4];
    const int64_t n = blockIdx.x;
    const float *row = W + n * K;
    float s;
    if (s_in) {
        s = s_in[n];
    } else {
        const float mx = row_absmax<float>(row, K, part);
        s = (mx > 0.0f) ? mx / (float)QMAX : 1.0f;
    }
    if (threadIdx.x == 0) s_out[n] = s;
    uint8_t *qrow = q + n * (K / 4 * 3);
    for (int64_t kh = threadIdx.x; kh < K / 32; kh += blockDim.x) {
        int c[32];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float v[8];
            load8<float>(row + kh * 32 + j * 8, v);
#pragma unroll
            for (int i = 0; i < 8; ++i) c[8 * j + i] = quantize_code(v[i], s);
        }
        store_half_e3m2(qrow + (kh >> 1) * 48, (int)(kh & 1), c);
    }
}

static inline int grid_for(int64_t items, int threads = 256, int max_blocks = 256 * 16)
{
    int64_t b = ceil_div(items, threads);
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return (int)b;
}

}  // namespace mkq

using namespace mkq;

extern "C" int mkq_quantize(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                            float s_x, uint8_t *q_out, void *stream)
{
    if (x_dtype != MKQ_F32 && x_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (M < 0 || K < 0 || (K % 32) != 0 || ldx < K || (ldx % 8) != 0) return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (M == 0 || K == 0) return MKQ_OK;  // empty tensors may come with NULL pointers
    if (!x || !q_out) return MKQ_ERR_NULL;
    if (!aligned16(x) || !aligned16(q_out)) return MKQ_ERR_ALIGN;
    const int64_t words = M * (K / 8);
    if (ldx == K && words < 0x40000000LL) {
        const int g = (int)ceil_div(ceil_div(words, 2), 256);
        if (x_dtype == MKQ_F32)
            quantize_contig_kernel<float><<<g, 256, 0, as_stream(stream)>>>((const float *)x, (int)words, s_x,
                                                                             (uint32_t *)q_out);
        else
            quantize_contig_kernel<__half><<<g, 256, 0, as_stream(stream)>>>((const __half *)x, (int)words, s_x,
                                                                              (uint32_t *)q_out);
        return launch_status();
    }
    const int grid = grid_for(words);
    if (x_dtype == MKQ_F32)
        quantize_kernel<float><<<grid, 256, 0, as_stream(stream)>>>(
            (const float *)x, M, K, ldx, s_x, (uint32_t *)q_out, K);
    else
        quantize_kernel<__half><<<grid, 256, 0, as_stream(stream)>>>(
            (const __half *)x, M, K, ldx, s_x, (uint32_t *)q_out, K);
    return launch_status();
}

extern "C" int64_t mkq_padded_k(int64_t K)
{
    return K <= 0 ? 0 : (K + 127) / 128 * 128;  // whole 64-byte stages: the fast tile kernels apply
}

extern "C" int mkq_quantize_padded(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                                   float s_x, uint8_t *q_out, void *stream)
{
    if (x_dtype != MKQ_F32 && x_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (M < 0 || K < 0 || (K % 8) != 0 || ldx < K || (ldx % 8) != 0) return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (M == 0 || K == 0) return MKQ_OK;
    if (!x || !q_out) return MKQ_ERR_NULL;
    if (!aligned16(x) || !aligned16(q_out)) return MKQ_ERR_ALIGN;
    const int64_t Kp = mkq_padded_k(K);
    const int grid = grid_for(M * (Kp / 8));
    if (x_dtype == MKQ_F32)
        quantize_kernel<float><<<grid, 256, 0, as_stream(stream)>>>(
            (const float *)x, M, K, ldx, s_x, (uint32_t *)q_out, Kp);
    else
        quantize_kernel<__half><<<grid, 256, 0, as_stream(stream)>>>(
            (const __half *)x, M, K, ldx, s_x, (uint32_t *)q_out, Kp);
    return launch_status();
}

extern "C" int mkq_absmax_scale(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                                int per_row, float *s_out, void *stream)
{
    if (!x || !s_out) return MKQ_ERR_NULL;
    if (x_dtype != MKQ_F32 && x_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (M <= 0 || K <= 0 || (K % 8) != 0 || ldx < K || (ldx % 8) != 0) return MKQ_ERR_SHAPE;
    if (M > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(s_out) & 3u)) return MKQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    if (per_row) {
        if (x_dtype == MKQ_F32)
            absmax_rows_kernel<float><<<(int)M, 256, 0, st>>>((const float *)x, K, ldx, s_out);
        else
            absmax_rows_kernel<__half><<<(int)M, 256, 0, st>>>((const __half *)x, K, ldx, s_out);
        return launch_status();
    }
    fill_zero_kernel<<<1, 64, 0, st>>>((uint32_t *)s_out, 1);
    const int grid = grid_for(M * (K / 8), 256, 1024);
    if (x_dtype == MKQ_F32)
        absmax_tensor_kernel<float><<<grid, 256, 0, st>>>((const float *)x, M, K, ldx, (uint32_t *)s_out);
    else
        absmax_tensor_kernel<__half><<<grid, 256, 0, st>>>((const __half *)x, M, K, ldx, (uint32_t *)s_out);
    finalize_scale_kernel<<<1, 64, 0, st>>>(s_out, 1);
    return launch_status();
}

extern "C" size_t mkq_packed_weight_bytes(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0 || (K % 32) != 0) return 0;
    return (size_t)N * (size_t)(K / 2);
}

extern "C" int mkq_pack_weights_int4(const float *W, int64_t N, int64_t K, const float *s_w_in,
                                     float *s_w_out, uint8_t *Wq_out, void *stream)
{
    if (!W || !s_w_out || !Wq_out) return MKQ_ERR_NULL;
    if (N <= 0 || K <= 0 || (K % 32) != 0) return MKQ_ERR_SHAPE;
    if (N > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    if (!aligned16(W) || !aligned16(Wq_out) || (reinterpret_cast<uintptr_t>(s_w_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(s_w_in) & 3u))
        return MKQ_ERR_ALIGN;
    pack_weights_kernel<<<(int)N, 256, 0, as_stream(stream)>>>(W, K, s_w_in, s_w_out,
                                                               (uint32_t *)Wq_out, K);
    return launch_status();
}

extern "C" int mkq_pack_weights_int4_padded(const float *W, int64_t N, int64_t K, const float *s_w_in,
                                            float *s_w_out, uint8_t *Wq_out, void *stream)
{
    if (!W || !s_w_out || !Wq_out) return MKQ_ERR_NULL;
    if (N <= 0 || K <= 0 || (K % 8) != 0) return MKQ_ERR_SHAPE;
    if (N > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    if (!aligned16(W) || !aligned16(Wq_out) || (reinterpret_cast<uintptr_t>(s_w_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(s_w_in) & 3u))
        return MKQ_ERR_ALIGN;
    pack_weights_kernel<<<(int)N, 256, 0, as_stream(stream)>>>(W, K, s_w_in, s_w_out,
                                                               (uint32_t *)Wq_out, mkq_padded_k(K));
    return launch_status();
}

extern "C" int mkq_quantize_int8(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                                 float s_x, int8_t *q_out, void *stream)
{
    if (x_dtype != MKQ_F32 && x_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (M < 0 || K < 0 || (K % 16) != 0 || ldx < K || (ldx % 8) != 0) return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (M == 0 || K == 0) return MKQ_OK;
    if (!x || !q_out) return MKQ_ERR_NULL;
    if (!aligned16(x) || !aligned16(q_out)) return MKQ_ERR_ALIGN;
    const int grid = grid_for(M * (K / 8));
    if (x_dtype == MKQ_F32)
        quantize8_kernel<float><<<grid, 256, 0, as_stream(stream)>>>((const float *)x, M, K, ldx, s_x,
                                                                     (uint2 *)q_out);
    else
        quantize8_kernel<__half><<<grid, 256, 0, as_stream(stream)>>>((const __half *)x, M, K, ldx, s_x,
                                                                      (uint2 *)q_out);
    return launch_status();
}

extern "C" int mkq_pack_weights_int8(const float *W, int64_t N, int64_t K, const float *s_w_in,
                                     float *s_w_out, int8_t *Wq_out, void *stream)
{
    if (!W || !s_w_out || !Wq_out) return MKQ_ERR_NULL;
    if (N <= 0 || K <= 0 || (K % 16) != 0) return MKQ_ERR_SHAPE;
    if (N > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    if (!aligned16(W) || !aligned16(Wq_out) || (reinterpret_cast<uintptr_t>(s_w_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(s_w_in) & 3u))
        return MKQ_ERR_ALIGN;
    pack_weights8_kernel<<<(int)N, 256, 0, as_stream(stream)>>>(W, K, s_w_in, s_w_out, (uint2 *)Wq_out);
    return launch_status();
}

extern "C" int mkq_quantize_e3m2(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s_x,
                                 uint8_t *q_out, void *stream)
{
    if (x_dtype != MKQ_F32 && x_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (M < 0 || K < 0 || (K % 64) != 0 || ldx < K || (ldx % 8) != 0) return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (M == 0 || K == 0) return MKQ_OK;
    if (!x || !q_out) return MKQ_ERR_NULL;
    if (!aligned16(x) || !aligned16(q_out)) return MKQ_ERR_ALIGN;
    const int grid = grid_for(M * (K / 32));
    if (x_dtype == MKQ_F32)
        quantize_e3m2_kernel<float><<<grid, 256, 0, as_stream(stream)>>>((const float *)x, M, K, ldx, s_x, q_out);
    else
        quantize_e3m2_kernel<__half><<<grid, 256, 0, as_stream(stream)>>>((const __half *)x, M, K, ldx, s_x, q_out);
    return launch_status();
}

extern "C" int mkq_pack_codes_e3m2(const int8_t *codes, int64_t rows, int64_t K, uint8_t *q_out, void *stream)
{
    if (!codes || !q_out) return MKQ_ERR_NULL;
    if (rows <= 0 || K <= 0 || (K % 64) != 0) return MKQ_ERR_SHAPE;
    if (!aligned16(codes) || !aligned16(q_out)) return MKQ_ERR_ALIGN;
    const int64_t halves = rows * (K / 32);
    pack_codes_e3m2_kernel<<<grid_for(halves), 256, 0, as_stream(stream)>>>(codes, halves, q_out);
    return launch_status();
}

extern "C" int mkq_pack_weights_e3m2(const float *W, int64_t N, int64_t K, const float *s_w_in, float *s_w_out,
                                     uint8_t *Wq_out, void *stream)
{
    if (!W || !s_w_out || !Wq_out) return MKQ_ERR_NULL;
    if (N <= 0 || K <= 0 || (K % 64) != 0) return MKQ_ERR_SHAPE;
    if (N > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    if (!aligned16(W) || !aligned16(Wq_out) || (reinterpret_cast<uintptr_t>(s_w_out) & 3u) ||
        (reinterpret_cast<uintptr_t>(s_w_in) & 3u))
        return MKQ_ERR_ALIGN;
    pack_weights_e3m2_kernel<<<(int)N, 256, 0, as_stream(stream)>>>(W, K, s_w_in, s_w_out, Wq_out);
    return launch_status();
}

extern "C" int mkq_pack_codes_int4(const int8_t *codes, int64_t rows, int64_t K, uint8_t *q_out,
                                   void *stream)
{
    if (rows < 0 || K < 0 || (K % 32) != 0) return MKQ_ERR_SHAPE;
    if (rows == 0 || K == 0) return MKQ_OK;
    if (!codes || !q_out) return MKQ_ERR_NULL;
    if (!aligned16(codes) || !aligned16(q_out)) return MKQ_ERR_ALIGN;
    const int64_t words = rows * (K / 8);
    pack_codes_kernel<<<grid_for(words), 256, 0, as_stream(stream)>>>(codes, words, (uint32_t *)q_out);
    return launch_status();
}

extern "C" int mkq_unpack_weights_int4(const uint8_t *Wq, int64_t N, int64_t K, int8_t *codes_out,
                                       void *stream)
{
    if (N < 0 || K < 0 || (K % 32) != 0) return MKQ_ERR_SHAPE;
    if (N == 0 || K == 0) return MKQ_OK;
    if (!Wq || !codes_out) return MKQ_ERR_NULL;
    if (!aligned16(Wq) || !aligned16(codes_out)) return MKQ_ERR_ALIGN;
    const int64_t words = N * (K / 8);
    unpack_codes_kernel<<<grid_for(words), 256, 0, as_stream(stream)>>>((const uint32_t *)Wq, words,
                                                                        codes_out);
    return launch_status();
}

extern "C" const char *mkq_status_string(int status)
{
    switch (status) {
    case MKQ_OK: return "ok";
    case MKQ_ERR_NULL: return "required pointer is NULL";
    case MKQ_ERR_SHAPE: return "bad shape";
    case MKQ_ERR_ALIGN: return "pointer not 16-byte aligned";
    case MKQ_ERR_SCALE: return "step size must be positive and finite";
    case MKQ_ERR_DTYPE: return "unknown or unsupported dtype / activation";
    case MKQ_ERR_WORKSPACE: return "workspace missing or too small";
    case MKQ_ERR_UNSUPPORTED: return "request outside the supported range";
    case MKQ_ERR_HIP: return "HIP runtime error at launch";
    default: return "unknown status";
    }
}

extern "C" int mkq_version(void) { return 100; }
