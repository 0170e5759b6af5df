// Scale machinery of sections 3.1 and 4.1: the two scale-gradient sums of one tensor
// (STE-based and MSE-based) and percentile calibration of an activation step.  All are
// streaming reductions over the tensor, bound by HBM bandwidth (one read of x per pass).
#include "mkq_internal.h"

namespace mkq {

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ void zero_words_kernel(uint32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// g[0] += sum_i ( round(x_i/s) - x_i/s ),  g[1] += 2 sum_i ( Q[x_i] - x_i ) round(x_i/s)
// with round() = the code of Eq. 1 (clamp included), decided in binary32 like the quantizer;
// the terms and sums are binary64.
template <typename T, int BITS>
__global__ __launch_bounds__(256) void scale_gradients_kernel(const T *__restrict__ x, int64_t M, int64_t K,
                                                              int64_t ldx, float s, double *__restrict__ g)
{
    __shared__ double part[2][4];
    const double sd = (double)s, inv = 1.0 / sd;
    const int64_t groups_per_row = K / 8;
    const int64_t total = M * groups_per_row;
    double ste = 0.0, mse = 0.0;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total;
         w += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = w / groups_per_row;
        const int64_t kg = w - m * groups_per_row;
        float v[8];
        load8<T>(x + m * ldx + kg * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int c = (BITS == 4) ? quantize_code(v[e], s) : quantize_code8(v[e], s);
            const double cd = (double)c, xd = (double)v[e];
            ste += __builtin_fma(-xd, inv, cd);
            mse = __builtin_fma(__builtin_fma(sd, cd, -xd), cd, mse);
        }
    }
    ste = wave_sum_f64(ste);
    mse = wave_sum_f64(mse);
    if ((threadIdx.x & 63) == 0) {
        part[0][threadIdx.x >> 6] = ste;
        part[1][threadIdx.x >> 6] = mse;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        atomicAdd(g, (part[0][0] + part[0][1]) + (part[0][2] + part[0][3]));
        atomicAdd(g + 1, 2.0 * ((part[1][0] + part[1][1]) + (part[1][2] + part[1][3])));
    }
}

// ---- percentile calibration: exact k-th largest of |x| by radix selection -------------
// |x| >= 0, so its binary32 bit pattern (31 bits) orders like an unsigned integer.  Three
// passes count, among the elements whose higher bits equal the prefix chosen so far, the
// next 11, 10 and 10 bits; after each a single workgroup walks the counts from the top
// and fixes the digit in which the k-th largest falls.
constexpr int PCT_BINS = 2048;
struct PctWorkspace {
    uint32_t hist[3][PCT_BINS];
    uint32_t prefix;  // bits fixed so far
    uint32_t k;       // rank still to find inside the prefix
    uint32_t pad[2];
};

// Four copies of the counts, chosen by lane % 4: activations pile up in a few dozen bins
// (one binade is 8 bins of pass 0), and lanes of one LDS atomic that hit the same counter
// are served one after the other.
template <typename T, int PASS>
__global__ __launch_bounds__(256) void percentile_hist_kernel(const T *__restrict__ x, int64_t M, int64_t K,
                                                              int64_t ldx, PctWorkspace *__restrict__ ws)
{
    constexpr int COPIES = 4;  // interleaved, so the copies of one bin sit in different banks
    __shared__ uint32_t h[PCT_BINS * COPIES];
    for (int i = threadIdx.x; i < COPIES * PCT_BINS; i += 256) h[i] = 0u;
    __syncthreads();
    uint32_t *const mine = h + (threadIdx.x & (COPIES - 1));
    const uint32_t prefix = PASS ? ws->prefix : 0u;
    const int64_t groups_per_row = K / 8;
    const int64_t total = M * groups_per_row;
    for (int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; w < total;
         w += (int64_t)gridDim.x * blockDim.x) {
        const int64_t m = w / groups_per_row;
        const int64_t kg = w - m * groups_per_row;
        float v[8];
        load8<T>(x + m * ldx + kg * 8, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t bits = (v[e] != v[e]) ? 0u : (__float_as_uint(v[e]) & 0x7FFFFFFFu);
            if (PASS == 0) {
                atomicAdd(&mine[(bits >> 20) * COPIES], 1u);
            } else if (PASS == 1) {
                if ((bits >> 20) == prefix) atomicAdd(&mine[((bits >> 10) & 1023u) * COPIES], 1u);
            } else {
                if ((bits >> 10) == prefix) atomicAdd(&mine[(bits & 1023u) * COPIES], 1u);
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < PCT_BINS; i += 256) {
        const uint32_t c = (h[4 * i] + h[4 * i + 1]) + (h[4 * i + 2] + h[4 * i + 3]);
        if (c) atomicAdd(&ws->hist[PASS][i], c);
    }
}

// One workgroup.  PASS 0 starts from rank k0; the later passes from the rank left over.
// Thread t owns PER consecutive bins; the thread whose bins hold the k-th largest (fewer
// than k elements in the bins above its own, at least k from its lowest bin up) fixes
// the digit.  After PASS 2 the prefix is the whole bit pattern of T and the step
// T / qmax is written.
template <int PASS>
__global__ __launch_bounds__(256) void percentile_select_kernel(PctWorkspace *__restrict__ ws, uint32_t k0,
                                                                float qmax, float *__restrict__ s_out)
{
    constexpr int NB = PASS == 0 ? 2048 : 1024;
    constexpr int PER = NB / 256;
    __shared__ uint32_t chunk[256], group[16];
    const int t = threadIdx.x;
    uint32_t mine[PER], sum = 0;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        mine[i] = ws->hist[PASS][t * PER + i];
        sum += mine[i];
    }
    chunk[t] = sum;
    const uint32_t k = PASS ? ws->k : k0;
    const uint32_t old_prefix = PASS ? ws->prefix : 0u;
    __syncthreads();
    if (t < 16) {
        uint32_t gs = 0;
#pragma unroll
        for (int u = 0; u < 16; ++u) gs += chunk[16 * t + u];
        group[t] = gs;
    }
    __syncthreads();
    // elements in the bins above this thread's: later threads of its group of 16, later groups
    uint32_t above = 0;
#pragma unroll
    for (int u = 1; u < 16; ++u) above += ((t & 15) + u < 16) ? chunk[t + u] : 0u;
#pragma unroll
    for (int g = 1; g < 16; ++g) above += ((t >> 4) + g < 16) ? group[(t >> 4) + g] : 0u;
    if (above < k && above + sum >= k) {
        uint32_t cum = above;
        int b = 0;  // the lowest bin is taken when none above it reaches k
        bool found = false;
#pragma unroll
        for (int i = PER - 1; i > 0; --i) {
            if (!found) {
                if (cum + mine[i] >= k) {
                    found = true;
                    b = i;
                } else {
                    cum += mine[i];
                }
            }
        }
        const uint32_t prefix = PASS == 0 ? (uint32_t)(t * PER + b) : ((old_prefix << 10) | (uint32_t)(t * PER + b));
        ws->prefix = prefix;
        ws->k = k - cum;
        if (PASS == 2) {
            const float tv = __uint_as_float(prefix);
            s_out[0] = (tv > 0.0f) ? tv / qmax : 1.0f;
        }
    }
}

static inline int stream_grid(int64_t items, int max_blocks = 256 * 8)
{
    int64_t b = ceil_div(items, 256);
    if (b < 1) b = 1;
    if (b > max_blocks) b = max_blocks;
    return (int)b;
}

}  // namespace mkq

using namespace mkq;

static int check_tensor(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx)
{
    if (x_dtype != MKQ_F32 && x_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (M <= 0 || K <= 0 || (K % 8) != 0 || ldx < K || (ldx % 8) != 0) return MKQ_ERR_SHAPE;
    if (!x) return MKQ_ERR_NULL;
    if (!aligned16(x)) return MKQ_ERR_ALIGN;
    return MKQ_OK;
}

extern "C" int mkq_scale_gradients(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s, int bits,
                                   double *g_out, void *stream)
{
    const int rc = check_tensor(x, x_dtype, M, K, ldx);
    if (rc != MKQ_OK) return rc;
    if (bits != 4 && bits != 8) return MKQ_ERR_DTYPE;
    if (!scale_ok(s)) return MKQ_ERR_SCALE;
    if (!g_out) return MKQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(g_out) & 7u) return MKQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    zero_words_kernel<<<1, 64, 0, st>>>((uint32_t *)g_out, 4);
    const int grid = stream_grid(M * (K / 8));
#define MKQ_SG(T, B) scale_gradients_kernel<T, B><<<grid, 256, 0, st>>>((const T *)x, M, K, ldx, s, g_out)
    if (x_dtype == MKQ_F32) {
        if (bits == 4) MKQ_SG(float, 4); else MKQ_SG(float, 8);
    } else {
        if (bits == 4) MKQ_SG(__half, 4); else MKQ_SG(__half, 8);
    }
#undef MKQ_SG
    return launch_status();
}

extern "C" size_t mkq_percentile_scale_workspace_bytes(void) { return sizeof(PctWorkspace); }

extern "C" int mkq_percentile_scale(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, int64_t top_ppm,
                                    int bits, float *s_out, void *workspace, size_t workspace_bytes, void *stream)
{
    const int rc = check_tensor(x, x_dtype, M, K, ldx);
    if (rc != MKQ_OK) return rc;
    if (bits != 4 && bits != 8) return MKQ_ERR_DTYPE;
    if (top_ppm < 0 || top_ppm > 1000000) return MKQ_ERR_SHAPE;
    if (!s_out) return MKQ_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(s_out) & 3u) return MKQ_ERR_ALIGN;
    if (!workspace || workspace_bytes < sizeof(PctWorkspace) || !aligned16(workspace)) return MKQ_ERR_WORKSPACE;
    const int64_t n = M * K;
    if (n > 0xFFFFFFFFLL) return MKQ_ERR_UNSUPPORTED;  // 32-bit counts
    int64_t k = n * top_ppm / 1000000;
    if (k < 1) k = 1;
    const float qmax = bits == 4 ? 7.0f : 127.0f;
    PctWorkspace *ws = (PctWorkspace *)workspace;
    hipStream_t st = as_stream(stream);
    constexpr int words = (int)(sizeof(PctWorkspace) / 4);
    zero_words_kernel<<<(words + 255) / 256, 256, 0, st>>>((uint32_t *)ws, words);
    const int grid = stream_grid(M * (K / 8), 256 * 4);  // 32 KiB of LDS each: all resident at once
#define MKQ_PASS(P)                                                                                     \
    if (x_dtype == MKQ_F32) percentile_hist_kernel<float, P><<<grid, 256, 0, st>>>((const float *)x, M, K, ldx, ws); \
    else percentile_hist_kernel<__half, P><<<grid, 256, 0, st>>>((const __half *)x, M, K, ldx, ws);     \
    percentile_select_kernel<P><<<1, 256, 0, st>>>(ws, (uint32_t)k, qmax, s_out)
    MKQ_PASS(0);
    MKQ_PASS(1);
    MKQ_PASS(2);
#undef MKQ_PASS
    return launch_status();
}
