// Measured ceilings of the machine, beside which the benchmark prints every roofline fraction: plain
// streaming kernels (read, write, copy) for what HBM delivers, and a register-only loop of the int8 MFMA
// that the GEMMs use, fed with operands of the same kind (bytes 16 * code), for what the matrix cores deliver
// under the chip's power management.  Measurement helpers: they compute nothing of the method.
#include "gemm_common.h"
#include "mkq_tuning.h"

namespace mkq {

// grid-stride, one 16-byte access per thread and step: the whole grid touches one compact window that moves
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4 *__restrict__ a, uint4 *sink, size_t n)
{
    uint4 s = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const uint4 v = a[i];
        s.x ^= v.x; s.y ^= v.y; s.z ^= v.z; s.w ^= v.w;
    }
    if (s.x == 0x12345u && s.y == 0x6789u) sink[0] = s;  // (keeps the loads)
}

__global__ __launch_bounds__(256) void stream_write_kernel(uint4 *__restrict__ b, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256)
        b[i] = make_uint4(1u, 2u, 3u, 4u);
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4 *__restrict__ a, uint4 *__restrict__ b, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) b[i] = a[i];
}

// Every wave: 8 independent accumulator tiles, operands loaded once from `operands` (6 x 16 bytes per lane),
// `iters` rounds of 8 MFMAs (the 128 x 64 wave tile of the GEMM: 2 weight x 4 activation fragments).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void mfma_i8_loop_kernel(const v4i *__restrict__ operands, int iters, int *sink)
{
    const int gid = blockIdx.x * 256 + threadIdx.x;
    v4i w[2], a[4];
#pragma unroll
    for (int t = 0; t < 2; ++t) w[t] = operands[(size_t)gid * 6 + t];
#pragma unroll
    for (int j = 0; j < 4; ++j) a[j] = operands[(size_t)gid * 6 + 2 + j];
    v16i acc[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][t][v] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int t = 0; t < 2; ++t) acc[j][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w[t], a[j], acc[j][t], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) s ^= acc[j][t][v];
    if (s == 0x7FFFFFF1) sink[0] = s;  // (keeps the arithmetic)
}

}  // namespace mkq

using namespace mkq;

extern "C" int mkq_measure_stream(int kind, const void *src, void *dst, size_t bytes, void *stream)
{
    if (kind < 0 || kind > 2) return MKQ_ERR_DTYPE;
    if ((kind != 1 && !src) || !dst) return MKQ_ERR_NULL;
    if (!aligned16(src) || !aligned16(dst)) return MKQ_ERR_ALIGN;
    if (bytes < 16 || (bytes % 16) != 0) return MKQ_ERR_SHAPE;
    int cus = 256;
    if (!device_cus(&cus)) return MKQ_ERR_HIP;
    const size_t n = bytes / 16;
    const unsigned grid = (unsigned)(16 * cus);
    if (kind == 0) stream_read_kernel<<<grid, 256, 0, as_stream(stream)>>>((const uint4 *)src, (uint4 *)dst, n);
    else if (kind == 1) stream_write_kernel<<<grid, 256, 0, as_stream(stream)>>>((uint4 *)dst, n);
    else stream_copy_kernel<<<grid, 256, 0, as_stream(stream)>>>((const uint4 *)src, (uint4 *)dst, n);
    return launch_status();
}

extern "C" int64_t mkq_measure_mfma_i8_ops(int iters)
{
    int cus = 256;
    if (iters <= 0 || !device_cus(&cus)) return 0;
    // 2 workgroups of 4 waves per CU, 8 MFMAs of 32 x 32 x 32 (65536 operations) per round and wave
    return (int64_t)cus * 2 * 4 * (int64_t)iters * 8 * 65536;
}

extern "C" size_t mkq_measure_mfma_i8_operand_bytes(void)
{
    int cus = 256;
    if (!device_cus(&cus)) return 0;
    return (size_t)cus * 2 * 256 * 6 * 16;
}

extern "C" int mkq_measure_mfma_i8(const void *operands, size_t operand_bytes, int iters, void *sink, void *stream)
{
    if (!operands || !sink) return MKQ_ERR_NULL;
    if (!aligned16(operands) || !aligned16(sink)) return MKQ_ERR_ALIGN;
    if (iters <= 0) return MKQ_ERR_SHAPE;
    int cus = 256;
    if (!device_cus(&cus)) return MKQ_ERR_HIP;
    if (operand_bytes < mkq_measure_mfma_i8_operand_bytes()) return MKQ_ERR_WORKSPACE;
    mfma_i8_loop_kernel<<<(unsigned)(2 * cus), 256, 0, as_stream(stream)>>>((const v4i *)operands, iters, (int *)sink);
    return launch_status();
}
