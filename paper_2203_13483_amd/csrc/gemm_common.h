// Helpers shared by the hand-written MFMA GEMM kernels (int4 and binary16):
// LDS-only barrier, LDS swizzle, fragment row permutation, compile-time loops,
// XCD-aware tile order, direct global->LDS copies with explicit waits.
#pragma once

#include "mkq_internal.h"

namespace mkq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));

// Workgroup barrier that orders LDS traffic only: global loads issued before it
// stay in flight across it (a full __syncthreads would drain them).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// 16-byte-chunk swizzle for an LDS row of CH chunks; r = row % 16.  The slot of
// chunk c in row r is c ^ swz(r).  As a linear map over GF(2) of the row bits it
// is injective on every set of rows that 8 or 16 consecutive lanes touch together
// (16 rows of one fragment in natural or permuted order; consecutive rows of a
// staging write), so such lanes always land in distinct 16-byte bank groups.
template <int CH>
__device__ __forceinline__ int swz(int r);
template <>
__device__ __forceinline__ int swz<4>(int r)
{
    return ((r >> 3) & 1) ^ (((r >> 2) & 1) << 1) ^ (((r >> 1) & 1) * 3);
}
template <>
__device__ __forceinline__ int swz<2>(int r) { return ((r >> 2) ^ (r >> 3)) & 1; }
template <>
__device__ __forceinline__ int swz<8>(int r) { return (r & 7) ^ (((r >> 3) & 1) * 7); }

// Order in which the 32 rows of a W fragment are read: MFMA row i = 8g + 4h + e
// (g = i/8, h = (i/4)%2, e = i%4) reads tile row 16*(g/2) + 8h + 4*(g%2) + e.  The
// 32x32 result keeps rows 8*(v/4) + 4*(lane/32) + v%4 in register v, so after the
// permutation registers 0..7 / 8..15 of a lane are channels 8*(lane/32) + 0..7 of
// the first / second half of the 32-channel tile.
__device__ __forceinline__ int w_row_perm(int i)
{
    const int g = i >> 3, h = (i >> 2) & 1, e = i & 3;
    return 16 * (g >> 1) + 8 * h + 4 * (g & 1) + e;
}

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>).
// Used where an index selects accumulator registers, which must never become a
// run-time index (the array would be demoted to scratch memory).
template <int I>
struct IntC { static constexpr int value = I; };
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (N > 0) {
        static_for<N - 1>(f);
        f(IntC<N - 1>{});
    }
}

// XCD-aware tile order.  Workgroups are dealt round-robin to the 8 XCDs, each with
// its own L2; consecutive logical tiles are therefore given to the same XCD, and
// logical tiles walk GROUP_M token tiles before moving to the next channel tile, so
// the tiles resident on one XCD at a time share a few A and W row panels.
__device__ __forceinline__ void tile_coords(int bid, int tiles_m, int tiles_n, int &tm, int &tn)
{
    constexpr int XCDS = 8, GROUP_M = 8;
    const int total = tiles_m * tiles_n;
    int L = bid;
    if (total % XCDS == 0) L = (bid % XCDS) * (total / XCDS) + bid / XCDS;
    const int per_group = GROUP_M * tiles_n;
    const int group = L / per_group;
    const int first_m = group * GROUP_M;
    const int rows = (tiles_m - first_m) < GROUP_M ? (tiles_m - first_m) : GROUP_M;
    const int in_group = L - group * per_group;
    tm = first_m + in_group % rows;
    tn = in_group / rows;
}

// One wave-level global->LDS copy: lane l fetches 16 bytes at base + voff and they
// land at LDS address lds_base + LDS_IMM + 16 * l.
template <int LDS_IMM>
__device__ __forceinline__ void dma_copy16(const uint8_t *base, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base), "n"(LDS_IMM)
                 : "memory", "m0", "scc");
}

// Same with 4 bytes per lane: lane l's dword lands at lds_base + LDS_IMM + 4 * l.
template <int LDS_IMM>
__device__ __forceinline__ void dma_copy4(const uint8_t *base, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds_base), "v"(voff), "s"(base), "n"(LDS_IMM)
                 : "memory", "m0", "scc");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Resident workgroups of a persistent kernel on the current device: CUs x workgroups per CU.  The
// per-device setup (dynamic LDS limit, occupancy query) runs once per kernel instantiation and device.
template <class K>
inline int resident_workgroups(PerDeviceOnce &once, K kernel, int threads, size_t lds, int max_per_cu, int64_t *resident)
{
    const int wgs = once.get([&]() -> int {
        if (lds > 65536 &&
            hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return -1;
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, threads, lds) != hipSuccess || occ < 1) return -1;
        return occ > max_per_cu ? max_per_cu : occ;
    });
    int cus = 0;
    if (wgs <= 0 || !device_cus(&cus)) return MKQ_ERR_HIP;
    *resident = (int64_t)cus * wgs;
    return MKQ_OK;
}

}  // namespace mkq
