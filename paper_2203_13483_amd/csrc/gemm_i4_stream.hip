// Few tokens (M <= 128): the int4 linear is a stream of the weight matrix, bound by HBM.
//
// A workgroup of four waves owns 128 output channels and one slice of K.  Packed rows of W and of the
// activations are copied straight from global memory into an LDS ring with global_load_lds_dwordx4,
// 128 contiguous bytes (256 codes, one cache line) of a row per group of 8 lanes, so every request is a
// whole line that is fetched exactly once; the XOR swizzle of the 16-byte pieces is applied on the global
// side, which keeps the ds_read_b128 fragment reads bank-conflict free.  A wave copies and multiplies its
// own 32 weight rows; the activation rows of a stage (32 * TB tokens) are copied once per workgroup and
// read by all four waves, so there is one LDS barrier per stage of 256 codes.  S - 1 stages are in flight
// per workgroup (40 .. 64 KiB), two workgroups share a CU for TB <= 2.
//
// K split across workgroups: int32 partial sums are exactly associative, so any split gives the same
// accumulators.  With KS > 1 slices per channel tile every workgroup stores its partial accumulators to
// the scratch area with agent-scope (write-through) stores, waits for them, and takes a ticket from the
// tile's counter; the workgroup that draws the last ticket reads the other slices' partials with
// agent-scope loads, adds them to its own registers, resets the counter and runs the epilogue.  Nobody
// waits for anybody, so the scheme cannot hang; the counters must be zero when the kernel starts and are
// left zero when it ends.
#include "gemm_i4_params.h"

namespace mkq {

template <int TB_, int S_>
struct StreamCfg {
    static constexpr int TB = TB_, S = S_;
    static constexpr int WAVES = 4, THREADS = 256, BN = 128;
    static constexpr int A_ROWS = 32 * TB, A_BYTES = A_ROWS * 128;
    static constexpr int STAGE_BYTES = (A_ROWS + BN) * 128;
    static constexpr int LPW = 4 + TB;  // copies per wave per stage: its own 32 weight rows, TB of the activations'
    static constexpr int LDS_BYTES = S * STAGE_BYTES;
    // the epilogue sees the wave's accumulators as a column of TB 32 x 32 tiles
    static constexpr int TM = TB, TN = 1, WTM = 32 * TB, WTN = 32;
    static_assert(S >= 2 && (S - 1) * LPW <= 63, "vmcnt immediate is 6 bits");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS is 160 KiB per CU");
};

// K split across workgroups, the part after the k loop: the wave's partial accumulators go to the scratch
// area, the workgroup takes a ticket from the tile's counter, and only the workgroup that draws the last one
// returns true, with the other slices' partial sums added to its registers and the counter reset.
// A wave's partial tile is 16 registers x 64 lanes per token block; register pair j of all lanes is one
// contiguous 512-byte piece.  Agent-scope relaxed atomics: the stores write through to memory and the loads
// do not hit a stale line of this XCD's L2, without any cache-wide write-back or invalidate.
template <class Cfg>
__device__ __forceinline__ bool splitk_reduce(v16i (&acc)[Cfg::TB][1], const SplitKArgs &sk, int tile, int slice,
                                              int wave, int lane, int tid, int *last_ticket)
{
    constexpr int TB = Cfg::TB;
    uint64_t *const area = reinterpret_cast<uint64_t *>(sk.partials);
    const size_t wave_words = (size_t)TB * 8 * 64;  // 64-bit words per wave
    uint64_t *const mine = area + ((size_t)(tile * sk.ks + slice) * Cfg::WAVES + wave) * wave_words + lane;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint64_t v = (uint64_t)(uint32_t)acc[tb][0][2 * j] | ((uint64_t)(uint32_t)acc[tb][0][2 * j + 1] << 32);
            __hip_atomic_store(mine + (tb * 8 + j) * 64, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    wait_vmcnt<0>();   // this wave's partials have reached memory
    __syncthreads();   // ... and every other wave's
    if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(sk.counters + tile, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const int last = old == (unsigned)(sk.ks - 1);
        if (last) __hip_atomic_store(sk.counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *last_ticket = last;
    }
    __syncthreads();
    if (!*last_ticket) return false;
    for (int o = 0; o < sk.ks; ++o) {
        if (o == slice) continue;
        const uint64_t *theirs = area + ((size_t)(tile * sk.ks + o) * Cfg::WAVES + wave) * wave_words + lane;
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const uint64_t v = __hip_atomic_load(theirs + (tb * 8 + j) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                acc[tb][0][2 * j] += (int)(uint32_t)v;
                acc[tb][0][2 * j + 1] += (int)(uint32_t)(v >> 32);
            }
    }
    return true;
}

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_i4_stream_kernel(const GemmI4Params p, const SplitKArgs sk)
{
    constexpr int TB = Cfg::TB, S = Cfg::S, LPW = Cfg::LPW;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ int last_ticket;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;

    const int tiles_n = (p.N + Cfg::BN - 1) / Cfg::BN;
    const int tile = (int)blockIdx.x % tiles_n, slice = (int)blockIdx.x / tiles_n;
    const int n0 = tile * Cfg::BN;
    const int row_bytes = p.K / 2;
    const int groups = row_bytes / 128;  // stages of 256 codes in a row
    // slice s of ks takes the stages s, s + ks, s + 2 ks, ... (the slices of a tile walk k side by side)
    const int steps = (groups - slice + sk.ks - 1) / sk.ks;

    // copies: lanes 8r .. 8r+7 of a wave-level copy fetch the eight 16-byte pieces of one row
    const int c_row = lane >> 3, c_slot = lane & 7;
    uint32_t woff[4], aoff[TB];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = 32 * wave + 8 * q + c_row;
        int n = n0 + row;
        n = n < p.N ? n : p.N - 1;  // rows past the edge re-read the last row; never stored
        woff[q] = (uint32_t)n * (uint32_t)row_bytes + ((c_slot ^ swz<8>(row & 15)) * 16);
    }
#pragma unroll
    for (int i = 0; i < TB; ++i) {
        const int row = 8 * (wave + 4 * i) + c_row;
        const int m = row < p.M ? row : p.M - 1;
        aoff[i] = (uint32_t)m * (uint32_t)row_bytes + ((c_slot ^ swz<8>(row & 15)) * 16);
    }
    // Always LPW copies per stage, so the number in flight never depends on where the pipeline is: past
    // the slice's last stage it fetches that stage again into a slot that is not read any more.
    auto issue = [&](int slot, int t) {
        t = t < steps ? t : steps - 1;
        const int g = slice + t * sk.ks;
        const uint8_t *wk = p.W + (size_t)g * 128, *ak = p.A + (size_t)g * 128;
        const uint32_t st = lds0 + slot * Cfg::STAGE_BYTES;
        static_for<4>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            dma_copy16<q * 1024>(wk, woff[q], st + Cfg::A_BYTES + wave * 4096);
        });
        static_for<TB>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            dma_copy16<i * 4096>(ak, aoff[i], st + wave * 1024);
        });
    };

    // fragment reads: round r of a stage (64 codes) is the 16-byte pieces 2r + fh of the lane's rows
    int rdW[4], rdA[4];
    {
        const int wrow = 32 * wave + w_row_perm(fr);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            rdW[r] = Cfg::A_BYTES + wrow * 128 + (((2 * r + fh) ^ swz<8>(wrow & 15)) * 16);
            rdA[r] = fr * 128 + (((2 * r + fh) ^ swz<8>(fr & 15)) * 16);  // token block tb: + 4096 * tb
        }
    }

    v16i acc[TB][1];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tb][0][v] = 0;

#pragma unroll
    for (int i = 0; i < S - 1; ++i) issue(i, i);
    int slot = 0, fill = S - 1;
    for (int s = 0; s < steps; ++s) {
        // stage s has landed (the S - 2 younger ones may still be in flight); past the barrier every
        // wave has also finished reading the slot that is refilled next
        wait_vmcnt<(S - 2) * LPW>();
        lds_barrier();
        issue(fill, s + S - 1);
        fill = (fill + 1 == S) ? 0 : fill + 1;
        const uint8_t *st = smem + slot * Cfg::STAGE_BYTES;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const uint4 fw = *reinterpret_cast<const uint4 *>(st + rdW[r]);
            const v4i w0 = widen(fw.x, fw.y), w1 = widen(fw.z, fw.w);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                const uint4 fa = *reinterpret_cast<const uint4 *>(st + rdA[r] + 4096 * tb);
                acc[tb][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w0, widen(fa.x, fa.y), acc[tb][0], 0, 0, 0);
                acc[tb][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, widen(fa.z, fa.w), acc[tb][0], 0, 0, 0);
            }
        }
        slot = (slot + 1 == S) ? 0 : slot + 1;
    }
    wait_vmcnt<0>();  // the trailing copies must land before the LDS is released

    if (sk.ks > 1) {
        if (!splitk_reduce<Cfg>(acc, sk, tile, slice, wave, lane, tid, &last_ticket)) return;
    }
    gemm_i4_epilogue<Cfg, EpiGeneric>(p, acc, 0, n0 + 32 * wave, 0, 0, fr, fh);
}

// The same linear on weights in the streaming layout (mkq_repack_weights_int4_stream): the 32 channels of a
// panel and 64 codes of k form a 1 KiB block that holds, for lane l of a wave, the 16 bytes of MFMA operand
// it needs (channel 32 * panel + w_row_perm(l % 32), codes 64 * block + 32 * (l / 32) ...); the blocks of one
// k position of all panels follow each other, then the next k position.  A wave fetches its operands with
// whole-wave 1 KiB loads straight into registers (no LDS, every cache line touched once), P - 1 stages of
// 256 codes ahead of the arithmetic, and because all workgroups walk k together the chip as a whole reads
// one compact window of memory that moves forward -- the pattern on which HBM gives its full rate (rows a
// power-of-two pitch apart, or one long private stream per wave, reach about two thirds of it).  Only the
// activations, shared by the four waves of a workgroup, go through the LDS ring.
// Blocks per k position in the streaming layout: the number of panels, made odd -- with an even (above all
// a power-of-two) count the blocks that a wave has in flight, one k position apart each, fall on the same
// memory channels.
__host__ __device__ inline int stream_pitch_panels(int N) { return ((N + 31) / 32) | 1; }

template <int TB_, int P_>
struct WStreamCfg {
    static constexpr int TB = TB_, P = P_;
    static constexpr int WAVES = 4, THREADS = 256, BN = 128;
    static constexpr int STAGE_BYTES = 32 * TB * 128;  // activations only
    static constexpr int LPW = 4 + TB;                 // per wave per stage: 4 weight loads, TB activation copies
    static constexpr int LDS_BYTES = P * STAGE_BYTES;
    static constexpr int TM = TB, TN = 1, WTM = 32 * TB, WTN = 32;
    static_assert(P >= 2 && (P - 1) * LPW <= 63, "vmcnt immediate is 6 bits");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_i4_wstream_kernel(const GemmI4Params p, const SplitKArgs sk)
{
    constexpr int TB = Cfg::TB, P = Cfg::P, LPW = Cfg::LPW;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    __shared__ int last_ticket;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;

    const int tiles_n = (p.N + Cfg::BN - 1) / Cfg::BN;
    const int tile = (int)blockIdx.x % tiles_n, slice = (int)blockIdx.x / tiles_n;
    const int n0 = tile * Cfg::BN;
    const int row_bytes = p.K / 2;
    const int groups = row_bytes / 128;
    // slice s of ks takes the stages s, s + ks, s + 2 ks, ...: the slices of a tile walk k side by side, so all
    // workgroups of the launch read one window of memory (slices that each took a contiguous range of k
    // would read ks windows a power-of-two distance apart, which collide in the memory banks)
    const int steps = (groups - slice + sk.ks - 1) / sk.ks;

    // this wave's panel; a panel past the last one (N not a multiple of 128) re-reads the last: never stored
    const int panels = (p.N + 31) / 32;
    int panel = 4 * tile + wave;
    panel = panel < panels ? panel : panels - 1;
    const uint4 *const wp = reinterpret_cast<const uint4 *>(p.W) + (size_t)panel * 64 + lane;
    const size_t block_pitch = (size_t)stream_pitch_panels(p.N) * 64;  // in 16-byte pieces, to the next k position

    const int c_row = lane >> 3, c_slot = lane & 7;
    uint32_t aoff[TB];
#pragma unroll
    for (int i = 0; i < TB; ++i) {
        const int row = 8 * (wave + 4 * i) + c_row;
        const int m = row < p.M ? row : p.M - 1;
        aoff[i] = (uint32_t)m * (uint32_t)row_bytes + ((c_slot ^ swz<8>(row & 15)) * 16);
    }
    int rdA[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) rdA[r] = fr * 128 + (((2 * r + fh) ^ swz<8>(fr & 15)) * 16);

    uint4 fw[P][4];
    // stage t of the walk: four weight blocks into registers, the activation rows into ring slot j
    auto issue = [&](auto jc, int t) {
        constexpr int j = decltype(jc)::value;
        t = t < steps ? t : steps - 1;  // past the end: the last stage again (constant number of operations in flight)
        const int g = slice + t * sk.ks;
#pragma unroll
        for (int r = 0; r < 4; ++r) fw[j][r] = wp[(size_t)(4 * g + r) * block_pitch];
        const uint8_t *ak = p.A + (size_t)g * 128;
        static_for<TB>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            dma_copy16<i * 4096>(ak, aoff[i], lds0 + j * Cfg::STAGE_BYTES + wave * 1024);
        });
    };

    v16i acc[TB][1];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tb][0][v] = 0;

    // The epilogue's per-channel scales and biases are first touched here, so that their round trip to
    // memory overlaps the weight stream instead of following it.
    float touched;
    {
        int n = n0 + 32 * wave + fr;
        n = n < p.N ? n : p.N - 1;
        touched = p.s_w[n] + (p.bias ? p.bias[n] : 0.0f);
    }
    static_for<P - 1>([&](auto ic) { issue(ic, decltype(ic)::value); });
    // The loop body has no branches: the compiler counts the register loads in flight itself, and across
    // conditional blocks it falls back to waiting for nearly all of them.  Stages past the end of the slice
    // (the walk is rounded up to a multiple of P) multiply weights masked to zero.
    const int iters = (steps + P - 1) / P;
    for (int it = 0; it < iters; ++it) {
        static_for<P>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            const int t = it * P + j;
            wait_vmcnt<(P - 2) * LPW>();
            lds_barrier();
            issue(IntC<(j + P - 1) % P>{}, t + P - 1);
            const uint32_t live = t < steps ? 0xFFFFFFFFu : 0u;
            const uint8_t *st = smem + j * Cfg::STAGE_BYTES;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const v4i w0 = widen(fw[j][r].x & live, fw[j][r].y & live), w1 = widen(fw[j][r].z & live, fw[j][r].w & live);
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    const uint4 fa = *reinterpret_cast<const uint4 *>(st + rdA[r] + 4096 * tb);
                    acc[tb][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w0, widen(fa.x, fa.y), acc[tb][0], 0, 0, 0);
                    acc[tb][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, widen(fa.z, fa.w), acc[tb][0], 0, 0, 0);
                }
            }
        });
    }
    wait_vmcnt<0>();  // the trailing copies must land before the LDS is released
    asm volatile("" ::"v"(touched));  // (keeps the early loads)

    if (sk.ks > 1) {
        if (!splitk_reduce<Cfg>(acc, sk, tile, slice, wave, lane, tid, &last_ticket)) return;
    }
    gemm_i4_epilogue<Cfg, EpiGeneric>(p, acc, 0, n0 + 32 * wave, 0, 0, fr, fh);
}

template <class Cfg>
static int launch_stream(const GemmI4Params &p, const SplitKArgs &sk, hipStream_t st)
{
    static PerDeviceOnce once;
    const int ok = once.get([&]() -> int {
        if (Cfg::LDS_BYTES > 65536 &&
            hipFuncSetAttribute((const void *)gemm_i4_stream_kernel<Cfg>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                Cfg::LDS_BYTES) != hipSuccess)
            return -1;
        return 1;
    });
    if (ok < 0) return MKQ_ERR_HIP;
    if (p.setup_only) return MKQ_OK;
    const int64_t grid = ceil_div(p.N, Cfg::BN) * sk.ks;
    gemm_i4_stream_kernel<Cfg><<<(unsigned)grid, Cfg::THREADS, Cfg::LDS_BYTES, st>>>(p, sk);
    return launch_status();
}

bool gemm_i4_stream_ok(const GemmI4Params &p) { return p.M <= 128 && (p.K % 256) == 0; }

// Number of K slices per channel tile: enough workgroups to put one on every CU (more slices cost more in
// partial sums and tickets than the extra workgroups gain), slices of at least MIN_STAGES stages, and partial
// sums that fit the scratch area.  forced_ks > 0 overrides the choice (still clamped to what the scratch
// area and K allow).
int gemm_i4_stream_slices(const GemmI4Params &p, const SplitKScratch *scr, int forced_ks)
{
    if (!scr || !scr->counters || !scr->partials) return 1;
    const int tb = p.M <= 32 ? 1 : (p.M <= 64 ? 2 : 4);
    const int64_t tiles_n = ceil_div(p.N, 128), groups = p.K / 256;
    if (tiles_n > SPLITK_MAX_TILES) return 1;
    int cus = 256;
    device_cus(&cus);
    constexpr int MIN_STAGES = 4;
    int64_t ks = forced_ks > 0 ? forced_ks : (cus + tiles_n / 2) / tiles_n;
    if (forced_ks <= 0 && ks > groups / MIN_STAGES) ks = groups / MIN_STAGES;
    if (ks > groups) ks = groups;
    const int64_t per_slice = tiles_n * 4 * tb * 4096;  // bytes of partial sums per slice
    if (ks * per_slice > (int64_t)scr->partial_bytes) ks = (int64_t)scr->partial_bytes / per_slice;
    return ks < 1 ? 1 : (int)ks;
}

int run_gemm_i4_stream(const GemmI4Params &p, const SplitKScratch *scr, int forced_ks, hipStream_t st)
{
    SplitKArgs sk;
    sk.ks = p.setup_only ? 1 : gemm_i4_stream_slices(p, scr, forced_ks);
    sk.counters = sk.ks > 1 ? scr->counters : nullptr;
    sk.partials = sk.ks > 1 ? scr->partials : nullptr;
    if (p.M <= 32) return launch_stream<StreamCfg<1, 3>>(p, sk, st);
    if (p.M <= 64) return launch_stream<StreamCfg<2, 3>>(p, sk, st);
    return launch_stream<StreamCfg<4, 3>>(p, sk, st);
}

template <class Cfg>
static int launch_wstream(const GemmI4Params &p, const SplitKArgs &sk, hipStream_t st)
{
    static_assert(Cfg::LDS_BYTES <= 65536, "no dynamic LDS limit to raise");
    if (p.setup_only) return MKQ_OK;
    const int64_t grid = ceil_div(p.N, Cfg::BN) * sk.ks;
    gemm_i4_wstream_kernel<Cfg><<<(unsigned)grid, Cfg::THREADS, Cfg::LDS_BYTES, st>>>(p, sk);
    return launch_status();
}

// p.W is in the streaming layout.  variant: 0 = the library's choice, otherwise the prefetch depth P.
int run_gemm_i4_wstream(const GemmI4Params &p, const SplitKScratch *scr, int forced_ks, int variant, hipStream_t st)
{
    SplitKArgs sk;
    sk.ks = p.setup_only ? 1 : gemm_i4_stream_slices(p, scr, forced_ks);
    sk.counters = sk.ks > 1 ? scr->counters : nullptr;
    sk.partials = sk.ks > 1 ? scr->partials : nullptr;
    if (p.M <= 32) {
        if (variant == 2) return launch_wstream<WStreamCfg<1, 2>>(p, sk, st);
        if (variant == 3) return launch_wstream<WStreamCfg<1, 3>>(p, sk, st);
        if (variant == 6) return launch_wstream<WStreamCfg<1, 6>>(p, sk, st);
        return launch_wstream<WStreamCfg<1, 4>>(p, sk, st);
    }
    if (p.M <= 64) {
        if (variant == 2) return launch_wstream<WStreamCfg<2, 2>>(p, sk, st);
        if (variant == 3) return launch_wstream<WStreamCfg<2, 3>>(p, sk, st);
        if (variant == 6) return launch_wstream<WStreamCfg<2, 6>>(p, sk, st);
        if (variant == 4) return launch_wstream<WStreamCfg<2, 4>>(p, sk, st);
        return launch_wstream<WStreamCfg<2, 3>>(p, sk, st);
    }
    if (variant == 2) return launch_wstream<WStreamCfg<4, 2>>(p, sk, st);
    return launch_wstream<WStreamCfg<4, 3>>(p, sk, st);
}

// Streaming layout: 16-byte piece l of the block of k position g and panel q -- block number g * panels + q --
// is bytes [32 g + 16 (l / 32), + 16) of the canonical row of channel 32 q + w_row_perm(l % 32); channels past N
// are zero.
__global__ void repack_stream_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, int N, int K, int64_t chunks)
{
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (c >= chunks) return;
    const int l = (int)(c & 63);
    const int64_t blk = c >> 6;
    const int pitch = stream_pitch_panels(N);
    const int q = (int)(blk % pitch), g = (int)(blk / pitch);
    const int n = 32 * q + w_row_perm(l & 31);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = src[(int64_t)n * (K / 32) + 2 * g + (l >> 5)];
    dst[c] = v;
}

int setup_gemm_i4_stream(const GemmI4Params &p, hipStream_t st)
{
    SplitKArgs sk = {1, nullptr, nullptr};
    int rc = launch_stream<StreamCfg<1, 3>>(p, sk, st);
    if (rc == MKQ_OK) rc = launch_stream<StreamCfg<2, 3>>(p, sk, st);
    if (rc == MKQ_OK) rc = launch_stream<StreamCfg<4, 3>>(p, sk, st);
    return rc;
}

}  // namespace mkq

using namespace mkq;

extern "C" size_t mkq_stream_weight_bytes(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0) return 0;
    return (size_t)stream_pitch_panels((int)N) * 32 * (size_t)(K / 2);
}

extern "C" int mkq_repack_weights_int4_stream(const uint8_t *Wq, int64_t N, int64_t K, uint8_t *Wq_stream_out,
                                              void *stream)
{
    if (N <= 0 || K <= 0 || (K % 64) != 0) return MKQ_ERR_SHAPE;
    if (!Wq || !Wq_stream_out) return MKQ_ERR_NULL;
    if (!aligned16(Wq) || !aligned16(Wq_stream_out)) return MKQ_ERR_ALIGN;
    if (N > 0x7FFFFFFF || K >= 131072) return MKQ_ERR_UNSUPPORTED;
    const int64_t chunks = (int64_t)(mkq_stream_weight_bytes(N, K) / 16);
    repack_stream_kernel<<<(unsigned)ceil_div(chunks, 256), 256, 0, as_stream(stream)>>>(
        reinterpret_cast<const uint4 *>(Wq), reinterpret_cast<uint4 *>(Wq_stream_out), (int)N, (int)K, chunks);
    return launch_status();
}
