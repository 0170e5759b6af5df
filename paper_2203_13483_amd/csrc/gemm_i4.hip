// int4 x int4 -> int32 GEMM with fused dequantize / activation / requantize
// epilogue for gfx950 (CDNA4), the hot loop of the W4A4 linear layer.
//
// CDNA4 has no 4-bit integer MFMA, so nibbles are widened to int8 on the way from
// LDS to the matrix core.  The widening costs three VALU ops per eight codes: for
// a 32-bit word w of eight two's-complement nibbles,
//     hi = w & 0xF0F0F0F0          -> four int8 lanes equal to 16 * (odd codes)
//     lo = (w << 4) & 0xF0F0F0F0   -> four int8 lanes equal to 16 * (even codes)
// (the nibble's sign bit lands in bit 7 of its byte).  Both operands carry the
// factor 16, so the int32 accumulator holds exactly 256 * sum(a*w).  |sum| <= 64 K,
// so nothing overflows while 256 * 64 * K < 2^31, i.e. K < 131072.  The lo/hi split
// permutes k inside a word identically for both operands, which a dot product does
// not see.  The factor 256 is removed for free in the epilogue: the accumulator's
// low 8 bits are zero, so it has at most 18 significant bits and converts to
// binary32 exactly; the per-channel scale is pre-multiplied by 2^-8 (exact), and
// fma(256*sum, scale/256, bias) rounds the same real number as fma(sum, scale, bias).
//
// Data flow: packed rows of A [M, K/2] and W [N, K/2] (both K-contiguous) are
// fetched with 128-bit global loads into registers one stage ahead, written to
// LDS tiles of RB bytes per row (XOR-swizzled at 16-byte granularity so that the
// staging writes and the ds_read_b128 fragment reads are bank-conflict free), and
// each lane reads 16 bytes (32 codes) of one row, feeding two MFMA k-steps.
// W is the MFMA "A" operand and the activations the "B" operand; W rows are read
// in a permuted order so that a lane ends up with runs of 8 consecutive output
// channels of one token and stores them with one or two vector stores.
#include "gemm_i4_params.h"
#include "mkq_tuning.h"

namespace mkq {

// few-token weight-streaming kernel (gemm_i4_stream.hip)
bool gemm_i4_stream_ok(const GemmI4Params &p);
int run_gemm_i4_stream(const GemmI4Params &p, const SplitKScratch *scr, int forced_ks, hipStream_t st);
int setup_gemm_i4_stream(const GemmI4Params &p, hipStream_t st);
int run_gemm_i4_wstream(const GemmI4Params &p, const SplitKScratch *scr, int forced_ks, int variant, hipStream_t st);
int gemm_i4_stream_slices(const GemmI4Params &p, const SplitKScratch *scr, int forced_ks);

template <class Cfg, bool FULL_STAGES>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_i4_kernel(const GemmI4Params p)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, RB = Cfg::RB, CH = Cfg::CH;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, ROUNDS = Cfg::ROUNDS;
    constexpr int THREADS = Cfg::THREADS;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
    const int fr = lane & 31;  // row inside a 32-row fragment
    const int fh = lane >> 5;  // which 16-byte half of a 32-byte k slice

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const int total_tiles = tiles_m * tiles_n;
    const int row_bytes = p.K / 2;
    const int kt_count = (row_bytes + RB - 1) / RB;

    // The workgroup is persistent: it owns tiles blockIdx.x, blockIdx.x + gridDim.x, ...
    // and runs ONE software pipeline over all their k stages, so the loads of a tile's
    // first stages are already in flight while the previous tile's epilogue runs.
    const int my_tiles = (total_tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int steps = my_tiles * kt_count;

    // --- staging: which 16-byte chunks this thread copies each stage -------------
    uint4 ra[Cfg::A_PER_T], rw[Cfg::W_PER_T];
    uint32_t ga[Cfg::A_PER_T], gw[Cfg::W_PER_T];  // byte offsets of the chunks at k = 0
    int sa[Cfg::A_PER_T], sw[Cfg::W_PER_T];
    const int my_c = (tid % CH) * 16;  // byte offset of this thread's chunk inside a stage row
#pragma unroll
    for (int i = 0; i < Cfg::A_PER_T; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / CH, c = idx % CH;
        sa[i] = row * RB + ((c ^ swz<CH>(row & 15)) * 16);
    }
#pragma unroll
    for (int i = 0; i < Cfg::W_PER_T; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / CH, c = idx % CH;
        sw[i] = BM * RB + row * RB + ((c ^ swz<CH>(row & 15)) * 16);
    }
    auto set_tile = [&](int tile) {
        int tm, tn;
        tile_coords(tile, tiles_m, tiles_n, tm, tn);
#pragma unroll
        for (int i = 0; i < Cfg::A_PER_T; ++i) {
            const int idx = tid + i * THREADS;
            int gm = tm * BM + idx / CH;
            gm = gm < p.M ? gm : p.M - 1;  // rows past the edge re-read the last row; never stored
            ga[i] = (uint32_t)gm * (uint32_t)row_bytes + my_c;
        }
#pragma unroll
        for (int i = 0; i < Cfg::W_PER_T; ++i) {
            const int idx = tid + i * THREADS;
            int gn = tn * BN + idx / CH;
            gn = gn < p.N ? gn : p.N - 1;
            gw[i] = (uint32_t)gn * (uint32_t)row_bytes + my_c;
        }
    };

    int lt = blockIdx.x, lk = 0;  // load cursor: tile and k stage of the next stage to fetch
    set_tile(lt);
    auto load_next = [&]() {
        const int kb = lk * RB;
        const bool in = FULL_STAGES || (kb + my_c < row_bytes);
#pragma unroll
        for (int i = 0; i < Cfg::A_PER_T; ++i)
            ra[i] = in ? *reinterpret_cast<const uint4 *>(p.A + ga[i] + kb) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < Cfg::W_PER_T; ++i)
            rw[i] = in ? *reinterpret_cast<const uint4 *>(p.W + gw[i] + kb) : make_uint4(0, 0, 0, 0);
        if (++lk == kt_count) {
            lk = 0;
            lt += gridDim.x;
            if (lt < total_tiles) set_tile(lt);
        }
    };
    auto store_stage = [&](int buf) {
        uint8_t *base = smem + buf * Cfg::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < Cfg::A_PER_T; ++i) *reinterpret_cast<uint4 *>(base + sa[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < Cfg::W_PER_T; ++i) *reinterpret_cast<uint4 *>(base + sw[i]) = rw[i];
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][t][v] = 0;

    // fragment read offsets (bytes inside a stage) and the lane's swizzle keys
    int offA[TM], offW[TN], keyA[TM], keyW[TN];
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int row = wm * Cfg::WTM + j * 32 + fr;
        offA[j] = row * RB;
        keyA[j] = swz<CH>(row & 15);
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int row = wn * Cfg::WTN + t * 32 + w_row_perm(fr);
        offW[t] = BM * RB + row * RB;
        keyW[t] = swz<CH>(row & 15);
    }

    auto compute_round = [&](const uint8_t *base, int r) {
        const int c = r * 2 + fh;
        uint4 fw[TN], fa[TM];
#pragma unroll
        for (int t = 0; t < TN; ++t)
            fw[t] = *reinterpret_cast<const uint4 *>(base + offW[t] + ((c ^ keyW[t]) * 16));
#pragma unroll
        for (int j = 0; j < TM; ++j)
            fa[j] = *reinterpret_cast<const uint4 *>(base + offA[j] + ((c ^ keyA[j]) * 16));
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i wv[TN], av[TM];
#pragma unroll
            for (int t = 0; t < TN; ++t) wv[t] = ks ? widen(fw[t].z, fw[t].w) : widen(fw[t].x, fw[t].y);
#pragma unroll
            for (int j = 0; j < TM; ++j) av[j] = ks ? widen(fa[j].z, fa[j].w) : widen(fa[j].x, fa[j].y);
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int t = 0; t < TN; ++t)
                    acc[j][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wv[t], av[j], acc[j][t], 0, 0, 0);
        }
    };

    auto epilogue = [&](int tile) {
        int tile_m, tile_n;
        tile_coords(tile, tiles_m, tiles_n, tile_m, tile_n);
        gemm_i4_epilogue<Cfg, EpiGeneric>(p, acc, tile_m * BM, tile_n * BN, wm, wn, fr, fh);
    };  // epilogue

    // --- main loop: LDS double buffer, registers hold the stage after next --------
    load_next();
    store_stage(0);
    if (steps > 1) load_next();
    lds_barrier();

    int ct = blockIdx.x, ck = 0;  // compute cursor
    for (int s = 0; s < steps; ++s) {
        const uint8_t *base = smem + (s & 1) * Cfg::STAGE_BYTES;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            compute_round(base, r);
            if (r == ROUNDS / 2 - 1) {
                // the other buffer was last read in the previous step, before its barrier
                if (s + 1 < steps) store_stage((s + 1) & 1);
                if (s + 2 < steps) load_next();
            }
        }
        lds_barrier();
        if (++ck == kt_count) {
            epilogue(ct);
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[j][t][v] = 0;
            ck = 0;
            ct += gridDim.x;
        }
    }
}

// ---------------------------------------------------------------------------------
// Fast path: direct global->LDS copies (global_load_lds_dwordx4) into a ring of S
// stage buffers.  Needs whole stages (K/2 a multiple of RB) because the copy cannot
// zero-fill.  A wave-level copy instruction writes 64 x 16 bytes to consecutive LDS
// addresses (M0 + 16 * lane), i.e. 1024/RB whole tile rows; the XOR swizzle is
// applied on the global side (a lane fetches chunk slot ^ swz(row) of its row), so
// every row is still read as one contiguous RB-byte segment.  The copies bypass the
// registers, which lets S-1 stages be in flight per wave -- several microseconds of
// prefetch, enough to cover HBM latency even for small tiles -- and the compiler
// does not see them, so waiting is explicit: s_waitcnt vmcnt(n) with n = the copies
// issued after the stage that is about to be read, then one workgroup barrier.
template <int BM_, int BN_, int WGM_, int WGN_, int RB_, int S_>
struct GemmI4DmaCfg : GemmI4Cfg<BM_, BN_, WGM_, WGN_, RB_> {
    using Base = GemmI4Cfg<BM_, BN_, WGM_, WGN_, RB_>;
    static constexpr int S = S_;
    static constexpr int WAVES = WGM_ * WGN_;
    static constexpr int ROWS_PER_COPY = 1024 / RB_;
    static constexpr int COPIES = Base::STAGE_BYTES / 1024;  // per stage, whole workgroup
    static constexpr int LPW = COPIES / WAVES;               // per stage, per wave
    static constexpr int LDS_BYTES = S * Base::STAGE_BYTES;
    // resident waves per SIMD the kernel is compiled for: as many workgroups as the LDS
    // holds (at most 2 are useful), one wave of each per SIMD per WAVES / 4
    // two (small per-wave tiles: up to four, 128 registers each then) resident workgroups
    static constexpr int WGS_FIT = 160 * 1024 / (LDS_BYTES + WAVES * 512);
    static constexpr int WGS_WANT = (Base::TM * Base::TN <= 2) ? 4 : (Base::TM * Base::TN <= 4 ? 3 : 2);
    static constexpr int WGS_PER_CU = WGS_FIT < 1 ? 1 : (WGS_FIT < WGS_WANT ? WGS_FIT : WGS_WANT);
    static constexpr int WAVES_PER_EU = WGS_PER_CU * WAVES / 4;
    static_assert(COPIES % WAVES == 0, "copies must divide evenly over the waves");
    static_assert(BM_ % ROWS_PER_COPY == 0, "a copy must not straddle the A / W boundary");
    // Stages in flight right after a stage's copies are issued.  With one 64-code round
    // per stage a stage is entirely in registers before its own k steps start, so its
    // slot is refilled one stage earlier than with two rounds per stage.
    static constexpr int INFLIGHT = (RB_ == 64) ? S - 2 : S - 1;
    static_assert(RB_ == 32 || RB_ == 64, "a stage is one or two 64-code rounds");
    static_assert(S >= 3 && INFLIGHT * LPW <= 63, "vmcnt immediate is 6 bits");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS is 160 KiB per CU");
};

// Exchange buffer of the K split: per pass every wave of a non-first group hands over TPP of its
// 32x32 accumulator tiles (4 KiB each); tiles of 32x32 per wave need one pass, larger wave tiles go two
// tiles at a time so that the buffer fits beside the groups' rings.
template <class Cfg>
struct KSplitXch {
    static constexpr int TPP = (Cfg::TM * Cfg::TN >= 2) ? 2 : 1;
    static_assert((Cfg::TM * Cfg::TN) % TPP == 0, "whole passes");
    static constexpr int bytes(int ksplit) { return (ksplit - 1) * Cfg::WAVES * TPP * 4096; }
    static constexpr int lds(int ksplit)
    {
        return ksplit * (Cfg::LDS_BYTES + EpiShuffle<Cfg>::EXTRA_LDS) + bytes(ksplit);
    }
    // waves per SIMD the register allocator may assume: the configuration's own, except for split
    // workgroups of multi-tile waves, which are placed by their LDS footprint
    static constexpr int waves_per_eu(int ksplit)
    {
        return (ksplit == 1 || Cfg::TM * Cfg::TN == 1) ? Cfg::WAVES_PER_EU
                                                       : (160 * 1024 / lds(ksplit)) * Cfg::WAVES * ksplit / 4;
    }
};

// log2 of the wave-priority time slice, in shader cycles (0 = off); 2^15 measured best (2-4 %)
constexpr int PRIO_SLICE_LOG2 = 15;

// BITS = 4: nibble-packed operands, widened on the way to the matrix core.  BITS = 8: the
// operands are int8 codes already (the W8A8 comparison path): same ring, same epilogues, a
// 64-byte stage is then two k steps of 32 codes and nothing is widened.
// KSPLIT = 2 or 4: the workgroup is that many groups of Cfg::WAVES waves, each running this
// pipeline with a ring of its own over one share of K (for launches with few tiles and a long
// k loop, where a lone wave per SIMD is bound by its own instruction stream); the other groups'
// partial accumulators meet the first group's in LDS at the end of a tile and the first group
// runs the epilogue.
// XS: the reduction over K of an output tile is, beyond that, cut into p.ks slices that different workgroups
// sum (few tokens against a weight matrix with few output channels give too few tiles to fill the chip).
// The persistent loop then runs over (tile, slice) pairs; at the end of a pair the workgroup stores its partial
// accumulators to the caller's scratch area and draws a ticket on the tile's counter, and the one that draws the
// last ticket adds the others' partials to its registers and runs the epilogue ("last ticket": nobody waits
// for anybody, so the grid drains in any scheduling order).  int32 addition is associative: same bits as unsplit.
template <class Cfg, class Epi, int BITS, int KSPLIT = 1, bool XS = false>
__global__ __launch_bounds__(Cfg::THREADS * KSPLIT)
__attribute__((amdgpu_waves_per_eu(KSplitXch<Cfg>::waves_per_eu(KSPLIT), KSplitXch<Cfg>::waves_per_eu(KSPLIT))))
void gemm_i4_dma_kernel(const GemmI4Params p)
{
    const int ks = XS ? p.ks : 1;
    static_assert(BITS == 4 || (BITS == 8 && Cfg::RB == 64), "8-bit operands use 64-byte stages");
    static_assert(KSPLIT == 1 || KSPLIT == 2 || KSPLIT == 4, "one, two or four wave groups");
    constexpr int BM = Cfg::BM, BN = Cfg::BN, RB = Cfg::RB, CH = Cfg::CH;
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    constexpr int S = Cfg::S, LPW = Cfg::LPW;
    constexpr int ROUNDS = Cfg::ROUNDS, INFLIGHT = Cfg::INFLIGHT;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem_all[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave_all / Cfg::WAVES;   // K half of this wave's group (0 when KSPLIT == 1)
    const int wave = wave_all % Cfg::WAVES;
    // per group: the ring, then the scale / bias area of the row epilogue; after the groups: the
    // exchange buffer of the K split
    constexpr int GROUP_LDS = Cfg::LDS_BYTES + EpiShuffle<Cfg>::EXTRA_LDS;
    uint8_t *const smem = smem_all + grp * GROUP_LDS;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
    const int fr = lane & 31, fh = lane >> 5;

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const int total_tiles = tiles_m * tiles_n * ks;     // (tile, slice) pairs: pair v is slice v % ks of tile v / ks
    const int row_bytes = p.K * BITS / 8;
    const int kt_count = row_bytes / RB / KSPLIT / ks;  // stages per pair of this group
    // Persistent workgroup: pairs blockIdx.x, blockIdx.x + gridDim.x, ... run through ONE
    // software pipeline, so a tile's first stages are in flight during the previous
    // tile's epilogue.
    const int my_tiles = (total_tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int steps = my_tiles * kt_count;

    // copy q of this wave fills stage bytes [(wave*LPW + q) * 1024, +1024)
    uint32_t goff[LPW];  // byte offset (from A or W) of this lane's chunk at k = 0
    const int c_row = lane / CH;   // row inside the copy
    const int c_slot = lane % CH;  // 16-byte slot inside the row
    int k_first = 0;  // first byte, in a row, of this group's K range in the pair the copy cursor is in
    auto set_tile = [&](int pair) {
        int tm, tn;
        tile_coords(pair / ks, tiles_m, tiles_n, tm, tn);
        k_first = ((pair % ks) * KSPLIT + grp) * kt_count * RB;
#pragma unroll
        for (int q = 0; q < LPW; ++q) {
            const int row = (wave * LPW + q) * Cfg::ROWS_PER_COPY + c_row;  // stage row
            const int chunk = c_slot ^ swz<CH>(row & 15);
            int g;
            if (row < BM) {
                g = tm * BM + row;
                g = g < p.M ? g : p.M - 1;  // rows past the edge re-read the last row; never stored
            } else {
                g = tn * BN + (row - BM);
                g = g < p.N ? g : p.N - 1;
            }
            goff[q] = (uint32_t)g * (uint32_t)row_bytes + chunk * 16;
        }
    };
    v16i acc[TM][TN];
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][t][v] = 0;

    // Per-lane LDS read offsets of every fragment for the two 64-code rounds of a stage.
    // Fragments are numbered W first (0 .. TN-1), then activations (TN .. TN+TM-1).
    constexpr int NF = TN + TM;
    constexpr int NMFMA = TM * TN;
    int rd[NF][ROUNDS];
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int row = wn * Cfg::WTN + t * 32 + w_row_perm(fr);
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) rd[t][r] = (BM + row) * RB + (((r * 2 + fh) ^ swz<CH>(row & 15)) * 16);
    }
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int row = wm * Cfg::WTM + j * 32 + fr;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) rd[TN + j][r] = row * RB + (((r * 2 + fh) ^ swz<CH>(row & 15)) * 16);
    }

    // Software pipeline over k steps of 32 codes, four per 64-byte stage.  A k step is
    // NMFMA "slots": one MFMA each, followed by its share of the VALU widening of the
    // NEXT step's operands and, in steps 0 and 2, one LDS fragment read of the next
    // 64-code round (consumed a whole step later) and, in step 2, one global->LDS copy.
    // Slots are fenced with scheduling barriers so the matrix pipe always has the next
    // MFMA queued while the wave's VALU work runs in the shadow of the current one.
    uint32_t raw[2][NF][4];  // packed fragments of two rounds
    v4i wid[2][NF];          // widened operands of two k steps

    auto read_frag = [&](int stage_off, auto fc, auto rc, uint32_t(&dst)[4]) {
        constexpr int f = decltype(fc)::value, r = decltype(rc)::value;
        const uint4 v = *reinterpret_cast<const uint4 *>(smem + stage_off + rd[f][r]);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    };
    // register q of the widened operand: codes of word 2*ks + q/2, even (q even) or odd nibbles
    auto widen_reg = [&](const uint32_t(&src)[4], auto ksc, auto qc) -> int {
        constexpr int ks = decltype(ksc)::value, q = decltype(qc)::value;
        const uint32_t w = src[2 * ks + q / 2];
        return (int)(((q & 1) ? w : (w << 4)) & 0xF0F0F0F0u);
    };

    int lt = blockIdx.x, lk = 0;  // copy cursor
    set_tile(lt);
    // Per copy: one SALU op (M0 = LDS destination) and the copy itself.  The k offset
    // of the stage is folded into two base pointers that are advanced once per stage.
    const uint8_t *a_k = p.A + k_first, *w_k = p.W + k_first;
    const uint32_t lds_wave = lds0 + wave * (LPW * 1024);
    auto copy_one = [&](int slot, auto qc) {
        constexpr int q = decltype(qc)::value;
        const bool is_a = (wave * LPW + q) * Cfg::ROWS_PER_COPY < BM;  // wave-uniform
        dma_copy16<q * 1024>(is_a ? a_k : w_k, goff[q], lds_wave + slot * Cfg::STAGE_BYTES);
    };
    // Always issues LPW copies per stage, so the number in flight never depends on where
    // the pipeline is: past the last stage it re-fetches the last tile's stages into
    // slots that are never read again.
    auto copy_advance = [&]() {
        a_k += RB;
        w_k += RB;
        if (++lk == kt_count) {
            lk = 0;
            if (lt + (int)gridDim.x < total_tiles) {
                lt += gridDim.x;
                set_tile(lt);
            }
            a_k = p.A + k_first;
            w_k = p.W + k_first;
        }
    };

    // One k step.  H = step inside the stage.  Operands: wid[H & 1]; widens the next
    // step's into wid[(H + 1) & 1] from raw[SRC] half KS; READ: fetch round RR of the
    // stage at rd_off into raw[RB_]; COPY: issue this wave's copies into ring slot cslot.
    auto k_step = [&](auto hc, int rd_off, int cslot) {
        constexpr int H = decltype(hc)::value;
        constexpr int cb = H & 1, nb = cb ^ 1;
        constexpr int SRC = (H == 1 || H == 2) ? 1 : 0;   // raw buffer the next step is widened from
        constexpr int KS = (H == 0 || H == 2) ? 1 : 0;    // which half of it
        constexpr bool READ = (H == 0 || H == 2);
        constexpr int RDST = (H == 0) ? 1 : 0;            // raw buffer the reads fill
        constexpr int RR = (H == 0 && ROUNDS == 2) ? 1 : 0;  // round they fetch
        constexpr bool COPY = (H == 2) || (H == 0 && ROUNDS == 1);  // reads cross into the next stage
        static_for<NMFMA>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int j = i / TN, t = i % TN;
            if constexpr (Cfg::WAVES_PER_EU == 1) {
                // a single wave owns the SIMD's 512 registers: keep the accumulators in the
                // AGPR half by construction
                asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0"
                             : "+a"(acc[j][t]) : "v"(wid[cb][t]), "v"(wid[cb][TN + j]));
            } else {
                acc[j][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wid[cb][t], wid[cb][TN + j], acc[j][t], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (READ) {
                constexpr int f0 = i * NF / NMFMA, f1 = (i + 1) * NF / NMFMA;
                static_for<f1 - f0>([&](auto fc) {
                    constexpr int f = f0 + decltype(fc)::value;
                    read_frag(rd_off, IntC<f>{}, IntC<RR>{}, raw[RDST][f]);
                });
            }
            if constexpr (COPY) {
                constexpr int q0 = i * LPW / NMFMA, q1 = (i + 1) * LPW / NMFMA;
                static_for<q1 - q0>([&](auto qc) { copy_one(cslot, IntC<q0 + decltype(qc)::value>{}); });
            }
            constexpr int m0 = i * 4 * NF / NMFMA, m1 = (i + 1) * 4 * NF / NMFMA;
            static_for<m1 - m0>([&](auto mc) {
                constexpr int m = m0 + decltype(mc)::value;
                int w = widen_reg(raw[SRC][m / 4], IntC<KS>{}, IntC<m % 4>{});
                // pin the op to this slot: without a use here the optimizer sinks it to the
                // operand's first use, a whole k step (and possibly a branch) later
                asm volatile("" : "+v"(w));
                wid[nb][m / 4][m % 4] = w;
            });
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // 8-bit operands: one k step per 32-byte round, two per stage.  Step H multiplies the round
    // in raw[H] while round H^1 (of this stage in step 0, of the next stage in step 1, which also
    // issues the wave's copies) is fetched into raw[H^1].
    auto k_step8 = [&](auto hc, int rd_off, int cslot) {
        constexpr int H = decltype(hc)::value;
        static_for<NMFMA>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int j = i / TN, t = i % TN;
            const v4i fw = {(int)raw[H][t][0], (int)raw[H][t][1], (int)raw[H][t][2], (int)raw[H][t][3]};
            const v4i fa = {(int)raw[H][TN + j][0], (int)raw[H][TN + j][1], (int)raw[H][TN + j][2],
                            (int)raw[H][TN + j][3]};
            acc[j][t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw, fa, acc[j][t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            constexpr int f0 = i * NF / NMFMA, f1 = (i + 1) * NF / NMFMA;
            static_for<f1 - f0>([&](auto fc) {
                constexpr int f = f0 + decltype(fc)::value;
                read_frag(rd_off, IntC<f>{}, IntC<H == 0 ? 1 : 0>{}, raw[H ^ 1][f]);
            });
            if constexpr (H == 1) {
                constexpr int q0 = i * LPW / NMFMA, q1 = (i + 1) * LPW / NMFMA;
                static_for<q1 - q0>([&](auto qc) { copy_one(cslot, IntC<q0 + decltype(qc)::value>{}); });
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    // prologue: put INFLIGHT + 1 stages in flight, wait for stage 0, prime the register pipeline
#pragma unroll
    for (int i = 0; i < INFLIGHT + 1; ++i) {
        static_for<LPW>([&](auto qc) { copy_one(i, qc); });
        copy_advance();
    }
    wait_vmcnt<INFLIGHT * LPW>();
    lds_barrier();
    static_for<NF>([&](auto fc) { read_frag(0, fc, IntC<0>{}, raw[0][decltype(fc)::value]); });
    if constexpr (BITS == 4) {
        static_for<4 * NF>([&](auto mc) {
            constexpr int m = decltype(mc)::value;
            wid[0][m / 4][m % 4] = widen_reg(raw[0][m / 4], IntC<0>{}, IntC<m % 4>{});
        });
    }

    // Epilogue stores share the in-order vmcnt counter with the copies.  For the
    // INFLIGHT stage boundaries that follow an epilogue the wanted copies are older than
    // those stores, so the stores may stay outstanding if the wait allows for their
    // exact number; that number is only known at compile time for interior tiles of the
    // fixed epilogues.
    // (the row epilogue issues the same number of 16-byte-per-lane stores as the direct one,
    // and with a 16-bit residual its loads are all older than its first store only for the
    // direct path, so that variant waits for everything)
    constexpr int STORES_PER_UNIT = Epi::generic ? 0 : (Epi::out == MKQ_F32 ? 2 : 1);
    constexpr int EPI_STORES = TN * 2 * TM * STORES_PER_UNIT;
    constexpr bool ASYNC_STORES = !Epi::generic && ((INFLIGHT - 1) * LPW + EPI_STORES <= 63);
    int stores_pending = 0;  // boundaries left that may leave the epilogue's stores in flight

    // Stage boundary: the next stage becomes readable (INFLIGHT-1 younger stages may stay
    // in flight); past the barrier every wave is done with the slot that is refilled next.
    // Two workgroups share a CU and the SIMD arbiter always serves the older wave first: the
    // first-placed workgroup runs at full speed, the second in its gaps (and alone at the end).
    // Each workgroup therefore takes the higher wave priority in alternate time slices of the
    // CU's cycle counter, in opposite phase, so both progress at the same average rate.
    const unsigned prio_phase = (2 * blockIdx.x >= gridDim.x) ? 1u : 0u;
    unsigned long long tnow = 0;
    auto stage_boundary = [&]() {
        if constexpr (Cfg::WGS_PER_CU == 2 && PRIO_SLICE_LOG2 > 0) {
            const unsigned hi = __builtin_amdgcn_readfirstlane(((unsigned)(tnow >> PRIO_SLICE_LOG2) ^ prio_phase) & 1u);
            if (hi) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
        if (ASYNC_STORES && stores_pending > 0) {
            wait_vmcnt<ASYNC_STORES ? (INFLIGHT - 1) * LPW + EPI_STORES : 0>();
            --stores_pending;
        } else {
            wait_vmcnt<(INFLIGHT - 1) * LPW>();
        }
        lds_barrier();
    };
    auto next_slot = [&](int b) { return (b + 1 == S) ? 0 : b + 1; };

    constexpr bool ROWS_EPI = !Epi::generic && EpiShuffle<Cfg>::usable;
    float *const sc_lds = reinterpret_cast<float *>(smem + Cfg::LDS_BYTES + wave * EpiShuffle<Cfg>::SCALE_BYTES);
    // copies s_w / bias of this wave's channels of tile `tile` to sc_lds
    auto stage_scales = [&](int pair) {
        int tm, tn;
        tile_coords(pair / ks, tiles_m, tiles_n, tm, tn);
        const uint32_t dst = lds0 + Cfg::LDS_BYTES + wave * EpiShuffle<Cfg>::SCALE_BYTES;
        static_for<EpiShuffle<Cfg>::NSL>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            int n = tn * BN + wn * Cfg::WTN + 64 * i + lane;
            n = n < p.N ? n : p.N - 1;
            dma_copy4<256 * i>(reinterpret_cast<const uint8_t *>(p.s_w), (uint32_t)n * 4u, dst);
            if (p.bias)
                dma_copy4<EpiShuffle<Cfg>::BIAS_AT * 4 + 256 * i>(reinterpret_cast<const uint8_t *>(p.bias),
                                                                  (uint32_t)n * 4u, dst);
        });
    };

    // The copies are issued INFLIGHT stages before the tile ends (or at its first stage):
    // by the epilogue every vector memory operation still in flight is then younger.
    const int scale_stage = kt_count > INFLIGHT ? kt_count - INFLIGHT : 0;

    int ct = blockIdx.x, ck = 0;  // compute cursor
    int buf = 0;                  // ring slot of the stage being computed
    for (int s = 0; s < steps; s += 3 - ROUNDS) {
        if constexpr (Cfg::WGS_PER_CU == 2 && PRIO_SLICE_LOG2 > 0) tnow = __builtin_readcyclecounter();  // used at the boundary
        if constexpr (ROWS_EPI) {
            if (grp == 0 && ck == scale_stage) stage_scales(ct);
        }
        if constexpr (BITS == 8) {
            const int nbuf = next_slot(buf);
            k_step8(IntC<0>{}, buf * Cfg::STAGE_BYTES, 0);
            stage_boundary();
            k_step8(IntC<1>{}, nbuf * Cfg::STAGE_BYTES, buf == 0 ? S - 1 : buf - 1);
            copy_advance();
            buf = nbuf;
            ck += 1;
        } else if constexpr (ROUNDS == 2) {
            // one 128-code stage: round 1 is fetched from the same stage, then the boundary,
            // then round 0 of the next stage while the slot of the previous one is refilled
            const int nbuf = next_slot(buf);
            k_step(IntC<0>{}, buf * Cfg::STAGE_BYTES, 0);
            k_step(IntC<1>{}, 0, 0);
            stage_boundary();
            k_step(IntC<2>{}, nbuf * Cfg::STAGE_BYTES, buf == 0 ? S - 1 : buf - 1);
            copy_advance();
            k_step(IntC<3>{}, 0, 0);
            buf = nbuf;
            ck += 1;
        } else {
            // two 64-code stages (the raw / wid register buffers alternate, so the body is
            // unrolled twice); each stage's own slot is refilled at its boundary
            int nbuf = next_slot(buf);
            stage_boundary();
            k_step(IntC<0>{}, nbuf * Cfg::STAGE_BYTES, buf);
            copy_advance();
            k_step(IntC<1>{}, 0, 0);
            buf = nbuf;
            nbuf = next_slot(buf);
            stage_boundary();
            k_step(IntC<2>{}, nbuf * Cfg::STAGE_BYTES, buf);
            copy_advance();
            k_step(IntC<3>{}, 0, 0);
            buf = nbuf;
            ck += 2;
        }

        if (ck == kt_count) {
            int tile_m, tile_n;
            tile_coords(ct / ks, tiles_m, tiles_n, tile_m, tile_n);
            if constexpr (KSPLIT > 1) {
                // the other groups hand their partial sums over, KSplitXch<Cfg>::TPP 32x32 tiles of a wave
                // (16 registers per lane, 4 KiB per tile) per pass through the exchange buffer
                constexpr int TPP = KSplitXch<Cfg>::TPP, PASSES = TM * TN / TPP;
                int *const xch = reinterpret_cast<int *>(smem_all + KSPLIT * GROUP_LDS) + wave * (TPP * 1024) + lane * 4;
                static_for<PASSES>([&](auto pc) {
                    constexpr int pass = decltype(pc)::value;
                    if (pass > 0) lds_barrier();  // the first group has read the previous pass
                    if (grp > 0) {
                        static_for<TPP>([&](auto uc) {
                            constexpr int u = decltype(uc)::value, i = pass * TPP + u, j = i / TN, t = i % TN;
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                *reinterpret_cast<int4 *>(xch + (grp - 1) * (Cfg::WAVES * TPP * 1024) + u * 1024 + q * 256) =
                                    make_int4(acc[j][t][4 * q], acc[j][t][4 * q + 1], acc[j][t][4 * q + 2],
                                              acc[j][t][4 * q + 3]);
                        });
                    }
                    lds_barrier();
                    if (grp == 0) {
                        static_for<TPP>([&](auto uc) {
                            constexpr int u = decltype(uc)::value, i = pass * TPP + u, j = i / TN, t = i % TN;
#pragma unroll
                            for (int g = 0; g < KSPLIT - 1; ++g)
#pragma unroll
                                for (int q = 0; q < 4; ++q) {
                                    const int4 v = *reinterpret_cast<const int4 *>(
                                        xch + g * (Cfg::WAVES * TPP * 1024) + u * 1024 + q * 256);
                                    acc[j][t][4 * q] += v.x; acc[j][t][4 * q + 1] += v.y;
                                    acc[j][t][4 * q + 2] += v.z; acc[j][t][4 * q + 3] += v.w;
                                }
                        });
                    }
                });
            }
            bool finish = true;  // this workgroup runs the tile's epilogue
            if constexpr (XS) {
                if (ks > 1) {
                    // partial tile of a wave: TM * TN blocks of 16 registers x 64 lanes; register pair q of all
                    // lanes is one contiguous 512-byte piece.  Agent-scope relaxed atomics: the stores write
                    // through to memory and the loads do not hit a stale line of this XCD's L2.
                    const int tile = ct / ks, slice = ct % ks;
                    constexpr size_t WAVE_WORDS = (size_t)TM * TN * 8 * 64;  // 64-bit words
                    uint64_t *const area = reinterpret_cast<uint64_t *>(p.sk_partials);
                    if (grp == 0) {
                        uint64_t *const mine = area + ((size_t)(tile * ks + slice) * Cfg::WAVES + wave) * WAVE_WORDS + lane;
#pragma unroll
                        for (int j = 0; j < TM; ++j)
#pragma unroll
                            for (int t = 0; t < TN; ++t)
#pragma unroll
                                for (int q = 0; q < 8; ++q) {
                                    const uint64_t v = (uint64_t)(uint32_t)acc[j][t][2 * q] |
                                                       ((uint64_t)(uint32_t)acc[j][t][2 * q + 1] << 32);
                                    __hip_atomic_store(mine + ((j * TN + t) * 8 + q) * 64, v, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT);
                                }
                    }
                    wait_vmcnt<0>();   // this wave's partials have reached memory (and every copy in flight has landed)
                    __syncthreads();   // ... and every other wave's
                    // whether this workgroup drew the last ticket is told through the first word of the first
                    // group's ring slot of the stage just finished (idle until the next stage boundary)
                    volatile int *const xs_last =
                        reinterpret_cast<volatile int *>(smem_all + ((buf == 0) ? S - 1 : buf - 1) * Cfg::STAGE_BYTES);
                    if (tid == 0) {
                        const unsigned old = __hip_atomic_fetch_add(p.sk_counters + tile, 1u, __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_AGENT);
                        const int last = old == (unsigned)(ks - 1);
                        if (last) __hip_atomic_store(p.sk_counters + tile, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        *xs_last = last;
                    }
                    __syncthreads();
                    finish = *xs_last != 0;
                    __syncthreads();  // (the slot serves the epilogue as scratch next)
                    if (finish && grp == 0) {
                        for (int o = 0; o < ks; ++o) {
                            if (o == slice) continue;
                            const uint64_t *theirs = area + ((size_t)(tile * ks + o) * Cfg::WAVES + wave) * WAVE_WORDS + lane;
#pragma unroll
                            for (int j = 0; j < TM; ++j)
#pragma unroll
                                for (int t = 0; t < TN; ++t)
#pragma unroll
                                    for (int q = 0; q < 8; ++q) {
                                        const uint64_t v = __hip_atomic_load(theirs + ((j * TN + t) * 8 + q) * 64,
                                                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                        acc[j][t][2 * q] += (int)(uint32_t)v;
                                        acc[j][t][2 * q + 1] += (int)(uint32_t)(v >> 32);
                                    }
                        }
                    }
                }
            }
            if (grp == 0 && finish) {
                if constexpr (ROWS_EPI) {
                    // the slot of the stage just finished is idle until every wave has passed
                    // the next stage boundary: each wave shuffles through its share of it
                    const int done_slot = (buf == 0) ? S - 1 : buf - 1;
                    // the scale / bias copies have landed: only the stage copies issued after
                    // them (INFLIGHT stages, or one per stage of a shorter tile) may be in flight
                    if (kt_count >= INFLIGHT) wait_vmcnt<INFLIGHT * LPW>();
                    else wait_vmcnt<LPW>();
                    // plain 16-bit outputs of 64-channel waves take the line epilogue, without its register
                    // cache of the scales (with it this kernel spills)
                    if constexpr (EpiLines16<Cfg, Epi>::usable)
                        gemm_epilogue_lines16<Cfg, Epi, false>(p, acc, tile_m * BM, tile_n * BN, wm, wn, lane,
                                                               smem + done_slot * Cfg::STAGE_BYTES +
                                                                   wave * EpiShuffle<Cfg>::REGION, sc_lds);
                    else
                        gemm_i4_epilogue_rows<Cfg, Epi>(p, acc, tile_m * BM, tile_n * BN, wm, wn, lane,
                                                        smem + done_slot * Cfg::STAGE_BYTES +
                                                            wave * EpiShuffle<Cfg>::REGION, sc_lds);
                } else {
                    gemm_i4_epilogue<Cfg, Epi>(p, acc, tile_m * BM, tile_n * BN, wm, wn, fr, fh);
                }
            }
            const bool interior = (tile_m + 1) * BM <= p.M && (tile_n + 1) * BN <= p.N;
            // (a group without stores must not count them in its waits)
            stores_pending = (ASYNC_STORES && interior && grp == 0 && finish) ? INFLIGHT : 0;
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[j][t][v] = 0;
            ck = 0;
            ct += gridDim.x;
        }
    }
    wait_vmcnt<0>();  // the trailing dummy copies must land before the LDS is released
}

// ---------------------------------------------------------------------------------
// Few tokens (M <= 128): the linear is a stream of the weight matrix, bound by HBM.
// One workgroup of 8 waves owns 32 output channels; the waves split K between them,
// each fetching its packed fragments straight from global memory into registers (no
// reuse between waves, so no LDS staging) with every load of its slice in flight at
// once, and the partial accumulators meet in LDS.  The activations ([M, K/2] bytes,
// resident in L2) are read the same way.  Waves 0 .. TB-1 then each sum one 32-token
// block over the 8 partials and run the generic epilogue on it.
struct SkinnyCfg {
    static constexpr int BM = 32, BN = 32, WGM = 1, WGN = 1, RB = 64;
    static constexpr int THREADS = 512, WAVES = 8;
    static constexpr int WTM = 32, WTN = 32, TM = 1, TN = 1;
};

// BITS = 8: the operands are int8 codes (the 8-bit linear): a 16-byte piece is one MFMA operand as it is.
template <int TB, int UG, int BITS = 4>
__global__ __launch_bounds__(SkinnyCfg::THREADS) void gemm_i4_skinny_kernel(const GemmI4Params p)
{
    __shared__ __attribute__((aligned(16))) int red[2][SkinnyCfg::WAVES][4][64][4];  // 64 KiB

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int fr = lane & 31, fh = lane >> 5;
    const int n0 = blockIdx.x * 32;
    const int row_bytes = p.K * BITS / 8;
    // A row is cut into groups of 128 bytes (256 4-bit codes), one cache line; a lane fetches
    // 64 contiguous bytes of its row per group (four 16-byte loads = eight k steps), so the
    // four loads of a group touch the same 32 lines.  Which codes a lane holds does not
    // matter to the dot product as long as weights and activations agree.
    const int groups = row_bytes / 128;
    const int gpw = (groups + SkinnyCfg::WAVES - 1) / SkinnyCfg::WAVES;
    const int g_begin = wave * gpw;
    const int g_end = (g_begin + gpw) < groups ? (g_begin + gpw) : groups;

    int wrow = n0 + w_row_perm(fr);
    wrow = wrow < p.N ? wrow : p.N - 1;  // rows past the edge are never stored
    const uint8_t *wp = p.W + (size_t)wrow * row_bytes + fh * 64;
    const uint8_t *ap[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        int tok = tb * 32 + fr;
        tok = tok < p.M ? tok : p.M - 1;
        ap[tb] = p.A + (size_t)tok * row_bytes + fh * 64;
    }

    v16i acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[tb][v] = 0;

    // The epilogue's per-channel scales and biases are first touched here, by the waves that will run
    // it, so that their round trip to memory overlaps the weight stream instead of following it.
    float touched = 0.0f;
    if (wave < 2) {
        int n = n0 + fr;
        n = n < p.N ? n : p.N - 1;
        touched = p.s_w[n] + (p.bias ? p.bias[n] : 0.0f);
    }

    // chunks of UG groups, the next chunk's loads in flight while this one is multiplied
    constexpr int NL = 4 * UG;  // 16-byte loads per chunk per operand row
    uint4 fw[2][NL], fa[2][TB][NL];
    auto fetch = [&](int buf, int g0) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            int g = g0 + u / 4;
            g = g < g_end ? g : g_end - 1;  // tail: fetched again, not used
            g = g < 0 ? 0 : g;
            const int off = g * 128 + (u % 4) * 16;
            fw[buf][u] = *reinterpret_cast<const uint4 *>(wp + off);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) fa[buf][tb][u] = *reinterpret_cast<const uint4 *>(ap[tb] + off);
        }
    };
    auto multiply = [&](int buf, int g0) {
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            if (g0 + u / 4 < g_end) {
                if constexpr (BITS == 8) {
                    const v4i w = {(int)fw[buf][u].x, (int)fw[buf][u].y, (int)fw[buf][u].z, (int)fw[buf][u].w};
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) {
                        const v4i a = {(int)fa[buf][tb][u].x, (int)fa[buf][tb][u].y, (int)fa[buf][tb][u].z, (int)fa[buf][tb][u].w};
                        acc[tb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w, a, acc[tb], 0, 0, 0);
                    }
                } else {
                    const v4i w0 = widen(fw[buf][u].x, fw[buf][u].y), w1 = widen(fw[buf][u].z, fw[buf][u].w);
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) {
                        acc[tb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w0, widen(fa[buf][tb][u].x, fa[buf][tb][u].y), acc[tb], 0, 0, 0);
                        acc[tb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(w1, widen(fa[buf][tb][u].z, fa[buf][tb][u].w), acc[tb], 0, 0, 0);
                    }
                }
            }
        }
    };
    if (g_begin < g_end) {
        fetch(0, g_begin);
        for (int g0 = g_begin; g0 < g_end; g0 += 2 * UG) {
            if (g0 + UG < g_end) fetch(1, g0 + UG);
            multiply(0, g0);
            if (g0 + 2 * UG < g_end) fetch(0, g0 + 2 * UG);
            if (g0 + UG < g_end) multiply(1, g0 + UG);
        }
    }

    asm volatile("" ::"v"(touched));  // (keeps the early loads)
    // reduce over the 8 waves, two token blocks per pass through LDS
#pragma unroll
    for (int pass = 0; pass < (TB + 1) / 2; ++pass) {
        if (pass) __syncthreads();
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int tb = 2 * pass + h;
            if (tb < TB) {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<int4 *>(&red[h][wave][q][lane][0]) =
                        make_int4(acc[tb][4 * q], acc[tb][4 * q + 1], acc[tb][4 * q + 2], acc[tb][4 * q + 3]);
            }
        }
        __syncthreads();
        if (wave < 2 && 2 * pass + wave < TB) {
            v16i sum[1][1];
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[0][0][v] = 0;
#pragma unroll
            for (int w = 0; w < SkinnyCfg::WAVES; ++w)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int4 t = *reinterpret_cast<const int4 *>(&red[wave][w][q][lane][0]);
                    sum[0][0][4 * q] += t.x; sum[0][0][4 * q + 1] += t.y;
                    sum[0][0][4 * q + 2] += t.z; sum[0][0][4 * q + 3] += t.w;
                }
            gemm_i4_epilogue<SkinnyCfg, EpiGeneric>(p, sum, (2 * pass + wave) * 32, n0, 0, 0, fr, fh);
        }
    }
}

template <int TB, int UG, int BITS = 4>
static int launch_skinny(const GemmI4Params &p, hipStream_t st)
{
    if (p.setup_only) return MKQ_OK;
    gemm_i4_skinny_kernel<TB, UG, BITS><<<(unsigned)ceil_div(p.N, 32), SkinnyCfg::THREADS, 0, st>>>(p);
    return launch_status();
}

// The same kernel on int8 codes (rows of K bytes: K % 128 == 0), M <= 64.
static int run_gemm_i8_skinny(const GemmI4Params &p, hipStream_t st)
{
    if (p.M <= 32) return p.K >= 4096 ? launch_skinny<1, 1, 8>(p, st) : launch_skinny<1, 2, 8>(p, st);
    return launch_skinny<2, 2, 8>(p, st);
}

static int run_gemm_i4_skinny(const GemmI4Params &p, hipStream_t st)
{
    // long rows: one group per chunk keeps the wave under 128 registers, so two workgroups share a CU and
    // one's ramp and reduction overlap the other's stream (4-6 % at K >= 8192, a loss of 3 % at K = 4096)
    if (p.M <= 32) return p.K >= 8192 ? launch_skinny<1, 1>(p, st) : launch_skinny<1, 2>(p, st);
    if (p.M <= 64) return launch_skinny<2, 2>(p, st);
    if (p.M <= 96) return launch_skinny<3, 1>(p, st);
    return launch_skinny<4, 1>(p, st);
}

template <class Cfg, bool FULL>
static int launch_one(const GemmI4Params &p, int64_t tiles, hipStream_t st)
{
    const size_t lds = 2 * (size_t)Cfg::STAGE_BYTES;
    static PerDeviceOnce once;  // per instantiation
    int64_t resident = 0;
    const int rc = resident_workgroups(once, gemm_i4_kernel<Cfg, FULL>, Cfg::THREADS, lds, 2, &resident);
    if (rc != MKQ_OK || p.setup_only) return rc;
    const unsigned grid = (unsigned)(tiles < resident ? tiles : resident);
    gemm_i4_kernel<Cfg, FULL><<<grid, Cfg::THREADS, lds, st>>>(p);
    return launch_status();
}

template <class Cfg>
static int launch_gemm_i4(const GemmI4Params &p, hipStream_t st)
{
    const int64_t tiles = ceil_div(p.M, Cfg::BM) * ceil_div(p.N, Cfg::BN);
    if (tiles > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    const bool full = ((p.K / 2) % Cfg::RB) == 0;
    return full ? launch_one<Cfg, true>(p, tiles, st) : launch_one<Cfg, false>(p, tiles, st);
}

template <class Cfg, class Epi, int BITS = 4, int KSPLIT = 1, bool XS = false>
static int launch_gemm_i4_dma(const GemmI4Params &p, hipStream_t st)
{
    const int64_t tiles = ceil_div(p.M, Cfg::BM) * ceil_div(p.N, Cfg::BN) * (XS ? p.ks : 1);
    if (tiles > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    constexpr bool rows_epi = !Epi::generic && EpiShuffle<Cfg>::usable;
    constexpr size_t lds_kernel =
        KSPLIT == 1 ? Cfg::LDS_BYTES + (rows_epi ? EpiShuffle<Cfg>::EXTRA_LDS : 0)
                    : KSplitXch<Cfg>::lds(KSPLIT);
    static_assert(lds_kernel <= 160 * 1024, "LDS is 160 KiB per CU");
    const size_t lds = lds_kernel;
    static PerDeviceOnce once;  // per instantiation
    int64_t resident = 0;
    const int rc = resident_workgroups(once, gemm_i4_dma_kernel<Cfg, Epi, BITS, KSPLIT, XS>, Cfg::THREADS * KSPLIT, lds,
                                       1 << 20, &resident);
    if (rc != MKQ_OK || p.setup_only) return rc;
    const unsigned grid = (unsigned)(tiles < resident ? tiles : resident);
    gemm_i4_dma_kernel<Cfg, Epi, BITS, KSPLIT, XS><<<grid, Cfg::THREADS * KSPLIT, lds, st>>>(p);
    return launch_status();
}

template <class Cfg>
static int launch_dma_by_epilogue(const GemmI4Params &p, int epi, hipStream_t st)
{
    switch (epi) {
    case EPI_F16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, false, false>>(p, st);
    case EPI_BF16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_BF16, false, false>>(p, st);
    case EPI_F32: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F32, false, false>>(p, st);
    case EPI_F16_RES16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, true, false>>(p, st);
    case EPI_I4_GELU: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_I4, false, true>>(p, st);
    case EPI_I4: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_I4, false, false>>(p, st);
    default: return launch_gemm_i4_dma<Cfg, EpiGeneric>(p, st);
    }
}

// Tiles whose k loop is also split across workgroups (p.ks slices, partial sums through the caller's scratch).
template <class Cfg, int KS>
static int launch_xsplit_by_epilogue(const GemmI4Params &p, int epi, hipStream_t st)
{
    switch (epi) {
    case EPI_F16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, false, false>, 4, KS, true>(p, st);
    case EPI_BF16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_BF16, false, false>, 4, KS, true>(p, st);
    case EPI_F16_RES16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, true, false>, 4, KS, true>(p, st);
    case EPI_I4_GELU: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_I4, false, true>, 4, KS, true>(p, st);
    default: return launch_gemm_i4_dma<Cfg, EpiGeneric, 4, KS, true>(p, st);
    }
}

// Tiles with the k loop split between two wave groups of one workgroup.
template <class Cfg, int KS>
static int launch_ksplit_by_epilogue(const GemmI4Params &p, int epi, hipStream_t st)
{
    switch (epi) {
    case EPI_F16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, false, false>, 4, KS>(p, st);
    case EPI_BF16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_BF16, false, false>, 4, KS>(p, st);
    case EPI_F32: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F32, false, false>, 4, KS>(p, st);
    case EPI_F16_RES16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, true, false>, 4, KS>(p, st);
    case EPI_I4_GELU: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_I4, false, true>, 4, KS>(p, st);
    case EPI_I4: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_I4, false, false>, 4, KS>(p, st);
    default: return launch_gemm_i4_dma<Cfg, EpiGeneric, 4, KS>(p, st);
    }
}

using DmaBig8 = GemmI4DmaCfg<256, 256, 2, 4, 64, 5>;   // 2 waves per SIMD, 128x64 per wave
using DmaMid = GemmI4DmaCfg<128, 128, 2, 2, 64, 4>;    // 64 KiB LDS: two workgroups per CU
using DmaSmall = GemmI4DmaCfg<64, 64, 2, 2, 64, 8>;

// Tile choice of the ring kernels, from sweeps over M = 256 .. 65536 at the BERT-base /
// BERT-large shapes (and 4096^2, 8192^2 weights).  Very large problems: 256x128 tiles, two
// workgroups per CU (18).  Few tiles: 64x64, four per CU (27; the launch is latency-bound,
// parallelism wins).  In between 128x128 with a three-stage ring, three per CU (29), or
// 128x64, four per CU (28), when 128x128 tiles would leave most of the 768 slots empty and
// the k loop is short.
static int choose_tiles(const GemmI4Params &p)
{
    const int64_t t128 = ceil_div(p.M, 128) * ceil_div(p.N, 128);
    const int64_t t128x64 = ceil_div(p.M, 128) * ceil_div(p.N, 64);
    const int64_t t256x128 = ceil_div(p.M, 256) * ceil_div(p.N, 128);
    const double ops = 2.0 * p.M * p.N * p.K;
    if (t256x128 >= 512 && ops >= 6e10) return 18;
    if (t128x64 <= 256) return 27;
    // GELU (and the code decision behind it) makes the epilogue a large share of a short tile: up to four 64x64
    // workgroups per CU spread it over all SIMDs (FFN-up at M = 1024: 9.2 instead of 10.4 us)
    if (p.act == MKQ_ACT_GELU && p.K < 2048 && ceil_div(p.M, 64) * ceil_div(p.N, 64) <= 1024) return 27;
    if (t128 >= 400 || p.K >= 2048) {
        // at most one 128x128 workgroup per CU and a long k loop: two wave groups share the tile's K
        // (a lone wave per SIMD is bound by its own instruction stream); 6-14 % at N = 768 / 1024,
        // K = 3072 ... 8192, M = 2560 ... 5120
        if (t128 <= 256 && p.K >= 2048 && (p.K % 256) == 0) return 35;
        return 29;
    }
    return 28;
}

// K split across workgroups of a tile kernel with BM x BN tiles and `groups` wave groups per workgroup: fills
// q.ks and the scratch pointers.  forced_ks: 0 = the largest power of two that keeps at least four 64-byte
// stages per wave group and pair, at most two (tile, slice) pairs per compute unit and partial sums that fit the scratch area.  Returns false when the
// split does not apply (no scratch, K does not divide, the partial sums or the tile count exceed the scratch).
static bool xsplit_plan(GemmI4Params &q, const SplitKScratch *scr, int BM, int BN, int groups, int forced_ks)
{
    if (!scr) return false;
    const int64_t tiles = ceil_div(q.M, BM) * ceil_div(q.N, BN);
    const int stages = q.K / 128 / groups;
    if ((q.K % (128 * groups)) != 0 || tiles > SPLITK_MAX_TILES) return false;
    int cus = 256;
    device_cus(&cus);
    int ks = forced_ks;
    if (ks <= 0) {
        ks = 1;
        while (ks < 32 && (stages % (2 * ks)) == 0 && stages / (2 * ks) >= 4 && tiles * 2 * ks <= 2 * cus &&
               (size_t)tiles * 2 * ks * BM * BN * sizeof(int32_t) <= scr->partial_bytes)
            ks *= 2;
    }
    if (ks < 1 || (stages % ks) != 0 || stages / ks < 2) return false;
    if ((size_t)tiles * ks * BM * BN * sizeof(int32_t) > scr->partial_bytes) return false;
    q.ks = ks;
    q.sk_counters = scr->counters;
    q.sk_partials = scr->partials;
    return true;
}

// forced_cfg: -1 = the library's own choice, otherwise one configuration by number (tuning interface);
// scr: scratch of a K split across workgroups, or null; forced_ks: 0 = automatic.
int run_gemm_i4(const GemmI4Params &p, hipStream_t st, int forced_cfg, const SplitKScratch *scr, int forced_ks)
{
    int cfg = forced_cfg;
    const bool dma_ok = (p.K % 128) == 0;  // whole 64-byte stages
    const int epi = classify_epilogue(p);
    if (cfg == 50) return gemm_i4_stream_ok(p) ? run_gemm_i4_stream(p, scr, forced_ks, st) : MKQ_ERR_UNSUPPORTED;
    if (cfg == 30) return (p.M <= 128 && (p.K % 256) == 0) ? run_gemm_i4_skinny(p, st) : MKQ_ERR_UNSUPPORTED;
    // Few tokens on canonical weights: up to 64 tokens the register kernel (the faster of the two at every
    // measured size); 65 .. 128 tokens against a large weight matrix the ring kernel with its shared
    // activation stages (60 instead of 88 us at K = N = 16384), against a small one the tile kernels.
    if (cfg < 0 && p.M <= 64 && (p.K % 256) == 0) return run_gemm_i4_skinny(p, st);
    if (cfg < 0 && gemm_i4_stream_ok(p) && (int64_t)p.N * p.K >= ((int64_t)1 << 27))
        return run_gemm_i4_stream(p, scr, forced_ks, st);
    if (cfg < 0) {
        if (!dma_ok) {
            cfg = 3;
        } else {
            cfg = choose_tiles(p);
        }
    }
    if (cfg >= 10 && !dma_ok) return MKQ_ERR_UNSUPPORTED;
    // few 64x64 tiles (at most two workgroups per CU) and a k loop long enough to halve: two wave
    // groups per workgroup, with the deeper ring when the k loop is very long (four groups gain
    // nothing over two: what is left is launch, first-load latency and the epilogue)
    if (forced_cfg < 0 && cfg == 27 && (p.K % 256) == 0 && p.K >= 512) {
        const int64_t t64 = ceil_div(p.M, 64) * ceil_div(p.N, 64);
        // (between one and two workgroups per CU the split pays only for a long k loop: at K = 768 the
        // unsplit tiles are 10 % faster there)
        // (the four-stage ring also for a weight matrix of 4 MiB and more, which comes from memory rather than
        // from the caches on most calls: 10.0-11.0 instead of 12.6-13.1 us at M = 65 ... 256, K = N = 4096 with a
        // different matrix on every call; with the same matrix every call the three-stage ring is 3 % faster)
        if (t64 <= 256 || (t64 <= 512 && p.K >= 2048))
            cfg = (t64 <= 256 && (p.K >= 6144 || (int64_t)p.N * p.K >= ((int64_t)8 << 20))) ? 31 : 33;
    }
    if ((cfg == 31 || cfg == 33 || cfg == 35) && (p.K % 256) != 0) return MKQ_ERR_UNSUPPORTED;
    if (cfg >= 60 && cfg <= 62) {  // tile kernels with the k loop also split across workgroups
        GemmI4Params q = p;
        if (cfg == 60) {
            if (!xsplit_plan(q, scr, 128, 128, 1, forced_ks)) return MKQ_ERR_UNSUPPORTED;
            return launch_xsplit_by_epilogue<GemmI4DmaCfg<128, 128, 2, 2, 64, 3>, 1>(q, epi, st);
        }
        if (cfg == 61) {
            if (!xsplit_plan(q, scr, 64, 64, 2, forced_ks)) return MKQ_ERR_UNSUPPORTED;
            return launch_xsplit_by_epilogue<GemmI4DmaCfg<64, 64, 2, 2, 64, 4>, 2>(q, epi, st);
        }
        if (!xsplit_plan(q, scr, 128, 64, 1, forced_ks)) return MKQ_ERR_UNSUPPORTED;
        return launch_xsplit_by_epilogue<GemmI4DmaCfg<128, 64, 2, 2, 64, 3>, 1>(q, epi, st);
    }
    switch (cfg) {
    case 2: return launch_gemm_i4<GemmI4Cfg<128, 128, 2, 2, 64>>(p, st);
    case 3: return launch_gemm_i4<GemmI4Cfg<64, 64, 2, 2, 64>>(p, st);
    case 11: return launch_dma_by_epilogue<DmaBig8>(p, epi, st);
    case 12: return launch_dma_by_epilogue<DmaMid>(p, epi, st);
    case 14: return launch_dma_by_epilogue<DmaSmall>(p, epi, st);
    case 18: return launch_dma_by_epilogue<GemmI4DmaCfg<256, 128, 2, 2, 64, 3>>(p, epi, st);
    case 19: return launch_dma_by_epilogue<GemmI4DmaCfg<128, 256, 2, 2, 64, 3>>(p, epi, st);
    case 20: return launch_dma_by_epilogue<GemmI4DmaCfg<256, 128, 2, 2, 32, 6>>(p, epi, st);
    case 27: return launch_dma_by_epilogue<GemmI4DmaCfg<64, 64, 2, 2, 64, 4>>(p, epi, st);
    case 28: return launch_dma_by_epilogue<GemmI4DmaCfg<128, 64, 2, 2, 64, 3>>(p, epi, st);
    case 29: return launch_dma_by_epilogue<GemmI4DmaCfg<128, 128, 2, 2, 64, 3>>(p, epi, st);
    case 31: return launch_ksplit_by_epilogue<GemmI4DmaCfg<64, 64, 2, 2, 64, 4>, 2>(p, epi, st);
    case 33: return launch_ksplit_by_epilogue<GemmI4DmaCfg<64, 64, 2, 2, 64, 3>, 2>(p, epi, st);
    case 35: return launch_ksplit_by_epilogue<GemmI4DmaCfg<128, 128, 2, 2, 64, 3>, 2>(p, epi, st);
    default: return MKQ_ERR_UNSUPPORTED;
    }
}

// 8-bit operands (W8A8 comparison path): [M, K] and [N, K] int8 codes, K a multiple of 64.
template <class Cfg>
static int launch_i8_by_epilogue(const GemmI4Params &p, int epi, hipStream_t st)
{
    switch (epi) {
    case EPI_F16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, false, false>, 8>(p, st);
    case EPI_BF16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_BF16, false, false>, 8>(p, st);
    case EPI_F32: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F32, false, false>, 8>(p, st);
    case EPI_F16_RES16: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_F16, true, false>, 8>(p, st);
    case EPI_I8_GELU: return launch_gemm_i4_dma<Cfg, EpiFixed<MKQ_I8, false, true>, 8>(p, st);
    default: return launch_gemm_i4_dma<Cfg, EpiGeneric, 8>(p, st);
    }
}

int run_gemm_i8(const GemmI4Params &p, hipStream_t st, int forced_cfg = -1)
{
    if ((p.K % 64) != 0) return MKQ_ERR_UNSUPPORTED;
    // few tokens: the linear is a stream of the weight matrix (the tile kernels take 24 us for 16 MiB of
    // weights where this takes 8)
    if (forced_cfg == 30) return (p.M <= 64 && (p.K % 128) == 0) ? run_gemm_i8_skinny(p, st) : MKQ_ERR_UNSUPPORTED;
    // (33 .. 64 tokens only against at least 4 MiB of weights: below that the tile kernels are 10-20 % faster)
    if (forced_cfg < 0 && (p.K % 128) == 0 && (p.M <= 32 || (p.M <= 64 && (int64_t)p.N * p.K >= ((int64_t)4 << 20))))
        return run_gemm_i8_skinny(p, st);
    int epi = classify_epilogue(p);
    if (epi == EPI_I4 || epi == EPI_I4_GELU) epi = EPI_GENERIC;
    switch (forced_cfg >= 0 ? forced_cfg : choose_tiles(p)) {
    case 18: return launch_i8_by_epilogue<GemmI4DmaCfg<256, 128, 2, 2, 64, 3>>(p, epi, st);
    case 29: return launch_i8_by_epilogue<GemmI4DmaCfg<128, 128, 2, 2, 64, 3>>(p, epi, st);
    case 28: return launch_i8_by_epilogue<GemmI4DmaCfg<128, 64, 2, 2, 64, 3>>(p, epi, st);
    default: return launch_i8_by_epilogue<GemmI4DmaCfg<64, 64, 2, 2, 64, 4>>(p, epi, st);
    }
}


// ---------------------------------------------------------------------------------
// Experimental: the same int4 x int4 -> exact integer contraction through the 6-bit float path of the
// matrix core.  Every code in [-8, 8] is an E3M2 value, products and sums of such values are exact in
// binary32 while |sum| < 2^24 (K < 2^18), and v_mfma_scale_f32_32x32x64_f8f6f4 with unit scales returns
// them exactly (checked by brute force in the tests).  Operands are stored as E3M2 codes, 6 bits each, in
// groups of 64 codes = 48 bytes: the 32 codes of half h of a group are one 192-bit MFMA operand of a lane,
// stored at bytes [16h, 16h + 16) and [32 + 8h, 40 + 8h) of the group, so that every lane fetches its
// operand with one aligned 16-byte and one aligned 8-byte LDS read.  No widening, and one MFMA covers 64
// codes of k.
// Tile 256 x 256, eight waves of 128 x 64, ring of 3 stages of 128 codes (96-byte rows = two container
// groups = two MFMA k steps, 48 KiB per stage, 48 wave copies of which every wave issues six); one
// persistent workgroup per CU.  The tile is this large and the stage rows this long because the route is
// bound by the number of 64-byte requests the global->LDS copies make, not by the matrix pipe: a 48-byte
// row segment straddles request boundaries (1.75 requests on average), a 96-byte one takes 1.5.
// (256 x 128 on four waves with a two-stage ring, two workgroups per CU, is the second shape.)
template <int BN_, int WGN_, int S_>
struct E3CfgT {
    static constexpr int BM = 256, BN = BN_, WGM = 2, WGN = WGN_, WAVES = WGM * WGN, THREADS = WAVES * 64;
    static constexpr int WTM = 128, WTN = 64, TM = 4, TN = 2;
    static_assert(BN == WGN * WTN, "waves of 128 x 64");
    // S slots keep S - 1 stages in flight: when a stage's second k step has been fetched by every wave its
    // slot is free for the stage S further on
    static constexpr int ROWB = 96, KSTEPS = 2, S = S_, STAGE_BYTES = (BM + BN) * ROWB, LDS_BYTES = S * STAGE_BYTES;
    static constexpr int CPR = ROWB / 16;                                   // 16-byte chunks per row
    static constexpr int A_COPIES = BM * CPR / 64, COPIES = (BM + BN) * CPR / 64, LPW = COPIES / WAVES;
    static_assert(COPIES % WAVES == 0 && (BM * CPR) % 64 == 0, "copies split evenly, none straddles A / W");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS is 160 KiB per CU");
};

template <class Cfg, class Epi>
__global__ __launch_bounds__(Cfg::THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
void gemm_e3m2_kernel(const GemmI4Params p)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, TM = Cfg::TM, TN = Cfg::TN, S = Cfg::S, ROWB = Cfg::ROWB;
    constexpr int LPW = Cfg::LPW, CPR = Cfg::CPR, WAVES = Cfg::WAVES;
    using Sh = EpiShuffle<Cfg>;
    static_assert(Cfg::WTN == 64 && Sh::NSL == 1, "one channel per lane in the scale copies");
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
    const int fr = lane & 31, fh = lane >> 5;
    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const int total_tiles = tiles_m * tiles_n;
    const int row_bytes = p.K / 4 * 3;
    const int kt_count = p.K / 128;

    // The workgroup is persistent: it walks tiles blockIdx.x, blockIdx.x + gridDim.x, ... and its copies
    // run ahead of the arithmetic as one stream of stages across tile boundaries, so the first stages of
    // a tile are fetched while the previous tile is still being multiplied and stored.
    // Copy q of this wave is stage copy c = wave + WAVES * q: chunks 64c .. 64c + 63, chunk g = row g / CPR,
    // slot g % CPR.
    uint32_t goff[LPW];
    auto set_fetch_tile = [&](int t) {
        int tm, tn;
        tile_coords(t, tiles_m, tiles_n, tm, tn);
        // (recomputed from the lane index at every tile change: kept across the k loop, the per-copy rows and
        // chunks would cost more registers than the wave has to spare)
        int l = lane;
        asm volatile("" : "+v"(l));
#pragma unroll
        for (int q = 0; q < LPW; ++q) {
            const int g = (wave + WAVES * q) * 64 + l;
            const int row = g / CPR, slot = g - row * CPR;
            // rows 8 .. 15 of every 16 hold their six chunks rotated by one: 16 consecutive rows then spread a
            // 16-byte column over all 64 banks (a row is 24 banks long)
            const int chunk = (slot + CPR - ((row >> 3) & 1)) % CPR;
            int src;
            if (row < BM) {
                src = tm * BM + row;
                src = src < p.M ? src : p.M - 1;  // rows past the edge re-read the last row; never stored
            } else {
                src = tn * BN + (row - BM);
                src = src < p.N ? src : p.N - 1;
            }
            goff[q] = (uint32_t)src * (uint32_t)row_bytes + chunk * 16;
        }
    };
    int ft = blockIdx.x, fk = 0;  // copy cursor: tile and stage; past the last tile it fetches that tile again
    set_fetch_tile(ft);
    auto issue = [&](int slot) {
        const int kb = fk * ROWB;
        const uint32_t dst = lds0 + slot * Cfg::STAGE_BYTES + wave * 1024;
        static_for<LPW>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            const bool is_a = (wave + WAVES * q) < Cfg::A_COPIES;  // wave-uniform
            dma_copy16<q * WAVES * 1024>((is_a ? p.A : p.W) + kb, goff[q], dst);
        });
        if (++fk == kt_count) {
            fk = 0;
            if (ft + (int)gridDim.x < total_tiles) {
                ft += gridDim.x;
                set_fetch_tile(ft);
            }
        }
    };
    // s_w and bias of the wave's 64 channels of tile t, copied to the wave's 512 bytes beyond the ring; always
    // SC copies, so the number of copies in flight never depends on the arguments
    constexpr int SC = 2;
    float *const sc_lds = reinterpret_cast<float *>(smem + Cfg::LDS_BYTES + wave * Sh::SCALE_BYTES);
    auto issue_scales = [&](int t) {
        int tm, tn;
        tile_coords(t, tiles_m, tiles_n, tm, tn);
        int n = tn * BN + wn * Cfg::WTN + lane;
        n = n < p.N ? n : p.N - 1;
        const uint32_t dst = lds0 + Cfg::LDS_BYTES + wave * Sh::SCALE_BYTES;
        dma_copy4<0>(reinterpret_cast<const uint8_t *>(p.s_w), (uint32_t)n * 4u, dst);
        dma_copy4<Sh::BIAS_AT * 4>(reinterpret_cast<const uint8_t *>(p.bias ? p.bias : p.s_w), (uint32_t)n * 4u, dst);
    };

    // fragment byte offsets inside a stage.  Logical chunk c of a row sits at chunk (c + rot) % 6, rot = bit 3
    // of the row.  K step r takes 16 bytes of chunk 3r + fh and 8 bytes (half fh) of chunk 3r + 2.
    // The rotation is the same for all row blocks of an operand (blocks are 32 rows apart), so one set of
    // offsets per operand serves every block with a constant added.
    int rdW[3], rdA[3];  // [0]: 16-byte read of k step 0 (k step 1: + 48), [1], [2]: the 8-byte reads
    auto offsets = [&](int row, int (&o)[3]) {
        const int rot = (row >> 3) & 1;
        o[0] = row * ROWB + (fh + rot) * 16;
        o[1] = row * ROWB + (2 + rot) * 16 + 8 * fh;
        o[2] = row * ROWB + (rot ? 0 : 80) + 8 * fh;
    };
    offsets(BM + wn * Cfg::WTN + w_row_perm(fr), rdW);
    offsets(wm * Cfg::WTM + fr, rdA);

    v16f acc[TM][TN];
    v8i fw[2][TN], fa[2][TM];  // fragments of two consecutive k steps
    // fragment of one operand row block: u = 0 .. TN-1: W blocks, TN .. TN+TM-1: A blocks
    auto read_one = [&](int sl, auto rc, auto bc, auto uc) {
        constexpr int r = decltype(rc)::value, b = decltype(bc)::value, u = decltype(uc)::value;
        const uint8_t *st = smem + sl * Cfg::STAGE_BYTES;
        if constexpr (u < TN) {
            const uint4 x = *reinterpret_cast<const uint4 *>(st + rdW[0] + (u * 32 * ROWB + r * 48));
            const uint2 y = *reinterpret_cast<const uint2 *>(st + rdW[1 + r] + u * 32 * ROWB);
            fw[b][u] = v8i{(int)x.x, (int)x.y, (int)x.z, (int)x.w, (int)y.x, (int)y.y, 0, 0};
        } else {
            constexpr int j = u - TN;
            const uint4 x = *reinterpret_cast<const uint4 *>(st + rdA[0] + (j * 32 * ROWB + r * 48));
            const uint2 y = *reinterpret_cast<const uint2 *>(st + rdA[1 + r] + j * 32 * ROWB);
            fa[b][j] = v8i{(int)x.x, (int)x.y, (int)x.z, (int)x.w, (int)y.x, (int)y.y, 0, 0};
        }
    };
    auto mfma_one = [&](auto bc, auto ic) {
        constexpr int b = decltype(bc)::value, i = decltype(ic)::value, j = i / TN, t = i % TN;
        acc[j][t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fw[b][t], fa[b][j], acc[j][t], 3, 3, 0, 0x7f7f7f7f,
                                                                    0, 0x7f7f7f7f);
    };

    // Epilogue stores share the in-order vmcnt counter with the copies.  At the S - 2 stage boundaries that
    // follow an epilogue the wanted copies are older than its stores, so the stores may stay outstanding if
    // the wait allows for their exact number (known for interior tiles of the fixed epilogues).
    constexpr int SPU = Epi::generic ? 0 : (Epi::out == MKQ_F32 ? 2 : 1);
    constexpr int EPI_STORES = TN * 2 * TM * SPU;
    constexpr int N0 = (S - 2) * LPW, N1 = N0 + EPI_STORES + SC;
    constexpr bool ASYNC_STORES = !Epi::generic && S >= 3 && N1 <= 63;
    int stores_pending = 0;

    // prologue: S stages and the first tile's scales in flight, stage 0 landed, its first k step in registers
#pragma unroll
    for (int i = 0; i < S; ++i) issue(i);
    issue_scales(blockIdx.x);
    wait_vmcnt<(S - 1) * LPW + SC>();
    lds_barrier();
    static_for<TM + TN>([&](auto uc) { read_one(0, IntC<0>{}, IntC<0>{}, uc); });
    int slot = 0;
    for (int tile = blockIdx.x; tile < total_tiles; tile += gridDim.x) {
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int t = 0; t < TN; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[j][t][v] = 0.0f;
        for (int s = 0; s < kt_count; ++s) {
            const int nslot = (slot + 1 == S) ? 0 : slot + 1;
            // k step 0 of the stage; one fragment block of its k step 1 is fetched behind each of the first
            // six MFMAs
            static_for<TM * TN>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                mfma_one(IntC<0>{}, ic);
                if constexpr (i < TM + TN) read_one(slot, IntC<1>{}, IntC<1>{}, ic);
                __builtin_amdgcn_sched_barrier(0);
            });
            // two MFMAs of k step 1 keep the matrix pipe busy across the boundary
            mfma_one(IntC<1>{}, IntC<0>{});
            mfma_one(IntC<1>{}, IntC<1>{});
            __builtin_amdgcn_sched_barrier(0);
            // boundary: the next stage has landed (the S - 2 stages after it may still be in flight); past
            // the barrier every wave holds all of this stage in registers, so its slot takes the stage S
            // further on -- except behind a tile's last stage, where the slot first serves the epilogue
            if (ASYNC_STORES && stores_pending > 0) {
                wait_vmcnt<ASYNC_STORES ? N1 : 0>();
                --stores_pending;
            } else {
                wait_vmcnt<N0>();
            }
            lds_barrier();
            if (s + 1 < kt_count) issue(slot);
            __builtin_amdgcn_sched_barrier(0);
            static_for<TM * TN - 2>([&](auto ic) {
                constexpr int i = decltype(ic)::value;
                read_one(nslot, IntC<0>{}, IntC<0>{}, ic);
                mfma_one(IntC<1>{}, IntC<i + 2>{});
                __builtin_amdgcn_sched_barrier(0);
            });
            slot = nslot;
        }

        const int done_slot = (slot == 0) ? S - 1 : slot - 1;  // idle: read by every wave, not yet refilled
        int tm, tn;
        tile_coords(tile, tiles_m, tiles_n, tm, tn);
        constexpr bool LINES16 = EpiLines16<Cfg, Epi>::usable;
        if constexpr (LINES16) {
            // the scale copies are older than every stage copy issued during the tile; a one-stage tile
            // issues none
            if (kt_count < 2) wait_vmcnt<0>();
            gemm_epilogue_lines16<Cfg, Epi>(p, acc, tm * BM, tn * BN, wm, wn, lane,
                                            smem + done_slot * Cfg::STAGE_BYTES + wave * 4096, sc_lds);
        } else {
            v16i acci[TM][TN];
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acci[j][t][v] = (int)acc[j][t][v];  // exact: integers below 2^24
            if constexpr (Epi::generic) {
                gemm_i4_epilogue<Cfg, Epi>(p, acci, tm * BM, tn * BN, wm, wn, fr, fh);
            } else {
                if (kt_count < 2) wait_vmcnt<0>();
                gemm_i4_epilogue_rows<Cfg, Epi>(p, acci, tm * BM, tn * BN, wm, wn, lane,
                                                smem + done_slot * Cfg::STAGE_BYTES + wave * 4096, sc_lds);
            }
        }
        const bool interior = (tm + 1) * BM <= p.M && (tn + 1) * BN <= p.N;
        stores_pending = (ASYNC_STORES && interior) ? S - 2 : 0;
        lds_barrier();  // every wave is done with its share of the slot
        issue(done_slot);
        issue_scales(tile + (int)gridDim.x < total_tiles ? tile + (int)gridDim.x : tile);
        // the next stage's first k step is fetched again rather than kept in registers across the epilogue
        static_for<TM + TN>([&](auto uc) { read_one(slot, IntC<0>{}, IntC<0>{}, uc); });
    }
    wait_vmcnt<0>();  // the trailing copies must land before the LDS is released
}

template <class Cfg, class Epi>
static int launch_gemm_e3m2(const GemmI4Params &p, hipStream_t st)
{
    const int64_t tiles = ceil_div(p.M, Cfg::BM) * ceil_div(p.N, Cfg::BN);
    if (tiles > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    constexpr int lds = Cfg::LDS_BYTES + EpiShuffle<Cfg>::EXTRA_LDS;
    static_assert(lds <= 160 * 1024, "LDS is 160 KiB per CU");
    static PerDeviceOnce once;  // per instantiation
    int64_t resident = 0;
    const int rc = resident_workgroups(once, gemm_e3m2_kernel<Cfg, Epi>, Cfg::THREADS, lds, (160 * 1024) / lds, &resident);
    if (rc != MKQ_OK || p.setup_only) return rc;
    const unsigned grid = (unsigned)(tiles < resident ? tiles : resident);
    gemm_e3m2_kernel<Cfg, Epi><<<grid, Cfg::THREADS, lds, st>>>(p);
    return launch_status();
}

template <class Cfg>
static int launch_e3m2_by_epilogue(const GemmI4Params &p, hipStream_t st)
{
    switch (classify_epilogue(p)) {
    case EPI_F16: return launch_gemm_e3m2<Cfg, EpiFixed<MKQ_F16, false, false>>(p, st);
    case EPI_BF16: return launch_gemm_e3m2<Cfg, EpiFixed<MKQ_BF16, false, false>>(p, st);
    case EPI_F32: return launch_gemm_e3m2<Cfg, EpiFixed<MKQ_F32, false, false>>(p, st);
    default: return launch_gemm_e3m2<Cfg, EpiGeneric>(p, st);
    }
}

int run_gemm_e3m2(const GemmI4Params &p, hipStream_t st, int forced_cfg)
{
    // 256 x 256 tiles (one 8-wave workgroup per CU) make the fewest global->LDS requests per MFMA; 256 x 128
    // (two 4-wave workgroups per CU) overlap one tile's epilogue with the other's k loop
    if (forced_cfg == 41) return launch_e3m2_by_epilogue<E3CfgT<256, 4, 3>>(p, st);
    if (forced_cfg == 42) return launch_e3m2_by_epilogue<E3CfgT<128, 2, 2>>(p, st);
    // (with a short k loop the large tile wins only when every workgroup walks many tiles: 8 % at
    // M = 65536, N = 4096, K = 1024, sixteen tiles per CU)
    const int64_t t256 = ceil_div(p.M, 256) * ceil_div(p.N, 256);
    if (p.K >= 2048 || t256 >= 2048) return launch_e3m2_by_epilogue<E3CfgT<256, 4, 3>>(p, st);
    return launch_e3m2_by_epilogue<E3CfgT<128, 2, 2>>(p, st);
}

}  // namespace mkq

using namespace mkq;

extern "C" size_t mkq_linear_int4_workspace_bytes(int64_t M, int64_t N, int64_t K, int a_dtype)
{
    (void)N;
    if (a_dtype == MKQ_I4 || M <= 0 || K <= 0) return 0;
    return ((size_t)M * (size_t)(K / 2) + 255) & ~(size_t)255;
}

extern "C" size_t mkq_splitk_scratch_bytes(void) { return SPLITK_STATE_BYTES + MKQ_SPLITK_PARTIAL_BYTES; }

namespace mkq {

__global__ void clear_words_kernel(unsigned *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// Splits a scratch area into ticket counters and room for partial sums.
static bool splitk_area(void *scratch, size_t bytes, SplitKScratch *out)
{
    if (!scratch || bytes <= SPLITK_STATE_BYTES + 65536) return false;
    out->counters = reinterpret_cast<unsigned *>(scratch);
    out->partials = reinterpret_cast<int32_t *>(reinterpret_cast<uint8_t *>(scratch) + SPLITK_STATE_BYTES);
    out->partial_bytes = bytes - SPLITK_STATE_BYTES;
    return true;
}

enum { W_CANONICAL = 0, W_STREAM = 1 };  // how the weight argument is laid out

// The linear on validated-or-not arguments; scr = scratch of a K split across workgroups or null.
static int linear_int4_run(const void *a, int a_dtype, float s_x, const uint8_t *Wq, const float *s_w,
                           const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                           const mkq_epilogue *epi, void *workspace, size_t workspace_bytes, void *stream,
                           const SplitKScratch *scr, int forced_cfg, int forced_ks, int w_layout = W_CANONICAL,
                           bool check_only = false)
{
    const bool stream_layout = w_layout == W_STREAM;
    const bool want_q = epi && epi->q_out;
    const bool want_acc = epi && epi->acc_out;
    if (a_dtype != MKQ_I4 && a_dtype != MKQ_F32 && a_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (out_dtype != MKQ_F32 && out_dtype != MKQ_F16 && out_dtype != MKQ_BF16 && out_dtype != MKQ_I4)
        return MKQ_ERR_DTYPE;
    if (epi) {
        if (epi->act != MKQ_ACT_NONE && epi->act != MKQ_ACT_GELU) return MKQ_ERR_DTYPE;
        if (epi->residual && epi->residual_dtype != MKQ_F32 && epi->residual_dtype != MKQ_F16)
            return MKQ_ERR_DTYPE;
    }
    const bool writes_codes = (out && out_dtype == MKQ_I4) || want_q;
    if (M < 0 || N <= 0 || K <= 0 || (K % 32) != 0) return MKQ_ERR_SHAPE;
    if (writes_codes && (N % 2) != 0) return MKQ_ERR_SHAPE;
    const int64_t q_pitch = epi ? epi->q_pitch : 0;
    if (q_pitch != 0 && (q_pitch < N || (q_pitch % 8) != 0 || q_pitch > 0x7FFFFFFF || (q_pitch != N && (N % 8) != 0)))
        return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (writes_codes && !scale_ok(epi ? epi->s_next : 0.0f)) return MKQ_ERR_SCALE;
    if (M == 0) return MKQ_OK;  // empty batch: pointers may be NULL
    if (!a || !Wq || !s_w) return MKQ_ERR_NULL;
    if (!out && !want_q && !want_acc) return MKQ_ERR_NULL;
    if (!aligned16(a) || !aligned16(Wq) || (out && !aligned16(out)) || !aligned16(s_w) ||
        (bias && !aligned16(bias)))
        return MKQ_ERR_ALIGN;
    if (epi && ((epi->residual && !aligned16(epi->residual)) || (epi->q_out && !aligned16(epi->q_out)) ||
                (epi->acc_out && !aligned16(epi->acc_out))))
        return MKQ_ERR_ALIGN;
    const size_t need = mkq_linear_int4_workspace_bytes(M, N, K, a_dtype);
    if (need && (!workspace || workspace_bytes < need || !aligned16(workspace))) return MKQ_ERR_WORKSPACE;
    // the kernel addresses operand bytes with 32-bit offsets
    if (K >= 131072 || M > 0x7FFFFFFF || N > 0x7FFFFFFF || M * (K / 2) > 0xFFFFFFFFLL ||
        N * (K / 2) > 0xFFFFFFFFLL)
        return MKQ_ERR_UNSUPPORTED;
    if (stream_layout && (M > 128 || (K % 256) != 0)) return MKQ_ERR_UNSUPPORTED;
    if (check_only) return MKQ_OK;

    GemmI4Params p;
    p.A = (a_dtype == MKQ_I4) ? (const uint8_t *)a : (const uint8_t *)workspace;
    p.W = Wq; p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.s_x = s_x; p.s_w = s_w; p.bias = bias;
    p.residual = epi ? epi->residual : nullptr;
    p.residual_dtype = epi ? epi->residual_dtype : MKQ_F32;
    p.act = epi ? epi->act : MKQ_ACT_NONE;
    p.out = out; p.out_dtype = out ? out_dtype : -1;
    p.s_next = epi ? epi->s_next : 1.0f;
    p.q_out = (epi && !(out && out_dtype == MKQ_I4)) ? epi->q_out : nullptr;
    p.acc_out = epi ? epi->acc_out : nullptr;
    p.q_pitch = (int)q_pitch;
    p.acc_shift = 8;
    p.acc_unit = 0.00390625f;
    // the kernel that will run is set up (and a forced configuration that does not apply is refused)
    // before anything is enqueued
    auto run = [&]() {
        return stream_layout ? run_gemm_i4_wstream(p, scr, forced_ks, forced_cfg, as_stream(stream))
                             : run_gemm_i4(p, as_stream(stream), forced_cfg, scr, forced_ks);
    };
    p.setup_only = true;
    int rc = run();
    if (rc != MKQ_OK) return rc;
    p.setup_only = false;
    if (a_dtype != MKQ_I4) {
        rc = mkq_quantize(a, a_dtype, M, K, K, s_x, (uint8_t *)workspace, stream);
        if (rc != MKQ_OK) return rc;
    }
    return run();
}

// scratch area named by the epilogue options, if any
static int epilogue_scratch(const mkq_epilogue *epi, SplitKScratch *scr, bool *have)
{
    *have = false;
    if (epi && epi->splitk_scratch) {
        if (!aligned16(epi->splitk_scratch)) return MKQ_ERR_ALIGN;
        if (epi->splitk_scratch_bytes < mkq_splitk_scratch_bytes()) return MKQ_ERR_WORKSPACE;
        *have = splitk_area(epi->splitk_scratch, epi->splitk_scratch_bytes, scr);
    }
    return MKQ_OK;
}

}  // namespace mkq

namespace mkq {
int setup_gemm_f16();  // gemm_f16.hip
}

// Scratch of the entry point that allocates nothing (mkq_linear_int4_stream_static): ticket counters, then
// room for partial sums.  One copy per GPU, at its own address on each, held until the process ends; zero
// when the code object is loaded, and every call leaves the counters zero again.
static __device__ __align__(256) unsigned char scratch[SPLITK_STATE_BYTES + MKQ_SPLITK_PARTIAL_BYTES];

namespace mkq {
// Device address of `scratch` on the current device.  In host code the array's name is only a handle:
// the address that kernels may use comes from hipGetSymbolAddress, once per device.
static int static_scratch(void **ptr_out)
{
    static std::mutex mu;
    static void *ptr[MAX_DEVICES] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return MKQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *q = nullptr;
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return MKQ_ERR_HIP;
        ptr[dev] = q;
    }
    *ptr_out = ptr[dev];
    return MKQ_OK;
}
}  // namespace mkq

extern "C" int mkq_init(void)
{
    GemmI4Params p = {};
    p.M = p.N = 256; p.K = 1024;
    p.setup_only = true;
    int rc = setup_gemm_i4_stream(p, nullptr);
    // (the configurations that split K across workgroups only look at the scratch area's size here)
    const SplitKScratch any_scratch = {reinterpret_cast<unsigned *>(16), reinterpret_cast<int32_t *>(16), (size_t)1 << 40};
    for (int cfg : {2, 3, 11, 12, 14, 18, 19, 20, 27, 28, 29, 31, 33, 35, 60, 61, 62}) {
        // one pass per epilogue class: the parameter block is made to classify as each in turn
        for (int e = 0; e < 7 && rc == MKQ_OK; ++e) {
            GemmI4Params q = p;
            q.out = &q; q.s_next = 1.0f;
            q.out_dtype = e == 0 ? MKQ_F16 : e == 1 ? MKQ_BF16 : e == 2 ? MKQ_F32 : e == 3 ? MKQ_F16 : MKQ_I4;
            if (e == 3) { q.residual = &q; q.residual_dtype = MKQ_F16; }
            if (e == 4) q.act = MKQ_ACT_GELU;
            if (e == 6) q.acc_out = reinterpret_cast<int32_t *>(&q);
            rc = run_gemm_i4(q, nullptr, cfg, cfg >= 60 ? &any_scratch : nullptr, 0);
            if (cfg < 10) break;  // the register-staged kernel has one epilogue
        }
    }
    for (int cfg : {18, 29, 28, 27}) {  // the four tile shapes of the 8-bit path
        for (int e = 0; e < 6 && rc == MKQ_OK; ++e) {
            GemmI4Params q = p;
            q.out = &q; q.s_next = 1.0f;
            q.out_dtype = e == 0 ? MKQ_F16 : e == 1 ? MKQ_BF16 : e == 2 ? MKQ_F32 : e == 3 ? MKQ_F16 : e == 4 ? MKQ_I8 : MKQ_F32;
            if (e == 3) { q.residual = &q; q.residual_dtype = MKQ_F16; }
            if (e == 4) q.act = MKQ_ACT_GELU;
            if (e == 5) q.acc_out = reinterpret_cast<int32_t *>(&q);
            rc = run_gemm_i8(q, nullptr, cfg);
        }
    }
    for (int cfg : {41, 42}) {
        for (int e = 0; e < 4 && rc == MKQ_OK; ++e) {
            GemmI4Params q = p;
            q.out = &q;
            q.out_dtype = e == 0 ? MKQ_F16 : e == 1 ? MKQ_BF16 : MKQ_F32;
            if (e == 3) q.acc_out = reinterpret_cast<int32_t *>(&q);
            rc = run_gemm_e3m2(q, nullptr, cfg);
        }
    }
    if (rc == MKQ_OK) rc = setup_gemm_f16();
    void *scratch_ptr = nullptr;
    if (rc == MKQ_OK) rc = static_scratch(&scratch_ptr);
    return rc;
}

extern "C" int mkq_splitk_scratch_init(void *scratch, size_t scratch_bytes, void *stream)
{
    if (!scratch) return MKQ_ERR_NULL;
    if (!aligned16(scratch)) return MKQ_ERR_ALIGN;
    if (scratch_bytes < mkq_splitk_scratch_bytes()) return MKQ_ERR_WORKSPACE;
    clear_words_kernel<<<SPLITK_MAX_TILES / 256, 256, 0, as_stream(stream)>>>((unsigned *)scratch, SPLITK_MAX_TILES);
    return launch_status();
}

extern "C" int mkq_linear_int4(const void *a, int a_dtype, float s_x, const uint8_t *Wq,
                               const float *s_w, const float *bias, int64_t M, int64_t N, int64_t K,
                               void *out, int out_dtype, const mkq_epilogue *epi, void *workspace,
                               size_t workspace_bytes, void *stream)
{
    SplitKScratch scr;
    bool have = false;
    const int rc = epilogue_scratch(epi, &scr, &have);
    if (rc != MKQ_OK) return rc;
    return linear_int4_run(a, a_dtype, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, workspace, workspace_bytes,
                           stream, have ? &scr : nullptr, -1, 0);
}

extern "C" int mkq_linear_int4_stream(const void *a, int a_dtype, float s_x, const uint8_t *Wq_stream,
                                      const float *s_w, const float *bias, int64_t M, int64_t N, int64_t K,
                                      void *out, int out_dtype, const mkq_epilogue *epi, void *workspace,
                                      size_t workspace_bytes, void *stream)
{
    SplitKScratch scr;
    bool have = false;
    const int rc = epilogue_scratch(epi, &scr, &have);
    if (rc != MKQ_OK) return rc;
    return linear_int4_run(a, a_dtype, s_x, Wq_stream, s_w, bias, M, N, K, out, out_dtype, epi, workspace,
                           workspace_bytes, stream, have ? &scr : nullptr, 0, 0, W_STREAM);
}

extern "C" int mkq_linear_int4_stream_static(const uint8_t *a, float s_x, const uint8_t *Wq_stream, const float *s_w,
                                             const float *bias, int64_t M, int64_t N, int64_t K, void *out,
                                             int out_dtype, const mkq_epilogue *epi, void *stream)
{
    // argument errors first, as everywhere; then the limits of the static area; only then the device
    int rc = linear_int4_run(a, MKQ_I4, s_x, Wq_stream, s_w, bias, M, N, K, out, out_dtype, epi, nullptr, 0, stream,
                             nullptr, 0, 0, W_STREAM, true);
    if (rc != MKQ_OK || M == 0) return rc;
    // the K split that mkq_linear_int4_stream would choose with room to spare must fit the static area
    GemmI4Params shape = {};
    shape.M = (int)M; shape.N = (int)N; shape.K = (int)K;
    SplitKScratch unbounded = {reinterpret_cast<unsigned *>(16), reinterpret_cast<int32_t *>(16), (size_t)1 << 60};
    const int tb = M <= 32 ? 1 : (M <= 64 ? 2 : 4);
    const int64_t tiles_n = ceil_div(N, 128);
    if (tiles_n > SPLITK_MAX_TILES) return MKQ_ERR_UNSUPPORTED;
    const int64_t ks = gemm_i4_stream_slices(shape, &unbounded, 0);
    if (ks > 1 && ks * tiles_n * 4 * tb * 4096 > (int64_t)MKQ_SPLITK_PARTIAL_BYTES) return MKQ_ERR_UNSUPPORTED;
    void *area = nullptr;
    rc = static_scratch(&area);
    if (rc != MKQ_OK) return rc;
    SplitKScratch scr;
    if (!splitk_area(area, SPLITK_STATE_BYTES + MKQ_SPLITK_PARTIAL_BYTES, &scr)) return MKQ_ERR_HIP;
    return linear_int4_run(a, MKQ_I4, s_x, Wq_stream, s_w, bias, M, N, K, out, out_dtype, epi, nullptr, 0, stream, &scr,
                           0, 0, W_STREAM);
}

extern "C" int mkq_tuning_linear_int4(const void *a, int a_dtype, float s_x, const uint8_t *Wq, const float *s_w,
                                      const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                                      const mkq_epilogue *epi, void *workspace, size_t workspace_bytes, void *stream,
                                      int config, int k_slices)
{
    SplitKScratch scr;
    bool have = false;
    const int rc = epilogue_scratch(epi, &scr, &have);
    if (rc != MKQ_OK) return rc;
    return linear_int4_run(a, a_dtype, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, workspace, workspace_bytes,
                           stream, have ? &scr : nullptr, config, k_slices);
}

extern "C" int mkq_tuning_linear_int4_stream(const void *a, int a_dtype, float s_x, const uint8_t *Wq_stream,
                                             const float *s_w, const float *bias, int64_t M, int64_t N, int64_t K,
                                             void *out, int out_dtype, const mkq_epilogue *epi, void *workspace,
                                             size_t workspace_bytes, void *stream, int prefetch_stages, int k_slices)
{
    if (prefetch_stages != 0 && prefetch_stages != 2 && prefetch_stages != 3 && prefetch_stages != 4 &&
        prefetch_stages != 6)
        return MKQ_ERR_UNSUPPORTED;
    SplitKScratch scr;
    bool have = false;
    const int rc = epilogue_scratch(epi, &scr, &have);
    if (rc != MKQ_OK) return rc;
    return linear_int4_run(a, a_dtype, s_x, Wq_stream, s_w, bias, M, N, K, out, out_dtype, epi, workspace,
                           workspace_bytes, stream, have ? &scr : nullptr, prefetch_stages, k_slices, W_STREAM);
}

static int linear_int8_run(const int8_t *a, float s_x, const int8_t *Wq, const float *s_w, const float *bias,
                           int64_t M, int64_t N, int64_t K, void *out, int out_dtype, const mkq_epilogue *epi,
                           void *stream, int forced_cfg)
{
    const bool want_acc = epi && epi->acc_out;
    if (out_dtype == MKQ_I4 || (epi && epi->q_out)) return MKQ_ERR_UNSUPPORTED;
    if (out_dtype != MKQ_F32 && out_dtype != MKQ_F16 && out_dtype != MKQ_BF16 && out_dtype != MKQ_I8)
        return MKQ_ERR_DTYPE;
    if (epi) {
        if (epi->act != MKQ_ACT_NONE && epi->act != MKQ_ACT_GELU) return MKQ_ERR_DTYPE;
        if (epi->residual && epi->residual_dtype != MKQ_F32 && epi->residual_dtype != MKQ_F16)
            return MKQ_ERR_DTYPE;
    }
    if (M < 0 || N <= 0 || K <= 0 || (K % 64) != 0) return MKQ_ERR_SHAPE;
    const int64_t q_pitch = epi ? epi->q_pitch : 0;
    if (q_pitch != 0 && (q_pitch < N || (q_pitch % 8) != 0 || q_pitch > 0x7FFFFFFF || (q_pitch != N && (N % 8) != 0)))
        return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (out && out_dtype == MKQ_I8 && !scale_ok(epi ? epi->s_next : 0.0f)) return MKQ_ERR_SCALE;
    if (M == 0) return MKQ_OK;
    if (!a || !Wq || !s_w) return MKQ_ERR_NULL;
    if (!out && !want_acc) return MKQ_ERR_NULL;
    if (!aligned16(a) || !aligned16(Wq) || (out && !aligned16(out)) || !aligned16(s_w) ||
        (bias && !aligned16(bias)))
        return MKQ_ERR_ALIGN;
    if (epi && ((epi->residual && !aligned16(epi->residual)) || (epi->acc_out && !aligned16(epi->acc_out))))
        return MKQ_ERR_ALIGN;
    // 32-bit byte offsets into the operands
    if (K >= 65536 || M > 0x7FFFFFFF || N > 0x7FFFFFFF || M * K > 0xFFFFFFFFLL || N * K > 0xFFFFFFFFLL)
        return MKQ_ERR_UNSUPPORTED;

    GemmI4Params p;
    p.A = (const uint8_t *)a; p.W = (const uint8_t *)Wq; p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.s_x = s_x; p.s_w = s_w; p.bias = bias;
    p.residual = epi ? epi->residual : nullptr;
    p.residual_dtype = epi ? epi->residual_dtype : MKQ_F32;
    p.act = epi ? epi->act : MKQ_ACT_NONE;
    p.out = out; p.out_dtype = out ? out_dtype : -1;
    p.s_next = (epi && out_dtype == MKQ_I8) ? epi->s_next : 1.0f;
    p.q_out = nullptr;
    p.acc_out = epi ? epi->acc_out : nullptr;
    p.q_pitch = (int)q_pitch;
    p.acc_shift = 0;   // byte operands enter the MFMA as they are
    p.acc_unit = 1.0f;
    return run_gemm_i8(p, as_stream(stream), forced_cfg);
}

extern "C" int mkq_linear_int8(const int8_t *a, float s_x, const int8_t *Wq, const float *s_w,
                               const float *bias, int64_t M, int64_t N, int64_t K, void *out,
                               int out_dtype, const mkq_epilogue *epi, void *stream)
{
    return linear_int8_run(a, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, stream, -1);
}

extern "C" int mkq_tuning_linear_int8(const int8_t *a, float s_x, const int8_t *Wq, const float *s_w,
                                      const float *bias, int64_t M, int64_t N, int64_t K, void *out,
                                      int out_dtype, const mkq_epilogue *epi, void *stream, int config)
{
    if (config != -1 && config != 18 && config != 27 && config != 28 && config != 29 && config != 30)
        return MKQ_ERR_UNSUPPORTED;
    return linear_int8_run(a, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, stream, config);
}

static int linear_int4_e3m2_run(const uint8_t *a, float s_x, const uint8_t *Wq, const float *s_w,
                                const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                                const mkq_epilogue *epi, void *stream, int forced_cfg)
{
    const bool want_q = epi && epi->q_out;
    const bool want_acc = epi && epi->acc_out;
    if (out_dtype != MKQ_F32 && out_dtype != MKQ_F16 && out_dtype != MKQ_BF16 && out_dtype != MKQ_I4)
        return MKQ_ERR_DTYPE;
    if (epi) {
        if (epi->act != MKQ_ACT_NONE && epi->act != MKQ_ACT_GELU) return MKQ_ERR_DTYPE;
        if (epi->residual && epi->residual_dtype != MKQ_F32 && epi->residual_dtype != MKQ_F16)
            return MKQ_ERR_DTYPE;
    }
    const bool writes_codes = (out && out_dtype == MKQ_I4) || want_q;
    if (M < 0 || N <= 0 || K <= 0 || (K % 128) != 0) return MKQ_ERR_SHAPE;
    if (writes_codes && (N % 2) != 0) return MKQ_ERR_SHAPE;
    const int64_t q_pitch = epi ? epi->q_pitch : 0;
    if (q_pitch != 0 && (q_pitch < N || (q_pitch % 8) != 0 || q_pitch > 0x7FFFFFFF || (q_pitch != N && (N % 8) != 0)))
        return MKQ_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_ERR_SCALE;
    if (writes_codes && !scale_ok(epi ? epi->s_next : 0.0f)) return MKQ_ERR_SCALE;
    if (M == 0) return MKQ_OK;
    if (!a || !Wq || !s_w) return MKQ_ERR_NULL;
    if (!out && !want_q && !want_acc) return MKQ_ERR_NULL;
    if (!aligned16(a) || !aligned16(Wq) || (out && !aligned16(out)) || !aligned16(s_w) || (bias && !aligned16(bias)))
        return MKQ_ERR_ALIGN;
    if (epi && ((epi->residual && !aligned16(epi->residual)) || (epi->q_out && !aligned16(epi->q_out)) ||
                (epi->acc_out && !aligned16(epi->acc_out))))
        return MKQ_ERR_ALIGN;
    // exact sums need |acc| <= 64 K < 2^24; 32-bit byte offsets
    if (K >= 262144 || M > 0x7FFFFFFF || N > 0x7FFFFFFF || M * (K / 4 * 3) > 0xFFFFFFFFLL ||
        N * (K / 4 * 3) > 0xFFFFFFFFLL)
        return MKQ_ERR_UNSUPPORTED;
    GemmI4Params p;
    p.A = a; p.W = Wq; p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.s_x = s_x; p.s_w = s_w; p.bias = bias;
    p.residual = epi ? epi->residual : nullptr;
    p.residual_dtype = epi ? epi->residual_dtype : MKQ_F32;
    p.act = epi ? epi->act : MKQ_ACT_NONE;
    p.out = out; p.out_dtype = out ? out_dtype : -1;
    p.s_next = epi ? epi->s_next : 1.0f;
    p.q_out = (epi && !(out && out_dtype == MKQ_I4)) ? epi->q_out : nullptr;
    p.acc_out = epi ? epi->acc_out : nullptr;
    p.q_pitch = (int)q_pitch;
    p.acc_shift = 0;
    p.acc_unit = 1.0f;
    return run_gemm_e3m2(p, as_stream(stream), forced_cfg);
}

extern "C" int mkq_linear_int4_e3m2(const uint8_t *a, float s_x, const uint8_t *Wq, const float *s_w,
                                    const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                                    const mkq_epilogue *epi, void *stream)
{
    return linear_int4_e3m2_run(a, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, stream, -1);
}

extern "C" int mkq_tuning_linear_int4_e3m2(const uint8_t *a, float s_x, const uint8_t *Wq, const float *s_w,
                                           const float *bias, int64_t M, int64_t N, int64_t K, void *out,
                                           int out_dtype, const mkq_epilogue *epi, void *stream, int config)
{
    return linear_int4_e3m2_run(a, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, stream, config);
}
