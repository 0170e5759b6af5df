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
#include "mkq_internal.h"

namespace mkq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

struct GemmI4Params {
    const uint8_t *A;   // [M, K/2]
    const uint8_t *W;   // [N, K/2]
    int M, N, K;
    float s_x;
    const float *s_w;   // [N]
    const float *bias;  // [N] or null
    const void *residual;
    int residual_dtype;
    int act;
    void *out;          // [M,N] float type, or [M,N/2] bytes
    int out_dtype;      // MKQ_F32/F16/BF16/I4, or -1 for none
    float s_next;
    uint8_t *q_out;     // extra packed codes, or null
    int32_t *acc_out;   // raw accumulators, or null
};

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
__device__ __forceinline__ int swz<8>(int r) { return (r & 7) ^ (((r >> 3) & 1) * 7); }

// Widen two packed words (16 codes) to four int8x4 words (values 16*code).
__device__ __forceinline__ v4i widen(uint32_t w0, uint32_t w1)
{
    v4i r;
    r.x = (int)((w0 << 4) & 0xF0F0F0F0u);
    r.y = (int)(w0 & 0xF0F0F0F0u);
    r.z = (int)((w1 << 4) & 0xF0F0F0F0u);
    r.w = (int)(w1 & 0xF0F0F0F0u);
    return r;
}

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

template <int BM_, int BN_, int WGM_, int WGN_, int RB_>
struct GemmI4Cfg {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, RB = RB_;
    static constexpr int THREADS = WGM * WGN * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // per-wave tile (tokens x channels)
    static constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 MFMA tiles per wave
    static constexpr int CH = RB / 16;                    // 16-byte chunks per LDS row
    static constexpr int ROUNDS = RB / 32;                // ds_read_b128 per fragment per stage
    static constexpr int STAGE_BYTES = (BM + BN) * RB;
    static constexpr int A_PER_T = BM * CH / THREADS, W_PER_T = BN * CH / THREADS;
    static_assert((BM * CH) % THREADS == 0 && (BN * CH) % THREADS == 0, "tile/threads mismatch");
    static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be a multiple of 32");
};

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
    int tile_m, tile_n;
    tile_coords(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int row_bytes = p.K / 2;
    const int kt_count = (row_bytes + RB - 1) / RB;

    // --- staging: which 16-byte chunks this thread copies each stage -------------
    uint4 ra[Cfg::A_PER_T], rw[Cfg::W_PER_T];
    const uint8_t *ga[Cfg::A_PER_T];
    const uint8_t *gw[Cfg::W_PER_T];
    int sa[Cfg::A_PER_T], sw[Cfg::W_PER_T];
    const int my_c = (tid % CH) * 16;  // byte offset of this thread's chunk inside a stage row
#pragma unroll
    for (int i = 0; i < Cfg::A_PER_T; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / CH, c = idx % CH;
        int gm = m0 + row;
        gm = gm < p.M ? gm : p.M - 1;  // rows past the edge re-read the last row; never stored
        ga[i] = p.A + (int64_t)gm * row_bytes + c * 16;
        sa[i] = row * RB + ((c ^ swz<CH>(row & 15)) * 16);
    }
#pragma unroll
    for (int i = 0; i < Cfg::W_PER_T; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / CH, c = idx % CH;
        int gn = n0 + row;
        gn = gn < p.N ? gn : p.N - 1;
        gw[i] = p.W + (int64_t)gn * row_bytes + c * 16;
        sw[i] = BM * RB + row * RB + ((c ^ swz<CH>(row & 15)) * 16);
    }

    auto load_stage = [&](int kt) {
        const int kb = kt * RB;
        const bool in = FULL_STAGES || (kb + my_c < row_bytes);
#pragma unroll
        for (int i = 0; i < Cfg::A_PER_T; ++i)
            ra[i] = in ? *reinterpret_cast<const uint4 *>(ga[i] + kb) : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < Cfg::W_PER_T; ++i)
            rw[i] = in ? *reinterpret_cast<const uint4 *>(gw[i] + kb) : make_uint4(0, 0, 0, 0);
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

    // --- main loop: LDS double buffer, registers hold the stage after next --------
    load_stage(0);
    store_stage(0);
    if (kt_count > 1) load_stage(1);
    lds_barrier();

    for (int kt = 0; kt < kt_count; ++kt) {
        const uint8_t *base = smem + (kt & 1) * Cfg::STAGE_BYTES;
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            compute_round(base, r);
            if (r == ROUNDS / 2 - 1) {
                // the other buffer was last read in the previous iteration, before its barrier
                if (kt + 1 < kt_count) store_stage((kt + 1) & 1);
                if (kt + 2 < kt_count) load_stage(kt + 2);
            }
        }
        lds_barrier();
    }

    // --- epilogue ---------------------------------------------------------------
    // Register v of a lane holds channel 16*(v/8) + 8*fh + v%8 of its 32-channel tile,
    // token fr of its 32-token tile.
    const bool vec_ok = (p.N % 8) == 0;
    const bool need_y = (p.out_dtype >= 0) || p.q_out;
    static_for<TN>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        static_for<2>([&](auto Gc) {
            constexpr int G = decltype(Gc)::value;
            const int nb = n0 + wn * Cfg::WTN + t * 32 + 16 * G + 8 * fh;
            if (nb >= p.N) return;
            const int nvalid = (p.N - nb) < 8 ? (p.N - nb) : 8;
            float sc[8], bi[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int n = (e < nvalid) ? nb + e : nb;
                sc[e] = (p.s_x * p.s_w[n]) * 0.00390625f;  // exact: power of two
                bi[e] = p.bias ? p.bias[n] : 0.0f;
            }
            static_for<TM>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                const int m = m0 + wm * Cfg::WTM + j * 32 + fr;
                if (m >= p.M) return;
                const int64_t o = (int64_t)m * p.N + nb;
                int a[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = acc[j][t][8 * G + e];

                if (p.acc_out) {
                    if (vec_ok) {
                        *reinterpret_cast<int4 *>(p.acc_out + o) = make_int4(a[0] >> 8, a[1] >> 8, a[2] >> 8, a[3] >> 8);
                        *reinterpret_cast<int4 *>(p.acc_out + o + 4) = make_int4(a[4] >> 8, a[5] >> 8, a[6] >> 8, a[7] >> 8);
                    } else {
                        for (int e = 0; e < nvalid; ++e) p.acc_out[o + e] = a[e] >> 8;
                    }
                }
                if (!need_y) return;

                float y[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) y[e] = __fmaf_rn((float)a[e], sc[e], bi[e]);
                if (p.residual) {
                    if (p.residual_dtype == MKQ_F32) {
                        const float *r = (const float *)p.residual + o;
                        if (vec_ok) {
                            const float4 r0 = *reinterpret_cast<const float4 *>(r);
                            const float4 r1 = *reinterpret_cast<const float4 *>(r + 4);
                            y[0] += r0.x; y[1] += r0.y; y[2] += r0.z; y[3] += r0.w;
                            y[4] += r1.x; y[5] += r1.y; y[6] += r1.z; y[7] += r1.w;
                        } else {
                            for (int e = 0; e < nvalid; ++e) y[e] += r[e];
                        }
                    } else {
                        const uint16_t *r = (const uint16_t *)p.residual + o;
                        if (vec_ok) {
                            const uint4 rr = *reinterpret_cast<const uint4 *>(r);
                            const uint32_t rwd[4] = {rr.x, rr.y, rr.z, rr.w};
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                y[2 * e] += half_bits_to_float((uint16_t)(rwd[e] & 0xFFFFu));
                                y[2 * e + 1] += half_bits_to_float((uint16_t)(rwd[e] >> 16));
                            }
                        } else {
                            for (int e = 0; e < nvalid; ++e) y[e] += half_bits_to_float(r[e]);
                        }
                    }
                }
                if (p.act == MKQ_ACT_GELU) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = gelu_erf(y[e]);
                }

                if (p.out_dtype == MKQ_F32) {
                    float *dst = (float *)p.out + o;
                    if (vec_ok) {
                        *reinterpret_cast<float4 *>(dst) = make_float4(y[0], y[1], y[2], y[3]);
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(y[4], y[5], y[6], y[7]);
                    } else {
                        for (int e = 0; e < nvalid; ++e) dst[e] = y[e];
                    }
                } else if (p.out_dtype == MKQ_F16 || p.out_dtype == MKQ_BF16) {
                    uint32_t h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t lo = (p.out_dtype == MKQ_F16) ? float_to_half_bits(y[2 * e])
                                                                     : float_to_bf16_bits(y[2 * e]);
                        const uint32_t hi = (p.out_dtype == MKQ_F16) ? float_to_half_bits(y[2 * e + 1])
                                                                     : float_to_bf16_bits(y[2 * e + 1]);
                        h[e] = lo | (hi << 16);
                    }
                    uint16_t *dst = (uint16_t *)p.out + o;
                    if (vec_ok) {
                        *reinterpret_cast<uint4 *>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
                    } else {
                        for (int e = 0; e < nvalid; ++e) dst[e] = (uint16_t)(h[e >> 1] >> (16 * (e & 1)));
                    }
                }
                if (p.out_dtype == MKQ_I4 || p.q_out) {
                    // Eq. 1 on the binary32 value.  N is even and nb % 8 == 0, so o is even.
                    uint32_t packed = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        packed |= ((uint32_t)quantize_code(y[e], p.s_next) & 0xFu) << (4 * e);
                    uint8_t *qdst = (p.out_dtype == MKQ_I4 ? (uint8_t *)p.out : p.q_out) + (o >> 1);
                    if (vec_ok) {
                        *reinterpret_cast<uint32_t *>(qdst) = packed;
                    } else {
                        for (int e = 0; e < nvalid / 2; ++e) qdst[e] = (uint8_t)(packed >> (8 * e));
                    }
                }
            });
        });
    });
}

template <class Cfg, bool FULL>
static int launch_one(const GemmI4Params &p, int64_t tiles, hipStream_t st)
{
    const size_t lds = 2 * (size_t)Cfg::STAGE_BYTES;
    static bool attr_set = false;  // per instantiation
    if (!attr_set && lds > 65536) {
        if (hipFuncSetAttribute((const void *)gemm_i4_kernel<Cfg, FULL>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return MKQ_ERR_HIP;
        attr_set = true;
    }
    gemm_i4_kernel<Cfg, FULL><<<(unsigned)tiles, Cfg::THREADS, lds, st>>>(p);
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

static int g_forced_cfg = -1;  // tuning hook, see mkq_debug_set_gemm_config

int run_gemm_i4(const GemmI4Params &p, hipStream_t st)
{
    int cfg = g_forced_cfg;
    if (cfg < 0) {
        const int64_t t256 = ceil_div(p.M, 256) * ceil_div(p.N, 256);
        const int64_t t128 = ceil_div(p.M, 128) * ceil_div(p.N, 128);
        if (t256 >= 512) cfg = 0;
        else if (t128 >= 256) cfg = 2;
        else cfg = 3;
    }
    switch (cfg) {
    case 0: return launch_gemm_i4<GemmI4Cfg<256, 256, 2, 2, 64>>(p, st);
    case 1: return launch_gemm_i4<GemmI4Cfg<256, 128, 2, 2, 64>>(p, st);
    case 2: return launch_gemm_i4<GemmI4Cfg<128, 128, 2, 2, 64>>(p, st);
    case 3: return launch_gemm_i4<GemmI4Cfg<64, 64, 2, 2, 64>>(p, st);
    case 4: return launch_gemm_i4<GemmI4Cfg<256, 256, 2, 2, 128>>(p, st);
    case 5: return launch_gemm_i4<GemmI4Cfg<256, 128, 2, 2, 128>>(p, st);
    case 6: return launch_gemm_i4<GemmI4Cfg<128, 128, 2, 2, 128>>(p, st);
    default: return MKQ_ERR_UNSUPPORTED;
    }
}

}  // namespace mkq

using namespace mkq;

// Tuning hook (not part of the public header): force one tile configuration of the
// int4 GEMM (-1 = automatic choice).
extern "C" void mkq_debug_set_gemm_config(int cfg) { mkq::g_forced_cfg = cfg; }

extern "C" size_t mkq_linear_int4_workspace_bytes(int64_t M, int64_t N, int64_t K, int a_dtype)
{
    (void)N;
    if (a_dtype == MKQ_I4 || M <= 0 || K <= 0) return 0;
    return ((size_t)M * (size_t)(K / 2) + 255) & ~(size_t)255;
}

extern "C" int mkq_linear_int4(const void *a, int a_dtype, float s_x, const uint8_t *Wq,
                               const float *s_w, const float *bias, int64_t M, int64_t N, int64_t K,
                               void *out, int out_dtype, const mkq_epilogue *epi, void *workspace,
                               size_t workspace_bytes, void *stream)
{
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
    if (K >= 131072 || M > 0x7FFFFFFF || N > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;

    const uint8_t *codes = (const uint8_t *)a;
    if (a_dtype != MKQ_I4) {
        const int rc = mkq_quantize(a, a_dtype, M, K, K, s_x, (uint8_t *)workspace, stream);
        if (rc != MKQ_OK) return rc;
        codes = (const uint8_t *)workspace;
    }

    GemmI4Params p;
    p.A = codes; p.W = Wq; p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.s_x = s_x; p.s_w = s_w; p.bias = bias;
    p.residual = epi ? epi->residual : nullptr;
    p.residual_dtype = epi ? epi->residual_dtype : MKQ_F32;
    p.act = epi ? epi->act : MKQ_ACT_NONE;
    p.out = out; p.out_dtype = out ? out_dtype : -1;
    p.s_next = epi ? epi->s_next : 1.0f;
    p.q_out = (epi && !(out && out_dtype == MKQ_I4)) ? epi->q_out : nullptr;
    p.acc_out = epi ? epi->acc_out : nullptr;
    return run_gemm_i4(p, as_stream(stream));
}
