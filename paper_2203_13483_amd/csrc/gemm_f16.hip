// Binary16 GEMM  y = a W^T + b  (binary32 accumulate) with the same epilogue options
// as the quantized linear: the 16-bit float baseline that the W4A4 layer is timed
// against.  Same skeleton as the int4 kernel: persistent workgroups, a ring of LDS
// stages filled by direct global->LDS copies, XOR-swizzled 16-byte chunks,
// v_mfma_f32_32x32x16_f16 with W as the "A" operand (rows read in permuted order so
// that a lane owns runs of 8 consecutive output channels of one token), fragments
// of the next k step fetched from LDS while the current one is in the matrix core.
#include "gemm_common.h"

namespace mkq {

struct GemmF16Params {
    const uint8_t *A;  // [M, K] binary16
    const uint8_t *W;  // [N, K] binary16
    int M, N, K;
    const float *bias;        // [N] or null
    const uint16_t *residual; // [M, N] binary16 or null
    int act;
    void *out;
    int out_dtype;  // MKQ_F32 or MKQ_F16
};

template <int BM_, int BN_, int WGM_, int WGN_, int S_>
struct GemmF16Cfg {
    static constexpr int BM = BM_, BN = BN_, WGM = WGM_, WGN = WGN_, S = S_;
    static constexpr int RB = 128;  // bytes per row per stage = 64 elements of k
    static constexpr int CH = RB / 16;
    static constexpr int KSTEPS = RB / 32;  // MFMA k steps (16 elements) per stage
    static constexpr int WAVES = WGM * WGN, THREADS = WAVES * 64;
    static constexpr int WTM = BM / WGM, WTN = BN / WGN, TM = WTM / 32, TN = WTN / 32;
    static constexpr int STAGE_BYTES = (BM + BN) * RB;
    static constexpr int ROWS_PER_COPY = 1024 / RB;
    static constexpr int LPW = STAGE_BYTES / 1024 / WAVES;
    static constexpr int LDS_BYTES = S * STAGE_BYTES;
    static_assert((STAGE_BYTES / 1024) % WAVES == 0 && BM % ROWS_PER_COPY == 0, "copy split");
    static_assert(S >= 3 && (S - 2) * LPW <= 63 && LDS_BYTES <= 160 * 1024, "ring limits");
};

// KSPLIT = 2: two groups of Cfg::WAVES waves, each with a ring of its own over one half of K;
// the second group's partial sums are added to the first group's through LDS before the
// epilogue (for launches with few tiles, whose lone wave per SIMD is bound by its own
// instruction stream).
template <class Cfg, int KSPLIT>
__global__ __launch_bounds__(Cfg::THREADS * KSPLIT) void gemm_f16_kernel(const GemmF16Params p)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, RB = Cfg::RB, CH = Cfg::CH;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, S = Cfg::S, LPW = Cfg::LPW, KSTEPS = Cfg::KSTEPS;
    static_assert(KSPLIT == 1 || (KSPLIT == 2 && TM * TN == 1), "the K split is built for 32x32 per wave");

    extern __shared__ __attribute__((aligned(16))) uint8_t smem_all[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave_all / Cfg::WAVES, wave = wave_all % Cfg::WAVES;
    uint8_t *const smem = smem_all + grp * Cfg::LDS_BYTES;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)smem;
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
    const int fr = lane & 31, fh = lane >> 5;

    const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
    const int total_tiles = tiles_m * tiles_n;
    const int row_bytes = p.K * 2;
    const int kt_count = row_bytes / RB / KSPLIT;
    const int k_first = grp * kt_count * RB;
    const int my_tiles = (total_tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
    const int steps = my_tiles * kt_count;

    uint32_t goff[LPW];
    const int c_row = lane / CH, c_slot = lane % CH;
    auto set_tile = [&](int tile) {
        int tm, tn;
        tile_coords(tile, tiles_m, tiles_n, tm, tn);
#pragma unroll
        for (int q = 0; q < LPW; ++q) {
            const int row = (wave * LPW + q) * Cfg::ROWS_PER_COPY + c_row;
            const int chunk = c_slot ^ swz<CH>(row & 15);
            int g;
            if (row < BM) {
                g = tm * BM + row;
                g = g < p.M ? g : p.M - 1;
            } else {
                g = tn * BN + (row - BM);
                g = g < p.N ? g : p.N - 1;
            }
            goff[q] = (uint32_t)g * (uint32_t)row_bytes + chunk * 16;
        }
    };
    int lt = blockIdx.x, lk = 0;
    set_tile(lt);
    auto copy_next = [&](int slot) {  // always issues LPW copies (dummy re-fetch past the end)
        const uint32_t dst = lds0 + slot * Cfg::STAGE_BYTES + wave * (LPW * 1024);
        const uint8_t *a_k = p.A + k_first + lk * RB;
        const uint8_t *w_k = p.W + k_first + lk * RB;
#pragma unroll
        for (int q = 0; q < LPW; ++q) {
            const bool is_a = (wave * LPW + q) * Cfg::ROWS_PER_COPY < BM;
            dma_copy16<0>(is_a ? a_k : w_k, goff[q], dst + q * 1024);
        }
        if (++lk == kt_count) {
            lk = 0;
            if (lt + (int)gridDim.x < total_tiles) {
                lt += gridDim.x;
                set_tile(lt);
            }
        }
    };

    v16f acc[TM][TN];
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][t][v] = 0.0f;

    int rowA[TM], rowW[TN], keyA[TM], keyW[TN];
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int row = wm * Cfg::WTM + j * 32 + fr;
        rowA[j] = row * RB;
        keyA[j] = swz<CH>(row & 15);
    }
#pragma unroll
    for (int t = 0; t < TN; ++t) {
        const int row = wn * Cfg::WTN + t * 32 + w_row_perm(fr);
        rowW[t] = (BM + row) * RB;
        keyW[t] = swz<CH>(row & 15);
    }

    v8h fragW[2][TN], fragA[2][TM];
    auto read_step = [&](int stage_off, auto ksc, auto bc) {
        constexpr int ks = decltype(ksc)::value, b = decltype(bc)::value;
        const int c = ks * 2 + fh;
#pragma unroll
        for (int t = 0; t < TN; ++t)
            fragW[b][t] = *reinterpret_cast<const v8h *>(smem + stage_off + rowW[t] + ((c ^ keyW[t]) * 16));
#pragma unroll
        for (int j = 0; j < TM; ++j)
            fragA[b][j] = *reinterpret_cast<const v8h *>(smem + stage_off + rowA[j] + ((c ^ keyA[j]) * 16));
    };
    auto mfma_step = [&](auto bc) {
        constexpr int b = decltype(bc)::value;
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int t = 0; t < TN; ++t)
                acc[j][t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fragW[b][t], fragA[b][j], acc[j][t], 0, 0, 0);
    };

    // epilogue of one tile
    auto epilogue = [&](int tile) {
        int tile_m, tile_n;
        tile_coords(tile, tiles_m, tiles_n, tile_m, tile_n);
        const int m0 = tile_m * BM, n0 = tile_n * BN;
        const bool vec_ok = (p.N % 8) == 0;
        static_for<TN>([&](auto tc) {
            constexpr int t = decltype(tc)::value;
            static_for<2>([&](auto Gc) {
                constexpr int G = decltype(Gc)::value;
                const int nb = n0 + wn * Cfg::WTN + t * 32 + 16 * G + 8 * fh;
                if (nb >= p.N) return;
                const int nvalid = (p.N - nb) < 8 ? (p.N - nb) : 8;
                float bi[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) bi[e] = (p.bias && e < nvalid) ? p.bias[nb + e] : 0.0f;
                static_for<TM>([&](auto jc) {
                    constexpr int j = decltype(jc)::value;
                    const int m = m0 + wm * Cfg::WTM + j * 32 + fr;
                    if (m >= p.M) return;
                    const int64_t o = (int64_t)m * p.N + nb;
                    float y[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = acc[j][t][8 * G + e] + bi[e];
                    if (p.residual) {
                        const uint16_t *r = p.residual + o;
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
                    } else {
                        uint16_t *dst = (uint16_t *)p.out + o;
                        if (vec_ok) {
                            *reinterpret_cast<uint4 *>(dst) = make_uint4(pack2_f16(y[0], y[1]), pack2_f16(y[2], y[3]),
                                                                         pack2_f16(y[4], y[5]), pack2_f16(y[6], y[7]));
                        } else {
                            for (int e = 0; e < nvalid; ++e) dst[e] = float_to_half_bits(y[e]);
                        }
                    }
                });
            });
        });
    };

    // prologue
#pragma unroll
    for (int i = 0; i < S - 1; ++i) copy_next(i);
    wait_vmcnt<(S - 2) * LPW>();
    lds_barrier();
    read_step(0, IntC<0>{}, IntC<0>{});

    int ct = blockIdx.x, ck = 0, buf = 0;
    static_assert(KSTEPS == 4, "the loop body below is written for four k steps per stage");
    for (int s = 0; s < steps; ++s) {
        const int stage_off = buf * Cfg::STAGE_BYTES;
        const int nbuf = (buf + 1 == S) ? 0 : buf + 1;
        read_step(stage_off, IntC<1>{}, IntC<1>{});
        mfma_step(IntC<0>{});
        read_step(stage_off, IntC<2>{}, IntC<0>{});
        mfma_step(IntC<1>{});
        read_step(stage_off, IntC<3>{}, IntC<1>{});
        mfma_step(IntC<0>{});
        // stage s+1 readable; slot of stage s-1 refilled with stage s+S-1
        wait_vmcnt<(S - 3) * LPW>();
        lds_barrier();
        copy_next(buf == 0 ? S - 1 : buf - 1);
        read_step(nbuf * Cfg::STAGE_BYTES, IntC<0>{}, IntC<0>{});
        mfma_step(IntC<1>{});
        buf = nbuf;
        if (++ck == kt_count) {
            if constexpr (KSPLIT == 2) {
                float *const xch = reinterpret_cast<float *>(smem_all + KSPLIT * Cfg::LDS_BYTES) + wave * 1024 + lane * 4;
                if (grp == 1) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        *reinterpret_cast<float4 *>(xch + q * 256) = make_float4(acc[0][0][4 * q], acc[0][0][4 * q + 1],
                                                                                 acc[0][0][4 * q + 2], acc[0][0][4 * q + 3]);
                }
                lds_barrier();
                if (grp == 0) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 t = *reinterpret_cast<const float4 *>(xch + q * 256);
                        acc[0][0][4 * q] += t.x; acc[0][0][4 * q + 1] += t.y;
                        acc[0][0][4 * q + 2] += t.z; acc[0][0][4 * q + 3] += t.w;
                    }
                }
            }
            if (grp == 0) epilogue(ct);
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int t = 0; t < TN; ++t)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[j][t][v] = 0.0f;
            ck = 0;
            ct += gridDim.x;
        }
    }
    wait_vmcnt<0>();
}

template <class Cfg, int KSPLIT = 1>
static int launch_gemm_f16(const GemmF16Params &p, hipStream_t st, bool setup_only = false)
{
    const int64_t tiles = ceil_div(p.M, Cfg::BM) * ceil_div(p.N, Cfg::BN);
    if (tiles > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    constexpr size_t lds = KSPLIT * Cfg::LDS_BYTES + (KSPLIT - 1) * Cfg::WAVES * 4096;
    static_assert(lds <= 160 * 1024, "LDS is 160 KiB per CU");
    static PerDeviceOnce once;  // per instantiation
    int64_t resident = 0;
    const int rc = resident_workgroups(once, gemm_f16_kernel<Cfg, KSPLIT>, Cfg::THREADS * KSPLIT, lds, 1 << 20, &resident);
    if (rc != MKQ_OK || setup_only) return rc;
    const unsigned grid = (unsigned)(tiles < resident ? tiles : resident);
    gemm_f16_kernel<Cfg, KSPLIT><<<grid, Cfg::THREADS * KSPLIT, lds, st>>>(p);
    return launch_status();
}

int run_gemm_f16(const GemmF16Params &p, hipStream_t st)
{
    const int64_t t128 = ceil_div(p.M, 128) * ceil_div(p.N, 128);
    const int64_t t64 = ceil_div(p.M, 64) * ceil_div(p.N, 64);
    if (t128 >= 192) return launch_gemm_f16<GemmF16Cfg<128, 128, 2, 2, 4>>(p, st);
    // few tiles: 64x64; while there is at most one workgroup per CU the k loop is split between two
    // wave groups (four-stage rings), beyond that a three-stage ring lets three workgroups share a CU
    if (t64 <= 256 && (p.K % 128) == 0 && p.K >= 256) return launch_gemm_f16<GemmF16Cfg<64, 64, 2, 2, 4>, 2>(p, st);
    return launch_gemm_f16<GemmF16Cfg<64, 64, 2, 2, 3>>(p, st);
}

// once-per-device setup of every instantiation (nothing is launched)
int setup_gemm_f16()
{
    GemmF16Params p = {};
    p.M = p.N = p.K = 256;
    int rc = launch_gemm_f16<GemmF16Cfg<128, 128, 2, 2, 4>>(p, nullptr, true);
    if (rc == MKQ_OK) rc = launch_gemm_f16<GemmF16Cfg<64, 64, 2, 2, 4>, 2>(p, nullptr, true);
    if (rc == MKQ_OK) rc = launch_gemm_f16<GemmF16Cfg<64, 64, 2, 2, 3>>(p, nullptr, true);
    return rc;
}

}  // namespace mkq

using namespace mkq;

extern "C" int mkq_linear_fp16(const void *a, const void *W, const float *bias, int64_t M, int64_t N,
                               int64_t K, void *out, int out_dtype, int act, const void *residual,
                               void *stream)
{
    if (out_dtype != MKQ_F32 && out_dtype != MKQ_F16) return MKQ_ERR_DTYPE;
    if (act != MKQ_ACT_NONE && act != MKQ_ACT_GELU) return MKQ_ERR_DTYPE;
    if (M < 0 || N <= 0 || K <= 0 || (K % 64) != 0) return MKQ_ERR_SHAPE;
    if (M == 0) return MKQ_OK;
    if (!a || !W || !out) return MKQ_ERR_NULL;
    if (!aligned16(a) || !aligned16(W) || !aligned16(out) || (bias && !aligned16(bias)) ||
        (residual && !aligned16(residual)))
        return MKQ_ERR_ALIGN;
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || M * K * 2 > 0xFFFFFFFFLL || N * K * 2 > 0xFFFFFFFFLL)
        return MKQ_ERR_UNSUPPORTED;
    GemmF16Params p;
    p.A = (const uint8_t *)a; p.W = (const uint8_t *)W;
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    p.bias = bias; p.residual = (const uint16_t *)residual; p.act = act;
    p.out = out; p.out_dtype = out_dtype;
    return run_gemm_f16(p, as_stream(stream));
}
