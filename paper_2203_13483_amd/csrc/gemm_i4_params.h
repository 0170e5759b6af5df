// Parameter block, nibble widening and the generic (run-time) epilogue of the int4 GEMM kernels,
// shared by the tile kernels and the few-token streaming kernel.
#pragma once

#include "gemm_common.h"

namespace mkq {

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
    int q_pitch = 0;    // codes per row of the code outputs (out of MKQ_I4 / MKQ_I8, q_out); 0 = N
    // What the int32 accumulator holds: 2^acc_shift * sum(a*w).  The 4-bit path feeds the
    // matrix core 16*code on both sides (shift 8); the 8-bit path feeds the codes themselves.
    int acc_shift;
    float acc_unit;     // 2^-acc_shift, folded into the per-channel scale (exact)
    // K split across workgroups of the tile kernels (their XS instantiations): slices per output tile and the
    // caller's scratch area; 1 = no split
    int ks = 1;
    unsigned *sk_counters = nullptr;
    int32_t *sk_partials = nullptr;
    // host side only: do the once-per-device setup of the kernel that would run, launch nothing
    bool setup_only = false;
};

// Scratch of a K split across workgroups, as the host hands it over: `counters` (SPLITK_MAX_TILES
// ticket counters, zero between launches) and room for the slices' partial accumulators.
constexpr int SPLITK_MAX_TILES = 4096;
constexpr size_t MKQ_SPLITK_PARTIAL_BYTES = (size_t)16 << 20;
constexpr size_t SPLITK_STATE_BYTES = SPLITK_MAX_TILES * sizeof(unsigned);
struct SplitKScratch {
    unsigned *counters;
    int32_t *partials;
    size_t partial_bytes;
};
// ... and as a kernel takes it
struct SplitKArgs {
    int ks;  // slices per output tile; 1 = no split, the pointers are unused
    unsigned *counters;
    int32_t *partials;
};

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

// Compile-time description of an epilogue.  The fast kernels are instantiated for the
// few combinations the encoder layer and the benchmarks use, so that the fully
// unrolled per-tile epilogue stays a few KiB of code; EpiGeneric reads every option
// from the parameter block at run time (and also handles N % 8 != 0, the raw
// accumulator output and the extra code output).
template <int OUT, bool RES16, bool GELU>
struct EpiFixed {
    static constexpr bool generic = false;
    static constexpr int out = OUT;
    static constexpr bool res16 = RES16, gelu = GELU;
};
struct EpiGeneric {
    static constexpr bool generic = true;
    static constexpr int out = MKQ_F32;
    static constexpr bool res16 = false, gelu = false;
};

// Epilogue of one finished tile (m0, n0 = its first token / channel; wm, wn = the
// wave's position in the workgroup; fr = lane % 32, fh = lane / 32).
// Register v of a lane holds channel 16*(v/8) + 8*fh + v%8 of its 32-channel tile,
// token fr of its 32-token tile.
template <class Cfg, class Epi>
__device__ __forceinline__ void gemm_i4_epilogue(const GemmI4Params &p, v16i (&acc)[Cfg::TM][Cfg::TN],
                                                 int m0, int n0, int wm, int wn, int fr, int fh)
{
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    const int out_dtype = Epi::generic ? p.out_dtype : Epi::out;
    const bool has_res = Epi::generic ? (p.residual != nullptr) : Epi::res16;
    const bool res_f32 = Epi::generic ? (p.residual_dtype == MKQ_F32) : false;
    const bool gelu = Epi::generic ? (p.act == MKQ_ACT_GELU) : Epi::gelu;
    const bool vec_ok = Epi::generic ? ((p.N % 8) == 0) : true;
    int32_t *const acc_out = Epi::generic ? p.acc_out : nullptr;
    uint8_t *const q_extra = Epi::generic ? p.q_out : nullptr;
    const bool need_y = (out_dtype >= 0) || q_extra;
    static_for<TN>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        static_for<2>([&](auto Gc) {
            constexpr int G = decltype(Gc)::value;
            // keep the scheduler from hoisting every unit's loads to the top (register spills)
            __builtin_amdgcn_sched_barrier(0);
            const int nb = n0 + wn * Cfg::WTN + t * 32 + 16 * G + 8 * fh;
            if (nb >= p.N) return;
            const int nvalid = (p.N - nb) < 8 ? (p.N - nb) : 8;
            float sc[8], bi[8];
            if (vec_ok) {
                const float4 s0 = *reinterpret_cast<const float4 *>(p.s_w + nb);
                const float4 s1 = *reinterpret_cast<const float4 *>(p.s_w + nb + 4);
                sc[0] = s0.x; sc[1] = s0.y; sc[2] = s0.z; sc[3] = s0.w;
                sc[4] = s1.x; sc[5] = s1.y; sc[6] = s1.z; sc[7] = s1.w;
                if (p.bias) {
                    const float4 b0 = *reinterpret_cast<const float4 *>(p.bias + nb);
                    const float4 b1 = *reinterpret_cast<const float4 *>(p.bias + nb + 4);
                    bi[0] = b0.x; bi[1] = b0.y; bi[2] = b0.z; bi[3] = b0.w;
                    bi[4] = b1.x; bi[5] = b1.y; bi[6] = b1.z; bi[7] = b1.w;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) bi[e] = 0.0f;
                }
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int n = (e < nvalid) ? nb + e : nb;
                    sc[e] = p.s_w[n];
                    bi[e] = p.bias ? p.bias[n] : 0.0f;
                }
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sc[e] = (p.s_x * sc[e]) * p.acc_unit;  // power of two: exact
            static_for<TM>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                __builtin_amdgcn_sched_barrier(0);
                const int m = m0 + wm * Cfg::WTM + j * 32 + fr;
                if (m >= p.M) return;
                const int64_t o = (int64_t)m * p.N + nb;
                const int64_t oq = p.q_pitch ? (int64_t)m * p.q_pitch + nb : o;  // in the code outputs
                int a[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e] = acc[j][t][8 * G + e];

                if (acc_out) {
                    if (vec_ok) {
                        *reinterpret_cast<int4 *>(acc_out + o) = make_int4(a[0] >> p.acc_shift, a[1] >> p.acc_shift, a[2] >> p.acc_shift, a[3] >> p.acc_shift);
                        *reinterpret_cast<int4 *>(acc_out + o + 4) = make_int4(a[4] >> p.acc_shift, a[5] >> p.acc_shift, a[6] >> p.acc_shift, a[7] >> p.acc_shift);
                    } else {
                        for (int e = 0; e < nvalid; ++e) acc_out[o + e] = a[e] >> p.acc_shift;
                    }
                }
                if (!need_y) return;

                float y[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    y[e] = __fmaf_rn((float)a[e], sc[e], bi[e]);
                    // keep the binary32 rounding: without this the compiler folds the fma and a
                    // later narrowing into one v_fma_mixlo_f16, which rounds only once
                    asm volatile("" : "+v"(y[e]));
                }
                if (has_res) {
                    if (res_f32) {
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
                if (gelu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = gelu_erf(y[e]);
                }

                if (out_dtype == MKQ_F32) {
                    float *dst = (float *)p.out + o;
                    if (vec_ok) {
                        *reinterpret_cast<float4 *>(dst) = make_float4(y[0], y[1], y[2], y[3]);
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(y[4], y[5], y[6], y[7]);
                    } else {
                        for (int e = 0; e < nvalid; ++e) dst[e] = y[e];
                    }
                } else if (out_dtype == MKQ_F16 || out_dtype == MKQ_BF16) {
                    uint32_t h[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        h[e] = (out_dtype == MKQ_F16) ? pack2_f16(y[2 * e], y[2 * e + 1])
                                                      : pack2_bf16(y[2 * e], y[2 * e + 1]);
                    uint16_t *dst = (uint16_t *)p.out + o;
                    if (vec_ok) {
                        *reinterpret_cast<uint4 *>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
                    } else {
                        for (int e = 0; e < nvalid; ++e) dst[e] = (uint16_t)(h[e >> 1] >> (16 * (e & 1)));
                    }
                }
                if (out_dtype == MKQ_I8) {  // Eq. 1 at 8 bits, one byte per code
                    int cd[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) cd[e] = quantize_code8(y[e], p.s_next);
                    uint8_t *qdst = (uint8_t *)p.out + oq;
                    if (vec_ok) {
                        *reinterpret_cast<uint2 *>(qdst) = bytes8(cd);
                        if (p.q_pitch > p.N && nb + 8 == p.N)
                            for (int c = 8; c < p.q_pitch - nb; c += 8) reinterpret_cast<uint2 *>(qdst)[c / 8] = make_uint2(0u, 0u);
                    } else {
                        for (int e = 0; e < nvalid; ++e) qdst[e] = (uint8_t)cd[e];
                    }
                }
                if (out_dtype == MKQ_I4 || q_extra) {
                    // Eq. 1 on the binary32 value.  The pitch is even and nb % 8 == 0, so oq is even.
                    uint32_t packed = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        packed |= ((uint32_t)quantize_code(y[e], p.s_next) & 0xFu) << (4 * e);
                    uint8_t *qdst = (out_dtype == MKQ_I4 ? (uint8_t *)p.out : q_extra) + (oq >> 1);
                    if (vec_ok) {
                        *reinterpret_cast<uint32_t *>(qdst) = packed;
                        // a row with a pitch: the lane that owns the last 8 channels also writes the zero
                        // padding codes N .. pitch - 1 (both multiples of 8)
                        if (p.q_pitch > p.N && nb + 8 == p.N)
                            for (int c = 8; c < p.q_pitch - nb; c += 8) reinterpret_cast<uint32_t *>(qdst)[c / 8] = 0u;
                    } else {
                        for (int e = 0; e < nvalid / 2; ++e) qdst[e] = (uint8_t)(packed >> (8 * e));
                    }
                }
            });
        });
    });
}

// Epilogue of the ring kernel through LDS, for the compile-time epilogues.  In the MFMA
// result layout a lane owns 8 consecutive channels of one token, so a direct store
// instruction writes 32 rows x 32 bytes and every lane needs the scales of its own
// channels for each 8-value unit.  Here a wave instead drops one 32-token x 32-channel
// accumulator tile at a time, as raw int32, into a wave-private LDS area (rows of 128
// bytes, 16-byte pieces XOR-swizzled so that writes and reads are bank-conflict free)
// and reads it back transposed: lane l then owns channels 8*(l%4) .. +7 of rows l/4
// and l/4 + 16, i.e. the same 8 channels for the whole pass, dequantizes (and adds the
// residual, applies GELU, re-quantizes) and stores 16 rows x 64 contiguous bytes per
// instruction (128 for binary32, 16 for codes).  The per-channel scales and biases of
// the wave's WTN channels are copied to LDS (sc_lds, wave-private, beyond the ring)
// while the tile's last k stages run, so the epilogue issues no global loads that
// would have to wait, in order, behind every copy in flight.
// scr: wave-private LDS, 4 KiB, not in use by the ring.
template <class Cfg>
struct EpiShuffle {
    static constexpr int REGION = Cfg::STAGE_BYTES / Cfg::WAVES;   // a wave's share of an idle ring slot
    // per wave, beyond the ring: s_w then bias, each a whole number of 64-lane copies
    static constexpr int NSL = (Cfg::WTN + 63) / 64;
    static constexpr int BIAS_AT = NSL * 64;                       // in floats
    static constexpr int SCALE_BYTES = 2 * BIAS_AT * 4;
    static constexpr int EXTRA_LDS = Cfg::WAVES * SCALE_BYTES;
    static constexpr bool usable = REGION >= 4096 && Cfg::RB == 64 &&
                                   (Cfg::LDS_BYTES + EXTRA_LDS) * Cfg::WGS_PER_CU <= 160 * 1024;
};

template <class Cfg, class Epi>
__device__ __forceinline__ void gemm_i4_epilogue_rows(const GemmI4Params &p, v16i (&acc)[Cfg::TM][Cfg::TN],
                                                      int m0, int n0, int wm, int wn, int lane, uint8_t *scr,
                                                      float *sc_lds)
{
    using Sh = EpiShuffle<Cfg>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, WTN = Cfg::WTN;
    const int fr = lane & 31, fh = lane >> 5;
    const int nw = n0 + wn * WTN;      // first channel of the wave
    const int rrow = lane >> 2;        // reader: rows rrow and rrow + 16
    const int pc = lane & 3;           // reader: channels 8 * pc .. + 7 of the 32-channel tile

    // sc_lds holds s_w then bias of the wave's WTN channels.  Fold s_x and the accumulator's
    // power-of-two unit (exact) into the scales once; no bias -> zeros.
#pragma unroll
    for (int c = lane; c < WTN; c += 64) {
        sc_lds[c] = (p.s_x * sc_lds[c]) * p.acc_unit;
        if (!p.bias) sc_lds[Sh::BIAS_AT + c] = 0.0f;
    }
    QuantStep qs4 = {}, qs8 = {};
    if constexpr (Epi::out == MKQ_I4) qs4 = quant_step<4>(p.s_next);
    if constexpr (Epi::out == MKQ_I8) qs8 = quant_step<8>(p.s_next);
    // writer: the lane's 8 values of unit G are pieces 4G + 2fh, 4G + 2fh + 1 of row fr
    const int wr_base = fr * 128;
    const int wr_key = fr & 7;
    // reader: pieces 2pc, 2pc + 1 of its two rows
    int rd_off[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int r = rrow + 16 * i;
#pragma unroll
        for (int h = 0; h < 2; ++h) rd_off[i][h] = r * 128 + (((2 * pc + h) ^ (r & 7)) * 16);
    }

    // 16-bit residual: the two rows a lane needs of a 32 x 32 unit are fetched RES_AHEAD units before
    // they are used (units in the order they are processed, j fastest), so that their latency is covered
    // by the units in between instead of being waited for in every unit.
    constexpr int RES_AHEAD = 2, UNITS = TN * TM;
    uint4 res_q[RES_AHEAD][2];
    auto fetch_residual = [&](auto uc, uint4(&dst)[2]) {
        constexpr int u = decltype(uc)::value, t = u / TM, j = u % TM;
        const int n = nw + t * 32 + 8 * pc;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int m = m0 + wm * Cfg::WTM + j * 32 + rrow + 16 * i;
            dst[i] = (m < p.M && n < p.N)
                         ? *reinterpret_cast<const uint4 *>((const uint16_t *)p.residual + (int64_t)m * p.N + n)
                         : make_uint4(0, 0, 0, 0);
        }
    };
    if constexpr (Epi::res16) {
        static_for<(RES_AHEAD < UNITS ? RES_AHEAD : UNITS)>([&](auto uc) { fetch_residual(uc, res_q[decltype(uc)::value]); });
    }

    static_for<TN>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        const int c0 = t * 32 + 8 * pc;  // first of the reader lane's channels, wave-relative
        const int n = nw + c0;
        const float4 s0 = *reinterpret_cast<const float4 *>(sc_lds + c0);
        const float4 s1 = *reinterpret_cast<const float4 *>(sc_lds + c0 + 4);
        const float4 b0 = *reinterpret_cast<const float4 *>(sc_lds + Sh::BIAS_AT + c0);
        const float4 b1 = *reinterpret_cast<const float4 *>(sc_lds + Sh::BIAS_AT + c0 + 4);
        const float sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
        const float bi[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
        static_for<TM>([&](auto jc) {
            constexpr int j = decltype(jc)::value;
            __builtin_amdgcn_sched_barrier(0);
            // write the raw tile
#pragma unroll
            for (int G = 0; G < 2; ++G)
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    *reinterpret_cast<int4 *>(scr + wr_base + (((4 * G + 2 * fh + h) ^ wr_key) * 16)) =
                        make_int4(acc[j][t][8 * G + 4 * h], acc[j][t][8 * G + 4 * h + 1],
                                  acc[j][t][8 * G + 4 * h + 2], acc[j][t][8 * G + 4 * h + 3]);
            // read it back row-wise
            int4 raw[2][2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int h = 0; h < 2; ++h) raw[i][h] = *reinterpret_cast<const int4 *>(scr + rd_off[i][h]);
            const int mbase = m0 + wm * Cfg::WTM + j * 32 + rrow;
            uint4 res[2];
            if constexpr (Epi::res16) {
                constexpr int u = t * TM + j;
                res[0] = res_q[u % RES_AHEAD][0];
                res[1] = res_q[u % RES_AHEAD][1];
                if constexpr (u + RES_AHEAD < UNITS) fetch_residual(IntC<u + RES_AHEAD>{}, res_q[u % RES_AHEAD]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int a[8] = {raw[i][0].x, raw[i][0].y, raw[i][0].z, raw[i][0].w,
                                  raw[i][1].x, raw[i][1].y, raw[i][1].z, raw[i][1].w};
                float y[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    y[e] = __fmaf_rn((float)a[e], sc[e], bi[e]);
                    asm volatile("" : "+v"(y[e]));  // keep the binary32 rounding (no fused narrowing)
                }
                if (Epi::res16) {
                    const uint32_t rwd[4] = {res[i].x, res[i].y, res[i].z, res[i].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        y[2 * e] += half_bits_to_float((uint16_t)(rwd[e] & 0xFFFFu));
                        y[2 * e + 1] += half_bits_to_float((uint16_t)(rwd[e] >> 16));
                    }
                }
                if (Epi::gelu) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) y[e] = gelu_erf(y[e]);
                }
                const int m = mbase + 16 * i;
                const bool ok = m < p.M && n < p.N;  // N % 8 == 0: a lane's 8 channels are all in or all out
                const int64_t o = (int64_t)m * p.N + n;
                if (Epi::out == MKQ_F32) {
                    if (ok) {
                        float *dst = (float *)p.out + o;
                        *reinterpret_cast<float4 *>(dst) = make_float4(y[0], y[1], y[2], y[3]);
                        *reinterpret_cast<float4 *>(dst + 4) = make_float4(y[4], y[5], y[6], y[7]);
                    }
                } else if (Epi::out == MKQ_F16 || Epi::out == MKQ_BF16) {
                    uint32_t hw[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        hw[e] = (Epi::out == MKQ_F16) ? pack2_f16(y[2 * e], y[2 * e + 1]) : pack2_bf16(y[2 * e], y[2 * e + 1]);
                    if (ok) *reinterpret_cast<uint4 *>((uint16_t *)p.out + o) = make_uint4(hw[0], hw[1], hw[2], hw[3]);
                } else if (Epi::out == MKQ_I8) {
                    const uint2 pk8 = quantize8<8>(y, qs8);
                    // code rows may have a pitch; the lane that owns a row's last 8 channels writes its zero padding
                    const int pitch = p.q_pitch ? p.q_pitch : p.N;
                    uint2 *dst = reinterpret_cast<uint2 *>((uint8_t *)p.out + (int64_t)m * pitch + n);
                    if (ok) {
                        *dst = pk8;
                        if (n + 8 == p.N)
                            for (int c = 8; c < pitch - n; c += 8) dst[c / 8] = make_uint2(0u, 0u);
                    }
                } else {
                    const uint32_t packed = quantize8<4>(y, qs4).x;  // Eq. 1 on the binary32 values
                    const int pitch = p.q_pitch ? p.q_pitch : p.N;
                    uint32_t *dst = reinterpret_cast<uint32_t *>((uint8_t *)p.out + (((int64_t)m * pitch + n) >> 1));
                    if (ok) {
                        *dst = packed;
                        if (n + 8 == p.N)
                            for (int c = 8; c < pitch - n; c += 8) dst[c / 8] = 0u;
                    }
                }
            }
        });
    });
}

// Row epilogue for 16-bit outputs of waves that own 64 channels (TN = 2); accumulators are int32 or binary32
// holding exact integers.  Values are dequantized and narrowed in the MFMA register layout first, so the
// transposition moves 2 bytes per value instead of 4, and a 32-token block is laid out as rows of 128
// bytes (64 channels): every store instruction then writes 8 whole 128-byte lines.
// scr: wave-private LDS, 4 KiB; sc_lds: s_w then bias of the wave's 64 channels (as for the row epilogue).
template <class Cfg, class Epi>
struct EpiLines16 {
    static constexpr bool usable = !Epi::generic && !Epi::res16 && !Epi::gelu && Cfg::TN == 2 && Cfg::WTN == 64 &&
                                   (Epi::out == MKQ_F16 || Epi::out == MKQ_BF16);
};

template <class Cfg, class Epi, bool CACHE_SCALES = true, class AccV>
__device__ __forceinline__ void gemm_epilogue_lines16(const GemmI4Params &p, AccV (&acc)[Cfg::TM][Cfg::TN],
                                                      int m0, int n0, int wm, int wn, int lane, uint8_t *scr,
                                                      float *sc_lds)
{
    using Sh = EpiShuffle<Cfg>;
    constexpr int TM = Cfg::TM, TN = Cfg::TN;
    static_assert(EpiLines16<Cfg, Epi>::usable, "64 channels per wave, plain 16-bit outputs");
    const int fr = lane & 31, fh = lane >> 5;
    sc_lds[lane] = (p.s_x * sc_lds[lane]) * p.acc_unit;
    if (!p.bias) sc_lds[Sh::BIAS_AT + lane] = 0.0f;

    // the lane's 32 channels: register 8h + e of tile t is channel 32t + 16h + 8fh + e.  Their scales and
    // biases are either held in 64 registers for the whole tile or fetched again for every 8 values.
    auto load8 = [&](int t, int h, float (&s8)[8], float (&b8)[8]) {
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int c = 32 * t + 16 * h + 8 * fh + 4 * q;
            const float4 s4 = *reinterpret_cast<const float4 *>(sc_lds + c);
            const float4 b4 = *reinterpret_cast<const float4 *>(sc_lds + Sh::BIAS_AT + c);
            s8[4 * q] = s4.x; s8[4 * q + 1] = s4.y; s8[4 * q + 2] = s4.z; s8[4 * q + 3] = s4.w;
            b8[4 * q] = b4.x; b8[4 * q + 1] = b4.y; b8[4 * q + 2] = b4.z; b8[4 * q + 3] = b4.w;
        }
    };
    float sc[CACHE_SCALES ? TN * 2 : 1][8], bi[CACHE_SCALES ? TN * 2 : 1][8];
    if constexpr (CACHE_SCALES) {
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) load8(t, h, sc[2 * t + h], bi[2 * t + h]);
    }
    // writer: 16-byte piece 4t + 2h + fh of row fr; pieces are XOR-swizzled with bits 1 .. 3 of the row so
    // that 16 consecutive rows spread one piece column over all banks.  reader: row lane / 8 + 8i, piece lane % 8.
    const int wr_base = fr * 128, wr_key = (fr >> 1) & 7;
    const int rrow = lane >> 3, rq = lane & 7;
    const int n = n0 + wn * 64 + 8 * rq;
    static_for<TM>([&](auto jc) {
        constexpr int j = decltype(jc)::value;
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < TN; ++t)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                uint32_t hw[4];
                constexpr int u = CACHE_SCALES ? 1 : 0;
                if constexpr (!CACHE_SCALES) load8(t, h, sc[0], bi[0]);
                const float(&s8)[8] = sc[u * (2 * t + h)];
                const float(&b8)[8] = bi[u * (2 * t + h)];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float y0 = __fmaf_rn((float)acc[j][t][8 * h + 2 * e], s8[2 * e], b8[2 * e]);
                    float y1 = __fmaf_rn((float)acc[j][t][8 * h + 2 * e + 1], s8[2 * e + 1], b8[2 * e + 1]);
                    asm volatile("" : "+v"(y0), "+v"(y1));  // keep the binary32 rounding (no fused narrowing)
                    hw[e] = (Epi::out == MKQ_F16) ? pack2_f16(y0, y1) : pack2_bf16(y0, y1);
                }
                *reinterpret_cast<uint4 *>(scr + wr_base + (((4 * t + 2 * h + fh) ^ wr_key) * 16)) =
                    make_uint4(hw[0], hw[1], hw[2], hw[3]);
            }
        const int mbase = m0 + wm * Cfg::WTM + j * 32 + rrow;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = rrow + 8 * i;
            const uint4 v = *reinterpret_cast<const uint4 *>(scr + r * 128 + ((rq ^ ((r >> 1) & 7)) * 16));
            const int m = mbase + 8 * i;
            // (streaming store: the output is written once and not read by this kernel; kept out of the way of
            // the operand panels that other tiles re-read from L2)
            if (m < p.M && n < p.N) {
                typedef unsigned v4u __attribute__((ext_vector_type(4)));
                __builtin_nontemporal_store(v4u{v.x, v.y, v.z, v.w},
                                            reinterpret_cast<v4u *>((uint16_t *)p.out + (int64_t)m * p.N + n));
            }
        }
    });
}

// Epilogue combinations with a dedicated instantiation of the fast kernels.
enum { EPI_F16 = 0, EPI_BF16, EPI_F32, EPI_F16_RES16, EPI_I4_GELU, EPI_I4, EPI_I8_GELU, EPI_GENERIC };

inline int classify_epilogue(const GemmI4Params &p)
{
    if ((p.N % 8) != 0 || p.acc_out || p.q_out) return EPI_GENERIC;
    const bool res16 = p.residual && p.residual_dtype == MKQ_F16;
    const bool gelu = p.act == MKQ_ACT_GELU;
    if (p.residual && !res16) return EPI_GENERIC;
    if (p.out_dtype == MKQ_F16 && !gelu) return res16 ? EPI_F16_RES16 : EPI_F16;
    if (res16) return EPI_GENERIC;
    if (p.out_dtype == MKQ_BF16 && !gelu) return EPI_BF16;
    if (p.out_dtype == MKQ_F32 && !gelu) return EPI_F32;
    if (p.out_dtype == MKQ_I4) return gelu ? EPI_I4_GELU : EPI_I4;
    if (p.out_dtype == MKQ_I8 && gelu && !p.residual) return EPI_I8_GELU;
    return EPI_GENERIC;
}


}  // namespace mkq
