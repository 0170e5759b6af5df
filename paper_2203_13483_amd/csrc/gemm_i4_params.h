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
    // What the int32 accumulator holds: 2^acc_shift * sum(a*w).  The 4-bit path feeds the
    // matrix core 16*code on both sides (shift 8); the 8-bit path feeds the codes themselves.
    int acc_shift;
    float acc_unit;     // 2^-acc_shift, folded into the per-channel scale (exact)
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
                    uint8_t *qdst = (uint8_t *)p.out + o;
                    if (vec_ok) {
                        *reinterpret_cast<uint2 *>(qdst) = bytes8(cd);
                    } else {
                        for (int e = 0; e < nvalid; ++e) qdst[e] = (uint8_t)cd[e];
                    }
                }
                if (out_dtype == MKQ_I4 || q_extra) {
                    // Eq. 1 on the binary32 value.  N is even and nb % 8 == 0, so o is even.
                    uint32_t packed = 0;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        packed |= ((uint32_t)quantize_code(y[e], p.s_next) & 0xFu) << (4 * e);
                    uint8_t *qdst = (out_dtype == MKQ_I4 ? (uint8_t *)p.out : q_extra) + (o >> 1);
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

}  // namespace mkq
