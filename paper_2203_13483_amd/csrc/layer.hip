// The glue of the encoder layer (section 3.2; float32 islands of section 5):
// LayerNorm and the attention core, each with a fused re-quantization of its
// result for the next W4A4 linear, and the host-side sequencing of one post-LN
// BERT layer in the int4 and in the binary16 baseline flavour.
#include "gemm_common.h"

#include <type_traits>

namespace mkq {

// ---------------------------------------------------------------------------------
// LayerNorm over the last dimension: one wavefront per row, the row lives in
// registers (binary32), two passes for mean and variance, wave-level reductions.
// Writes the binary16 result and / or its 4-bit codes (Eq. 1 on the binary32 value).
template <int MAXC>
__global__ __launch_bounds__(256) void layernorm_kernel(const uint16_t *__restrict__ x, int M, int D,
                                                        const float *__restrict__ gamma,
                                                        const float *__restrict__ beta, float eps,
                                                        uint16_t *__restrict__ y, float s_next,
                                                        uint32_t *__restrict__ q, int q_bits, int q_chunks)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= M) return;
    const int chunks = D / 8;  // 16-byte chunks of 8 elements
    float v[MAXC][8];
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + i * 64;
        if (c < chunks) {
            const uint4 raw = *reinterpret_cast<const uint4 *>(x + (int64_t)row * D + c * 8);
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[i][2 * e] = half_bits_to_float((uint16_t)(w[e] & 0xFFFFu));
                v[i][2 * e + 1] = half_bits_to_float((uint16_t)(w[e] >> 16));
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) sum += v[i][e];
        }
    }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        if (lane + i * 64 < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = v[i][e] - mean;
                sq += d * d;
            }
        }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + i * 64;
        if (c < chunks) {
            float o[8];
            const float4 g0 = gamma ? *reinterpret_cast<const float4 *>(gamma + c * 8) : make_float4(1, 1, 1, 1);
            const float4 g1 = gamma ? *reinterpret_cast<const float4 *>(gamma + c * 8 + 4) : make_float4(1, 1, 1, 1);
            const float4 b0 = beta ? *reinterpret_cast<const float4 *>(beta + c * 8) : make_float4(0, 0, 0, 0);
            const float4 b1 = beta ? *reinterpret_cast<const float4 *>(beta + c * 8 + 4) : make_float4(0, 0, 0, 0);
            const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
            const float bb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (v[i][e] - mean) * rstd * gg[e] + bb[e];
            if (y)
                *reinterpret_cast<uint4 *>(y + (int64_t)row * D + c * 8) =
                    make_uint4(pack2_f16(o[0], o[1]), pack2_f16(o[2], o[3]), pack2_f16(o[4], o[5]), pack2_f16(o[6], o[7]));
            if (q && q_bits == 8) {
                const uint2 pk8 = quantize8<8>(o, quant_step<8>(s_next));
                reinterpret_cast<uint2 *>(q)[(int64_t)row * q_chunks + c] = pk8;
            } else if (q) {
                const uint32_t packed = quantize8<4>(o, quant_step<4>(s_next)).x;
                q[(int64_t)row * q_chunks + c] = packed;
            }
        } else if (q && c < q_chunks) {  // padding codes of a row with a pitch: zero
            if (q_bits == 8) reinterpret_cast<uint2 *>(q)[(int64_t)row * q_chunks + c] = make_uint2(0u, 0u);
            else q[(int64_t)row * q_chunks + c] = 0u;
        }
    }
}

// The same for D <= 1024: one row per half wave (32 lanes, chunks lane, lane + 32, ...: D = 768
// and 1024 divide evenly), so a lane has up to four 16-byte loads in flight and the two
// reductions take five steps; gamma and beta are fetched before the reductions, not after.
template <int MAXC>
__global__ __launch_bounds__(256) void layernorm_half_kernel(const uint16_t *__restrict__ x, int M, int D,
                                                             const float *__restrict__ gamma,
                                                             const float *__restrict__ beta, float eps,
                                                             uint16_t *__restrict__ y, float s_next,
                                                             uint32_t *__restrict__ q, int q_bits, int q_chunks)
{
    const int lane = threadIdx.x & 31;
    const int row = blockIdx.x * 8 + (threadIdx.x >> 5);
    if (row >= M) return;
    const int chunks = D / 8;
    float v[MAXC][8], gg[MAXC][8], bb[MAXC][8];
    uint4 raw[MAXC];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + i * 32;
        raw[i] = (c < chunks) ? *reinterpret_cast<const uint4 *>(x + (int64_t)row * D + c * 8) : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + i * 32;
        const bool in = c < chunks;
        const float4 g0 = (gamma && in) ? *reinterpret_cast<const float4 *>(gamma + c * 8) : make_float4(1, 1, 1, 1);
        const float4 g1 = (gamma && in) ? *reinterpret_cast<const float4 *>(gamma + c * 8 + 4) : make_float4(1, 1, 1, 1);
        const float4 b0 = (beta && in) ? *reinterpret_cast<const float4 *>(beta + c * 8) : make_float4(0, 0, 0, 0);
        const float4 b1 = (beta && in) ? *reinterpret_cast<const float4 *>(beta + c * 8 + 4) : make_float4(0, 0, 0, 0);
        gg[i][0] = g0.x; gg[i][1] = g0.y; gg[i][2] = g0.z; gg[i][3] = g0.w;
        gg[i][4] = g1.x; gg[i][5] = g1.y; gg[i][6] = g1.z; gg[i][7] = g1.w;
        bb[i][0] = b0.x; bb[i][1] = b0.y; bb[i][2] = b0.z; bb[i][3] = b0.w;
        bb[i][4] = b1.x; bb[i][5] = b1.y; bb[i][6] = b1.z; bb[i][7] = b1.w;
    }
    float sum = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const uint32_t w[4] = {raw[i].x, raw[i].y, raw[i].z, raw[i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v[i][2 * e] = half_bits_to_float((uint16_t)(w[e] & 0xFFFFu));
            v[i][2 * e + 1] = half_bits_to_float((uint16_t)(w[e] >> 16));
        }
        // chunks past the row hold zeros and add nothing; the order of the sum is the one of
        // the whole-wave kernel within a lane
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += v[i][e];
    }
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    const float mean = sum / (float)D;
    float sq = 0.0f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        if (lane + i * 32 < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float d = v[i][e] - mean;
                sq += d * d;
            }
        }
    }
#pragma unroll
    for (int off = 16; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
    const float rstd = 1.0f / sqrtf(sq / (float)D + eps);
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = lane + i * 32;
        if (c < chunks) {
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (v[i][e] - mean) * rstd * gg[i][e] + bb[i][e];
            if (y)
                *reinterpret_cast<uint4 *>(y + (int64_t)row * D + c * 8) =
                    make_uint4(pack2_f16(o[0], o[1]), pack2_f16(o[2], o[3]), pack2_f16(o[4], o[5]), pack2_f16(o[6], o[7]));
            if (q && q_bits == 8) {
                const uint2 pk8 = quantize8<8>(o, quant_step<8>(s_next));
                reinterpret_cast<uint2 *>(q)[(int64_t)row * q_chunks + c] = pk8;
            } else if (q) {
                const uint32_t packed = quantize8<4>(o, quant_step<4>(s_next)).x;
                q[(int64_t)row * q_chunks + c] = packed;
            }
        } else if (q && c < q_chunks) {  // padding codes of a row with a pitch: zero
            if (q_bits == 8) reinterpret_cast<uint2 *>(q)[(int64_t)row * q_chunks + c] = make_uint2(0u, 0u);
            else q[(int64_t)row * q_chunks + c] = 0u;
        }
    }
}

// ---------------------------------------------------------------------------------
// Attention core for one (sequence, head) per workgroup: d_k = 64, seq = 32*KT <= 128.
//   S^T = K Q^T / sqrt(d_k)   (MFMA "A" = keys in permuted row order, "B" = queries)
//   P   = softmax over keys   (binary32; a query's 32*KT scores sit in two lanes)
//   O^T = V^T P^T             ("A" = V^T from a transposed LDS copy, "B" = P, which is
//                              already in operand layout thanks to the key permutation)
// Each of the four waves owns 32 queries.  A lane ends with 8 consecutive head
// dimensions of one query, stored as binary16 and / or as 4-bit codes.
template <int KT>
__global__ __launch_bounds__(256) void attention_kernel(const uint16_t *__restrict__ qkv, int seq_fixed, int hidden,
                                                        int heads, uint16_t *__restrict__ ctx, float s_next,
                                                        uint8_t *__restrict__ qout, int q_bits,
                                                        const int32_t *__restrict__ cu_seqlens)
{
    constexpr int DK = 64, SMAX = 32 * KT;
    __shared__ __attribute__((aligned(16))) uint8_t sQ[SMAX * 128];
    __shared__ __attribute__((aligned(16))) uint8_t sK[SMAX * 128];
    // V^T as [d][key]; a row is VCHP 16-byte chunks (power of two, so the XOR swizzle stays inside it)
    constexpr int VCHP = (KT == 1) ? 4 : (KT == 2) ? 8 : 16;
    constexpr int VROW = VCHP * 16;
    __shared__ __attribute__((aligned(16))) uint8_t sVt[DK * VROW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fh = lane >> 5;
    const int b = blockIdx.x / heads, head = blockIdx.x % heads;
    // padding-free batches: sequence b is rows cu_seqlens[b] .. cu_seqlens[b+1] - 1 (at most 32*KT of
    // them, any number); otherwise every sequence has seq_fixed rows
    const int64_t row0 = cu_seqlens ? (int64_t)cu_seqlens[b] : (int64_t)b * seq_fixed;
    const int seq = cu_seqlens ? (cu_seqlens[b + 1] - cu_seqlens[b]) : seq_fixed;
    if (seq <= 0) return;
    const int ld = 3 * hidden;

    // stage Q, K (row-major, swizzled chunks) and V (transposed): all of a thread's loads are issued
    // before the first LDS write, so the tile arrives in one memory round trip
    constexpr int PER_T = SMAX * 8 / 256;  // 16-byte chunks of each of q, k, v per thread
    // With an even number of chunks per thread the v chunks of a thread are the same columns of two neighbouring
    // rows (chunks 2i, 2i + 1), so the transposition writes the two keys of a head dimension with one LDS store.
    constexpr bool PAIRS = (PER_T % 2) == 0;
    auto v_row = [&](int i) { return PAIRS ? 2 * ((tid + (i >> 1) * 256) >> 3) + (i & 1) : (tid + i * 256) >> 3; };
    auto v_col = [&](int i) { return PAIRS ? (tid + (i >> 1) * 256) & 7 : (tid + i * 256) & 7; };
    uint4 qv[PER_T], kv[PER_T], vv[PER_T];
#pragma unroll
    for (int i = 0; i < PER_T; ++i) {
        const int idx = tid + i * 256;
        const int r = idx >> 3, c = idx & 7;
        const uint16_t *src = qkv + (row0 + (r < seq ? r : seq - 1)) * ld + head * DK + c * 8;
        qv[i] = *reinterpret_cast<const uint4 *>(src);
        kv[i] = *reinterpret_cast<const uint4 *>(src + hidden);
        const int rv = v_row(i);
        vv[i] = *reinterpret_cast<const uint4 *>(qkv + (row0 + (rv < seq ? rv : seq - 1)) * ld + 2 * hidden + head * DK +
                                                 v_col(i) * 8);
    }
#pragma unroll
    for (int i = 0; i < PER_T; ++i) {
        const int idx = tid + i * 256;
        const int r = idx >> 3, c = idx & 7;
        const int slot = (c ^ swz<8>(r & 15)) * 16;
        *reinterpret_cast<uint4 *>(sQ + r * 128 + slot) = qv[i];
        *reinterpret_cast<uint4 *>(sK + r * 128 + slot) = kv[i];
        if constexpr (PAIRS) {
            if (i & 1) continue;  // (chunks 2i and 2i + 1 go together)
            const int rv = v_row(i), cv = v_col(i);
            const uint32_t w0[4] = {vv[i].x, vv[i].y, vv[i].z, vv[i].w};
            const uint32_t w1[4] = {vv[i | 1].x, vv[i | 1].y, vv[i | 1].z, vv[i | 1].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int d = cv * 8 + e;
                const uint32_t lo = (w0[e >> 1] >> (16 * (e & 1))) & 0xFFFFu, hi = (w1[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                const int vslot = ((rv >> 3) ^ (d & (VCHP - 1))) * 16;
                *reinterpret_cast<uint32_t *>(sVt + d * VROW + vslot + (rv & 7) * 2) = lo | (hi << 16);
            }
        } else {
            const uint32_t w[4] = {vv[i].x, vv[i].y, vv[i].z, vv[i].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int d = c * 8 + e;
                const uint16_t val = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                const int vslot = ((r >> 3) ^ (d & (VCHP - 1))) * 16;
                *reinterpret_cast<uint16_t *>(sVt + d * VROW + vslot + (r & 7) * 2) = val;
            }
        }
    }
    __syncthreads();
    if (wave * 32 >= seq) return;  // no queries for this wave (seq < 128)

    // scores (transposed): sc[kt] rows = keys of tile kt (permuted), column = query fr
    v16f sc[KT];
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[kt][v] = 0.0f;
    const int qrow = wave * 32 + fr;
#pragma unroll
    for (int ds = 0; ds < DK / 16; ++ds) {
        const int c = ds * 2 + fh;
        const v8h qf = *reinterpret_cast<const v8h *>(sQ + qrow * 128 + ((c ^ swz<8>(qrow & 15)) * 16));
#pragma unroll
        for (int kt = 0; kt < KT; ++kt) {
            const int krow = kt * 32 + w_row_perm(fr);
            const v8h kf = *reinterpret_cast<const v8h *>(sK + krow * 128 + ((c ^ swz<8>(krow & 15)) * 16));
            sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf, sc[kt], 0, 0, 0);
        }
    }
    // register v of tile kt is key kt*32 + 16*(v/8) + 8*fh + v%8; keys >= seq do not exist
    // exp(x / sqrt(64) - max) as exp2(x c - max c): one multiply-add and one exponential per score
    const float c_exp = 0.125f * 1.4426950408889634f;
    float mx = -1.0e30f;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = kt * 32 + 16 * (v / 8) + 8 * fh + (v % 8);
            sc[kt][v] = (key < seq) ? sc[kt][v] : -1.0e30f;
            mx = fmaxf(mx, sc[kt][v]);
        }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float shift = -mx * c_exp;
    float den = 0.0f;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            sc[kt][v] = __builtin_amdgcn_exp2f(__fmaf_rn(sc[kt][v], c_exp, shift));
            den += sc[kt][v];
        }
    den += __shfl_xor(den, 32, 64);
    const float inv = 1.0f / den;

    // O^T = V^T P^T
    v16f ot[2];
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) ot[dt][v] = 0.0f;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            v8h pf;
#pragma unroll
            for (int e = 0; e < 8; ++e) pf[e] = (_Float16)(sc[kt][8 * st + e] * inv);
            const int kc = (2 * kt + st) * 2 + fh;  // chunk of 8 keys
#pragma unroll
            for (int dt = 0; dt < 2; ++dt) {
                const int d = dt * 32 + w_row_perm(fr);
                const v8h vf = *reinterpret_cast<const v8h *>(sVt + d * VROW + ((kc ^ (d & (VCHP - 1))) * 16));
                ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, ot[dt], 0, 0, 0);
            }
        }

    if (qrow >= seq) return;
    const int64_t orow = row0 + qrow;
#pragma unroll
    for (int dt = 0; dt < 2; ++dt)
#pragma unroll
        for (int G = 0; G < 2; ++G) {
            const int d0 = dt * 32 + 16 * G + 8 * fh;
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = ot[dt][8 * G + e];
            const int64_t off = orow * hidden + head * DK + d0;
            if (ctx)
                *reinterpret_cast<uint4 *>(ctx + off) =
                    make_uint4(pack2_f16(o[0], o[1]), pack2_f16(o[2], o[3]), pack2_f16(o[4], o[5]), pack2_f16(o[6], o[7]));
            if (qout && q_bits == 8) {
                const uint2 pk8 = quantize8<8>(o, quant_step<8>(s_next));
                *reinterpret_cast<uint2 *>(qout + off) = pk8;
            } else if (qout) {
                const uint32_t packed = quantize8<4>(o, quant_step<4>(s_next)).x;
                *reinterpret_cast<uint32_t *>(qout + (off >> 1)) = packed;
            }
        }
}

// ---------------------------------------------------------------------------------
// Attention core for any sequence length and any even head size d_k <= DKP (DKP = 32 or 64; the head
// dimensions d_k .. DKP-1 are zero in the staged q, k, v and never stored).  One workgroup per (sequence,
// head, block of 128 queries); the keys go through LDS in blocks of 128, twice:
//   pass 1  S^T = K Q^T / sqrt(d_k) per key block, running row maximum and denominator of the softmax
//   pass 2  the same scores again, P = exp(S - max) / denominator in binary32, narrowed to binary16, and
//           O^T += V^T P^T
// so the probabilities that meet V are the normalized ones, as in the one-block kernel above (an online
// softmax would narrow unnormalized ones).  VEC = 8: 16-byte accesses (d_k % 8 == 0); VEC = 2: 4-byte ones.
template <int DKP, int VEC>
__global__ __launch_bounds__(256, 3) void attention_blocks_kernel(const uint16_t *__restrict__ qkv, int seq_fixed,
                                                               int hidden, int heads, int dk, int q_blocks,
                                                               uint16_t *__restrict__ ctx, float s_next,
                                                               uint8_t *__restrict__ qout, int q_bits, int q_pitch,
                                                               const int32_t *__restrict__ cu_seqlens)
{
    constexpr int ROWB = DKP * 2;  // bytes of a staged q or k row
    constexpr int CH = DKP / 8;    // its 16-byte chunks
    constexpr int VROW = 256;      // V^T row: 128 keys
    __shared__ __attribute__((aligned(16))) uint8_t sK[128 * ROWB];  // first the queries, then the key blocks
    __shared__ __attribute__((aligned(16))) uint8_t sVt[DKP * VROW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, fh = lane >> 5;
    const int qb = blockIdx.x % q_blocks, bh = blockIdx.x / q_blocks;
    const int b = bh / heads, head = bh % heads;
    const int64_t row0 = cu_seqlens ? (int64_t)cu_seqlens[b] : (int64_t)b * seq_fixed;
    const int seq = cu_seqlens ? (cu_seqlens[b + 1] - cu_seqlens[b]) : seq_fixed;
    const int q_base = qb * 128;
    if (q_base >= seq) return;  // the whole workgroup: no barrier has been passed
    const int ld = 3 * hidden;
    const int key_blocks = (seq + 127) / 128;

    using Piece = typename std::conditional<VEC == 8, uint4, uint32_t>::type;
    constexpr int PER_T = 128 * DKP / VEC / 256;  // pieces of one 128-row block per thread
    // rows r_base .. r_base + 127 of the sequence (clamped to its last row), columns col + head * dk + [0, DKP)
    auto load_block = [&](Piece (&v)[PER_T], int r_base, int col) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int idx = tid + i * 256;
            const int r = idx / (DKP / VEC), d = (idx % (DKP / VEC)) * VEC;
            int rr = r_base + r;
            rr = rr < seq ? rr : seq - 1;
            if (d < dk) v[i] = *reinterpret_cast<const Piece *>(qkv + (row0 + rr) * ld + col + head * dk + d);
            else v[i] = Piece{};
        }
    };
    auto store_rows = [&](uint8_t *dst, const Piece (&v)[PER_T]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int idx = tid + i * 256;
            const int r = idx / (DKP / VEC), d = (idx % (DKP / VEC)) * VEC;
            *reinterpret_cast<Piece *>(dst + r * ROWB + (((d >> 3) ^ swz<CH>(r & 15)) * 16) + (d & 7) * 2) = v[i];
        }
    };
    // V is stored transposed, [d][key]: a thread takes the same columns of two neighbouring rows (pieces 2i and
    // 2i + 1), so every LDS write carries the two keys of one head dimension
    static_assert(PER_T % 2 == 0, "pairs of rows");
    auto load_block_pairs = [&](Piece (&v)[PER_T], int r_base, int col) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER_T; ++i) {
            const int j = tid + (i >> 1) * 256;
            const int r = 2 * (j / (DKP / VEC)) + (i & 1), d = (j % (DKP / VEC)) * VEC;
            int rr = r_base + r;
            rr = rr < seq ? rr : seq - 1;
            if (d < dk) v[i] = *reinterpret_cast<const Piece *>(qkv + (row0 + rr) * ld + col + head * dk + d);
            else v[i] = Piece{};
        }
    };
    auto store_transposed = [&](const Piece (&v)[PER_T]) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < PER_T; i += 2) {
            const int j = tid + (i >> 1) * 256;
            const int r = 2 * (j / (DKP / VEC)), d0 = (j % (DKP / VEC)) * VEC;
            uint32_t w0[VEC / 2], w1[VEC / 2];
            if constexpr (VEC == 8) {
                w0[0] = v[i].x; w0[1] = v[i].y; w0[2] = v[i].z; w0[3] = v[i].w;
                w1[0] = v[i + 1].x; w1[1] = v[i + 1].y; w1[2] = v[i + 1].z; w1[3] = v[i + 1].w;
            } else {
                w0[0] = v[i];
                w1[0] = v[i + 1];
            }
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int d = d0 + e;
                const uint32_t lo = (w0[e >> 1] >> (16 * (e & 1))) & 0xFFFFu, hi = (w1[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                *reinterpret_cast<uint32_t *>(sVt + d * VROW + (((r >> 3) ^ (d & 15)) * 16) + (r & 7) * 2) = lo | (hi << 16);
            }
        }
    };

    const bool active = q_base + wave * 32 < seq;  // this wave has queries
    const int qrow = wave * 32 + fr;                // within the block
    // exp(x / sqrt(d_k)) as exp2(x * c): one multiply-add and one exponential per score
    const float c_exp = (1.0f / sqrtf((float)dk)) * 1.4426950408889634f;
    constexpr float MASKED = -1.0e30f;  // a key past the end of the sequence: exp2 gives 0
    v8h qf[DKP / 16];  // this lane's query as MFMA operand
    // raw scores q.k of the 32 keys of tile kt of block kb (transposed): register v is key
    // kb*128 + kt*32 + 16*(v/8) + 8*fh + v%8
    auto score_tile = [&](int kb, int kt) __attribute__((always_inline)) {
        v16f sc;
#pragma unroll
        for (int v = 0; v < 16; ++v) sc[v] = 0.0f;
        const int krow = kt * 32 + w_row_perm(fr);
#pragma unroll
        for (int ds = 0; ds < DKP / 16; ++ds) {
            const v8h kf = *reinterpret_cast<const v8h *>(sK + krow * ROWB + (((ds * 2 + fh) ^ swz<CH>(krow & 15)) * 16));
            sc = __builtin_amdgcn_mfma_f32_32x32x16_f16(kf, qf[ds], sc, 0, 0, 0);
        }
        if (kb * 128 + kt * 32 + 32 > seq) {  // (uniform) the tile holds keys that do not exist
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = kb * 128 + kt * 32 + 16 * (v / 8) + 8 * fh + (v % 8);
                sc[v] = (key < seq) ? sc[v] : MASKED;
            }
        }
        return sc;
    };

    // The next block's rows are loaded into registers before the current block is computed and written to
    // LDS after it, so the trip to memory hides behind the arithmetic.
    Piece ldK[PER_T], ldV[PER_T];
    load_block(ldV, q_base, 0);
    load_block(ldK, 0, hidden);
    store_rows(sK, ldV);
    __syncthreads();
#pragma unroll
    for (int ds = 0; ds < DKP / 16; ++ds)
        qf[ds] = *reinterpret_cast<const v8h *>(sK + qrow * ROWB + (((ds * 2 + fh) ^ swz<CH>(qrow & 15)) * 16));
    __syncthreads();
    store_rows(sK, ldK);
    __syncthreads();

    // pass 1: row maximum and denominator (each lane sums its half of the keys; the halves meet at the end)
    float mx = MASKED, den = 0.0f;  // mx: maximum of the raw scores so far
    for (int kb = 0; kb < key_blocks; ++kb) {
        const bool more = kb + 1 < key_blocks;
        if (more) {
            load_block(ldK, (kb + 1) * 128, hidden);
        } else {  // the first block of pass 2
            load_block_pairs(ldV, 0, 2 * hidden);
            if (key_blocks > 1) load_block(ldK, 0, hidden);
        }
        if (active) {
#pragma unroll 1
            for (int kt = 0; kt < 4; ++kt) {
                const v16f sc = score_tile(kb, kt);
                float bm = sc[0];
#pragma unroll
                for (int v = 1; v < 16; ++v) bm = fmaxf(bm, sc[v]);
                bm = fmaxf(bm, __shfl_xor(bm, 32, 64));
                const float m_new = fmaxf(mx, bm);
                const float shift = -m_new * c_exp;
                float part = 0.0f;
#pragma unroll
                for (int v = 0; v < 16; ++v) part += __builtin_amdgcn_exp2f(__fmaf_rn(sc[v], c_exp, shift));
                den = den * __builtin_amdgcn_exp2f((mx - m_new) * c_exp) + part;
                mx = m_new;
            }
        }
        __syncthreads();  // every wave is done with the block
        if (more) {
            store_rows(sK, ldK);
        } else {
            store_transposed(ldV);
            if (key_blocks > 1) store_rows(sK, ldK);  // one block: the keys are still there
        }
        __syncthreads();
    }
    den += __shfl_xor(den, 32, 64);
    // p = exp2(x c - max c - log2(denominator)): the division folded into the exponent
    const float shift2 = -mx * c_exp - __log2f(den);

    // pass 2: O^T = V^T P^T over the key blocks
    constexpr int DT = DKP / 32;
    v16f ot[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) ot[dt][v] = 0.0f;
    for (int kb = 0; kb < key_blocks; ++kb) {
        const bool more = kb + 1 < key_blocks;
        if (more) {
            load_block_pairs(ldV, (kb + 1) * 128, 2 * hidden);
            load_block(ldK, (kb + 1) * 128, hidden);
        }
        if (active) {
#pragma unroll 1
            for (int kt = 0; kt < 4; ++kt) {
                const v16f sc = score_tile(kb, kt);
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    v8h pf;
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        pf[e] = (_Float16)__builtin_amdgcn_exp2f(__fmaf_rn(sc[8 * st + e], c_exp, shift2));
                    const int kc = (2 * kt + st) * 2 + fh;  // chunk of 8 keys
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        const int d = dt * 32 + w_row_perm(fr);
                        const v8h vf = *reinterpret_cast<const v8h *>(sVt + d * VROW + ((kc ^ (d & 15)) * 16));
                        ot[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, ot[dt], 0, 0, 0);
                    }
                }
            }
        }
        if (more) {
            __syncthreads();
            store_transposed(ldV);
            store_rows(sK, ldK);
            __syncthreads();
        }
    }

    if (q_base + qrow >= seq) return;
    const int64_t orow = row0 + q_base + qrow;
    if (qout && head == heads - 1 && fh == 0 && q_pitch > hidden) {
        // padding codes of a row with a pitch: zero (hidden and the pitch are multiples of 8 codes)
        if (q_bits == 8) {
            for (int c = hidden; c < q_pitch; c += 8) *reinterpret_cast<uint2 *>(qout + orow * q_pitch + c) = make_uint2(0u, 0u);
        } else {
            for (int c = hidden; c < q_pitch; c += 8) *reinterpret_cast<uint32_t *>(qout + ((orow * q_pitch + c) >> 1)) = 0u;
        }
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int G = 0; G < 2; ++G) {
            const int d0 = dt * 32 + 16 * G + 8 * fh;
            if (d0 >= dk) continue;
            const int nvalid = (dk - d0) < 8 ? (dk - d0) : 8;  // even
            float o[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = ot[dt][8 * G + e];
            const uint32_t h[4] = {pack2_f16(o[0], o[1]), pack2_f16(o[2], o[3]), pack2_f16(o[4], o[5]), pack2_f16(o[6], o[7])};
            if (ctx) {
                uint16_t *dst = ctx + orow * hidden + head * dk + d0;
                if constexpr (VEC == 8) *reinterpret_cast<uint4 *>(dst) = make_uint4(h[0], h[1], h[2], h[3]);
                else
                    for (int e = 0; e < nvalid / 2; ++e) reinterpret_cast<uint32_t *>(dst)[e] = h[e];
            }
            const int64_t qo = orow * q_pitch + head * dk + d0;  // in codes
            if (qout && q_bits == 8) {
                const uint2 pk8 = quantize8<8>(o, quant_step<8>(s_next));
                const uint2 pk = pk8;
                if constexpr (VEC == 8) *reinterpret_cast<uint2 *>(qout + qo) = pk;
                else
                    for (int e = 0; e < nvalid; ++e) qout[qo + e] = (uint8_t)((e < 4 ? pk.x : pk.y) >> (8 * (e & 3)));
            } else if (qout) {
                const uint32_t packed = quantize8<4>(o, quant_step<4>(s_next)).x;
                if constexpr (VEC == 8) *reinterpret_cast<uint32_t *>(qout + (qo >> 1)) = packed;
                else
                    for (int e = 0; e < nvalid / 2; ++e) qout[(qo >> 1) + e] = (uint8_t)(packed >> (8 * e));
            }
        }
}

static inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace mkq

using namespace mkq;

// q_pitch: codes per row of q_out (0: D; at most D rounded up to a multiple of 128, which every kernel
// variant's lanes cover): the codes D .. q_pitch - 1 of a row are written as zero
static int layernorm_run(const void *x, int64_t M, int64_t D, const float *gamma, const float *beta, float eps,
                         void *y, float s_next, void *q_out, int q_bits, void *stream, int64_t q_pitch = 0)
{
    if (M < 0 || D <= 0 || (D % 8) != 0) return MKQ_ERR_SHAPE;
    if (q_pitch == 0) q_pitch = D;
    if (q_pitch < D || (q_pitch % 8) != 0 || q_pitch > ceil_div(D, 128) * 128) return MKQ_ERR_SHAPE;
    const int q_chunks = (int)(q_pitch / 8);
    if (D > 8192) return MKQ_ERR_UNSUPPORTED;
    if (q_out && !scale_ok(s_next)) return MKQ_ERR_SCALE;
    if (!(eps >= 0.0f)) return MKQ_ERR_SCALE;
    if (M == 0) return MKQ_OK;
    if (!x || (!y && !q_out)) return MKQ_ERR_NULL;
    if (!aligned16(x) || (y && !aligned16(y)) || (q_out && !aligned16(q_out)) || (gamma && !aligned16(gamma)) ||
        (beta && !aligned16(beta)))
        return MKQ_ERR_ALIGN;
    if (M > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    const unsigned grid = (unsigned)ceil_div(M, 4);
    hipStream_t st = as_stream(stream);
#define MKQ_LN(C)                                                                                       \
    layernorm_kernel<C><<<grid, 256, 0, st>>>((const uint16_t *)x, (int)M, (int)D, gamma, beta, eps, \
                                              (uint16_t *)y, s_next, (uint32_t *)q_out, q_bits, q_chunks)
    if (D <= 1024 && M >= 2048) {
        const unsigned grid8 = (unsigned)ceil_div(M, 8);
#define MKQ_LNH(C)                                                                                             \
    layernorm_half_kernel<C><<<grid8, 256, 0, st>>>((const uint16_t *)x, (int)M, (int)D, gamma, beta, eps, \
                                                    (uint16_t *)y, s_next, (uint32_t *)q_out, q_bits, q_chunks)
        if (D <= 256) MKQ_LNH(1);
        else if (D <= 512) MKQ_LNH(2);
        else if (D <= 768) MKQ_LNH(3);
        else MKQ_LNH(4);
#undef MKQ_LNH
    } else if (D <= 1024) MKQ_LN(2);
    else if (D <= 2048) MKQ_LN(4);
    else if (D <= 4096) MKQ_LN(8);
    else MKQ_LN(16);
#undef MKQ_LN
    return launch_status();
}

extern "C" int mkq_layernorm(const void *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                             float eps, void *y, float s_next, uint8_t *q_out, void *stream)
{
    return layernorm_run(x, M, D, gamma, beta, eps, y, s_next, q_out, 4, stream);
}

extern "C" int mkq_layernorm_int8(const void *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                                  float eps, void *y, float s_next, int8_t *q_out, void *stream)
{
    return layernorm_run(x, M, D, gamma, beta, eps, y, s_next, q_out, 8, stream);
}

// Longest sequence the attention kernels take (the key loop has no limit of its own; this bounds the grid).
constexpr int64_t ATTENTION_MAX_SEQ = 4096;

// cu: null (every sequence has seq rows) or device array [batch + 1] of row offsets (then seq is only an
// upper bound of the lengths).  q_pitch: codes per row of q_out (0: hidden).
static int attention_run(const void *qkv, int64_t batch, int64_t seq, int64_t hidden, int64_t heads, void *ctx,
                         float s_next, void *q_out_v, int q_bits, void *stream, const int32_t *cu = nullptr,
                         int64_t q_pitch = 0)
{
    uint8_t *q_out = (uint8_t *)q_out_v;
    if (batch < 0 || seq <= 0 || hidden <= 0 || heads <= 0 || (hidden % heads) != 0) return MKQ_ERR_SHAPE;
    if (q_pitch == 0) q_pitch = hidden;
    if (q_pitch < hidden || (q_pitch % 8) != 0) return MKQ_ERR_SHAPE;
    if (q_out && !scale_ok(s_next)) return MKQ_ERR_SCALE;
    const int64_t dk = hidden / heads;
    const int64_t q_blocks = ceil_div(seq, 128);
    if (dk > 64 || (dk % 2) != 0 || (hidden % 8) != 0 || seq > ATTENTION_MAX_SEQ ||
        batch * heads * q_blocks > 0x7FFFFFFF)
        return MKQ_ERR_UNSUPPORTED;
    if (batch == 0) return MKQ_OK;
    if (!qkv || (!ctx && !q_out)) return MKQ_ERR_NULL;
    if (!aligned16(qkv) || (ctx && !aligned16(ctx)) || (q_out && !aligned16(q_out))) return MKQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    const uint16_t *in = (const uint16_t *)qkv;
    if (dk != 64 || seq > 128 || q_pitch != hidden) {
        const unsigned grid = (unsigned)(batch * heads * q_blocks);
#define MKQ_ATT(DKP, VEC)                                                                                        \
    attention_blocks_kernel<DKP, VEC><<<grid, 256, 0, st>>>(in, (int)seq, (int)hidden, (int)heads, (int)dk,     \
                                                            (int)q_blocks, (uint16_t *)ctx, s_next, q_out, q_bits, \
                                                            (int)q_pitch, cu)
        if ((dk % 8) == 0) {
            if (dk <= 32) MKQ_ATT(32, 8);
            else MKQ_ATT(64, 8);
        } else {
            if (dk <= 32) MKQ_ATT(32, 2);
            else MKQ_ATT(64, 2);
        }
#undef MKQ_ATT
        return launch_status();
    }
    const unsigned grid = (unsigned)(batch * heads);
    switch (ceil_div(seq, 32)) {
    case 1: attention_kernel<1><<<grid, 256, 0, st>>>(in, (int)seq, (int)hidden, (int)heads, (uint16_t *)ctx, s_next, q_out, q_bits, cu); break;
    case 2: attention_kernel<2><<<grid, 256, 0, st>>>(in, (int)seq, (int)hidden, (int)heads, (uint16_t *)ctx, s_next, q_out, q_bits, cu); break;
    case 3: attention_kernel<3><<<grid, 256, 0, st>>>(in, (int)seq, (int)hidden, (int)heads, (uint16_t *)ctx, s_next, q_out, q_bits, cu); break;
    default: attention_kernel<4><<<grid, 256, 0, st>>>(in, (int)seq, (int)hidden, (int)heads, (uint16_t *)ctx, s_next, q_out, q_bits, cu); break;
    }
    return launch_status();
}

extern "C" int mkq_attention(const void *qkv, int64_t batch, int64_t seq, int64_t hidden, int64_t heads,
                             void *ctx, float s_next, uint8_t *q_out, void *stream)
{
    return attention_run(qkv, batch, seq, hidden, heads, ctx, s_next, q_out, 4, stream);
}

extern "C" int mkq_attention_int8(const void *qkv, int64_t batch, int64_t seq, int64_t hidden, int64_t heads,
                                  void *ctx, float s_next, int8_t *q_out, void *stream)
{
    return attention_run(qkv, batch, seq, hidden, heads, ctx, s_next, q_out, 8, stream);
}

extern "C" int mkq_attention_varlen(const void *qkv, const int32_t *cu_seqlens, int64_t batch, int64_t max_seq,
                                    int64_t hidden, int64_t heads, void *ctx, float s_next, void *q_out,
                                    int q_bits, void *stream)
{
    if (!cu_seqlens) return MKQ_ERR_NULL;
    if (q_bits != 4 && q_bits != 8) return MKQ_ERR_DTYPE;
    if (reinterpret_cast<uintptr_t>(cu_seqlens) & 3u) return MKQ_ERR_ALIGN;
    return attention_run(qkv, batch, max_seq, hidden, heads, ctx, s_next, q_out, q_bits, stream, cu_seqlens);
}

// ---------------------------------------------------------------------------------
// varlen: seq is an upper bound of the sequence lengths of a padding-free batch of `tokens` rows.
// bits: 4, 8, or 16 for the binary16 baseline.  Only the 4-bit layer pads reduction lengths.
static int check_layer_dims(int bits, int64_t batch, int64_t seq, int64_t hidden, int64_t heads, int64_t ffn,
                            bool varlen = false, int64_t tokens = 0)
{
    if (batch < 0 || seq <= 0 || hidden <= 0 || heads <= 0 || ffn <= 0) return MKQ_ERR_SHAPE;
    const int64_t unit = bits == 4 ? 8 : 64;
    if ((hidden % unit) != 0 || (ffn % unit) != 0 || (hidden % heads) != 0) return MKQ_ERR_SHAPE;
    if (varlen && (tokens < 0 || tokens > batch * seq)) return MKQ_ERR_SHAPE;
    const int64_t dk = hidden / heads;
    if (dk > 64 || (dk % 2) != 0 || seq > ATTENTION_MAX_SEQ || hidden > 8192) return MKQ_ERR_UNSUPPORTED;
    return MKQ_OK;
}

// Codes per row of a buffer that feeds a linear of reduction length K: the 4-bit linear takes K % 32 == 0,
// other lengths are padded with zero codes.
static inline int64_t code_row(int bits, int64_t K)
{
    return (bits == 4 && (K % 32) != 0) ? mkq_padded_k(K) : K;
}


template <class P>
static inline int64_t layer_tokens(const P *p)
{
    return p->cu_seqlens ? p->total_tokens : p->batch * p->seq;
}

// bits = 4: two codes per byte; bits = 8: one
static int layer_workspace(const mkq_bert_layer_params *p, mkq_bert_layer_workspace_layout *L, int bits)
{
    if (!p || !L) return MKQ_ERR_NULL;
    const int rc = check_layer_dims(bits, p->batch, p->seq, p->hidden, p->heads, p->ffn, p->cu_seqlens != nullptr,
                                    p->total_tokens);
    if (rc != MKQ_OK) return rc;
    const size_t M = (size_t)layer_tokens(p), H = (size_t)p->hidden;
    const size_t Hp = (size_t)code_row(bits, p->hidden), Fp = (size_t)code_row(bits, p->ffn);
    const size_t cpb = bits == 4 ? 2 : 1;  // codes per byte
    size_t o = 0;
    L->c0 = o;  o += align256(M * Hp / cpb);
    L->qkv = o; o += align256(M * 3 * H * 2);
    L->c1 = o;  o += align256(M * Hp / cpb);
    L->u = o;   o += align256(M * H * 2);
    L->h1 = o;  o += align256(M * H * 2);
    L->c2 = o;  o += align256(M * Hp / cpb);
    L->c3 = o;  o += align256(M * Fp / cpb);
    L->d = o;   o += align256(M * H * 2);
    L->total = o;
    return MKQ_OK;
}

extern "C" int mkq_bert_layer_workspace(const mkq_bert_layer_params *p, mkq_bert_layer_workspace_layout *L)
{
    return layer_workspace(p, L, 4);
}

extern "C" int mkq_bert_layer_int8_workspace(const mkq_bert_layer_params *p, mkq_bert_layer_workspace_layout *L)
{
    return layer_workspace(p, L, 8);
}

// One linear of the layer at either width: codes in, `out` of out_dtype.
static int layer_linear(int bits, const uint8_t *codes, float s_x, const uint8_t *Wq, const float *s_w,
                        const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                        const mkq_epilogue *e, void *stream)
{
    if (bits == 8)
        return mkq_linear_int8((const int8_t *)codes, s_x, (const int8_t *)Wq, s_w, bias, M, N, K, out, out_dtype, e,
                               stream);
    return mkq_linear_int4(codes, MKQ_I4, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, e, nullptr, 0, stream);
}

static int bert_layer_run(int bits, const mkq_bert_layer_params *p, const void *h_in, int h_dtype,
                          const uint8_t *q_in, void *h_out, uint8_t *q_out_next, void *workspace,
                          size_t workspace_bytes, void *stream)
{
    if (!p) return MKQ_ERR_NULL;
    mkq_bert_layer_workspace_layout L;
    int rc = layer_workspace(p, &L, bits);
    if (rc != MKQ_OK) return rc;
    if (h_dtype != MKQ_F16 && h_dtype != MKQ_F32) return MKQ_ERR_DTYPE;
    if (!scale_ok(p->sx_qkv) || !scale_ok(p->sx_ao) || !scale_ok(p->sx_up) || !scale_ok(p->sx_down))
        return MKQ_ERR_SCALE;
    const bool want_next = p->s_out_next > 0.0f;
    if (want_next && !scale_ok(p->s_out_next)) return MKQ_ERR_SCALE;
    if (p->next_bits != 0 && p->next_bits != 4 && p->next_bits != 8) return MKQ_ERR_DTYPE;
    const int next_bits = p->next_bits ? p->next_bits : bits;
    if (p->batch == 0 || layer_tokens(p) == 0) return MKQ_OK;
    if (!h_in || !h_out || (want_next && !q_out_next)) return MKQ_ERR_NULL;
    if (!p->Wq_qkv || !p->Wq_ao || !p->Wq_up || !p->Wq_down || !p->sw_qkv || !p->sw_ao || !p->sw_up ||
        !p->sw_down)
        return MKQ_ERR_NULL;
    if (!p->ln1_gamma || !p->ln1_beta || !p->ln2_gamma || !p->ln2_beta) return MKQ_ERR_NULL;
    // every pointer the sub-steps will check, checked here: nothing is enqueued for a call that fails
    const void *const ptrs[] = {h_in, h_out, q_in, q_out_next, p->Wq_qkv, p->Wq_ao, p->Wq_up, p->Wq_down,
                                p->sw_qkv, p->sw_ao, p->sw_up, p->sw_down, p->b_qkv, p->b_ao, p->b_up, p->b_down,
                                p->ln1_gamma, p->ln1_beta, p->ln2_gamma, p->ln2_beta};
    for (const void *q : ptrs)
        if (q && !aligned16(q)) return MKQ_ERR_ALIGN;
    if (reinterpret_cast<uintptr_t>(p->cu_seqlens) & 3u) return MKQ_ERR_ALIGN;
    if (!workspace || workspace_bytes < L.total || !aligned16(workspace)) return MKQ_ERR_WORKSPACE;

    const int64_t M = layer_tokens(p), H = p->hidden, F = p->ffn;
    // rows of the code buffers: hidden / ffn, padded where the 4-bit linear that reads them needs it
    const int64_t Hp = code_row(bits, H), Fp = code_row(bits, F);
    const int64_t next_pitch = want_next ? code_row(next_bits, H) : H;
    if (next_bits == 8 && (H % 64) != 0) return MKQ_ERR_SHAPE;  // the 8-bit layer that would read them
    const int code_dtype = bits == 8 ? MKQ_I8 : MKQ_I4;
    uint8_t *ws = (uint8_t *)workspace;
    // (every writer of codes -- quantizer, attention, LayerNorm, the FFN-up epilogue -- fills the padding
    // columns of its rows with zero codes itself)
    const uint8_t *c0 = q_in;
    if (!c0) {
        rc = bits == 8   ? mkq_quantize_int8(h_in, h_dtype, M, H, H, p->sx_qkv, (int8_t *)(ws + L.c0), stream)
             : Hp != H ? mkq_quantize_padded(h_in, h_dtype, M, H, H, p->sx_qkv, ws + L.c0, stream)
                       : mkq_quantize(h_in, h_dtype, M, H, H, p->sx_qkv, ws + L.c0, stream);
        if (rc != MKQ_OK) return rc;
        c0 = ws + L.c0;
    }
    // q | k | v
    rc = layer_linear(bits, c0, p->sx_qkv, p->Wq_qkv, p->sw_qkv, p->b_qkv, M, 3 * H, Hp, ws + L.qkv, MKQ_F16,
                      nullptr, stream);
    if (rc != MKQ_OK) return rc;
    // attention context, re-quantized for the output projection
    rc = attention_run(ws + L.qkv, p->batch, p->seq, H, p->heads, nullptr, p->sx_ao, ws + L.c1, bits, stream,
                       p->cu_seqlens, Hp);
    if (rc != MKQ_OK) return rc;
    mkq_epilogue e = {};
    e.act = MKQ_ACT_NONE; e.residual = h_in; e.residual_dtype = h_dtype; e.s_next = 0.0f;
    e.q_out = nullptr; e.acc_out = nullptr;
    rc = layer_linear(bits, ws + L.c1, p->sx_ao, p->Wq_ao, p->sw_ao, p->b_ao, M, H, Hp, ws + L.u, MKQ_F16, &e, stream);
    if (rc != MKQ_OK) return rc;
    rc = layernorm_run(ws + L.u, M, H, p->ln1_gamma, p->ln1_beta, p->ln_eps, ws + L.h1, p->sx_up, ws + L.c2, bits,
                       stream, Hp);
    if (rc != MKQ_OK) return rc;
    // FFN up: GELU and re-quantization fused, only codes leave the kernel
    e.act = MKQ_ACT_GELU; e.residual = nullptr; e.s_next = p->sx_down; e.q_pitch = Fp != F ? Fp : 0;
    rc = layer_linear(bits, ws + L.c2, p->sx_up, p->Wq_up, p->sw_up, p->b_up, M, F, Hp, ws + L.c3, code_dtype, &e,
                      stream);
    if (rc != MKQ_OK) return rc;
    e.act = MKQ_ACT_NONE; e.residual = ws + L.h1; e.residual_dtype = MKQ_F16; e.s_next = 0.0f; e.q_pitch = 0;
    rc = layer_linear(bits, ws + L.c3, p->sx_down, p->Wq_down, p->sw_down, p->b_down, M, H, Fp, ws + L.d, MKQ_F16, &e,
                      stream);
    if (rc != MKQ_OK) return rc;
    return layernorm_run(ws + L.d, M, H, p->ln2_gamma, p->ln2_beta, p->ln_eps, h_out,
                         want_next ? p->s_out_next : 1.0f, want_next ? q_out_next : nullptr, next_bits, stream,
                         next_pitch);
}

extern "C" int mkq_bert_layer_int4(const mkq_bert_layer_params *p, const void *h_in, int h_dtype,
                                   const uint8_t *q_in, void *h_out, uint8_t *q_out_next, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    return bert_layer_run(4, p, h_in, h_dtype, q_in, h_out, q_out_next, workspace, workspace_bytes, stream);
}

extern "C" int mkq_bert_layer_int8(const mkq_bert_layer_params *p, const void *h_in, int h_dtype,
                                   const int8_t *q_in, void *h_out, int8_t *q_out_next, void *workspace,
                                   size_t workspace_bytes, void *stream)
{
    return bert_layer_run(8, p, h_in, h_dtype, (const uint8_t *)q_in, h_out, (uint8_t *)q_out_next, workspace,
                          workspace_bytes, stream);
}

extern "C" size_t mkq_bert_layer_fp16_workspace_bytes(const mkq_bert_layer_params_fp16 *p)
{
    if (!p || check_layer_dims(16, p->batch, p->seq, p->hidden, p->heads, p->ffn, p->cu_seqlens != nullptr,
                               p->total_tokens) != MKQ_OK)
        return 0;
    const size_t M = (size_t)layer_tokens(p), H = (size_t)p->hidden, F = (size_t)p->ffn;
    return align256(M * 3 * H * 2) + 4 * align256(M * H * 2) + align256(M * F * 2);
}

extern "C" int mkq_bert_layer_fp16(const mkq_bert_layer_params_fp16 *p, const void *h_in, void *h_out,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!p) return MKQ_ERR_NULL;
    const int rc0 = check_layer_dims(16, p->batch, p->seq, p->hidden, p->heads, p->ffn, p->cu_seqlens != nullptr,
                                     p->total_tokens);
    if (rc0 != MKQ_OK) return rc0;
    if (p->batch == 0 || layer_tokens(p) == 0) return MKQ_OK;
    if (!h_in || !h_out || !p->W_qkv || !p->W_ao || !p->W_up || !p->W_down) return MKQ_ERR_NULL;
    const size_t need = mkq_bert_layer_fp16_workspace_bytes(p);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return MKQ_ERR_WORKSPACE;
    const int64_t M = layer_tokens(p), H = p->hidden, F = p->ffn;
    uint8_t *ws = (uint8_t *)workspace;
    size_t o = 0;
    uint8_t *qkv = ws + o; o += align256((size_t)M * 3 * H * 2);
    uint8_t *ctx = ws + o; o += align256((size_t)M * H * 2);
    uint8_t *u = ws + o;   o += align256((size_t)M * H * 2);
    uint8_t *h1 = ws + o;  o += align256((size_t)M * H * 2);
    uint8_t *d = ws + o;   o += align256((size_t)M * H * 2);
    uint8_t *g = ws + o;
    int rc = mkq_linear_fp16(h_in, p->W_qkv, p->b_qkv, M, 3 * H, H, qkv, MKQ_F16, MKQ_ACT_NONE, nullptr, stream);
    if (rc != MKQ_OK) return rc;
    rc = attention_run(qkv, p->batch, p->seq, H, p->heads, ctx, 1.0f, nullptr, 4, stream, p->cu_seqlens);
    if (rc != MKQ_OK) return rc;
    rc = mkq_linear_fp16(ctx, p->W_ao, p->b_ao, M, H, H, u, MKQ_F16, MKQ_ACT_NONE, h_in, stream);
    if (rc != MKQ_OK) return rc;
    rc = mkq_layernorm(u, M, H, p->ln1_gamma, p->ln1_beta, p->ln_eps, h1, 1.0f, nullptr, stream);
    if (rc != MKQ_OK) return rc;
    rc = mkq_linear_fp16(h1, p->W_up, p->b_up, M, F, H, g, MKQ_F16, MKQ_ACT_GELU, nullptr, stream);
    if (rc != MKQ_OK) return rc;
    rc = mkq_linear_fp16(g, p->W_down, p->b_down, M, H, F, d, MKQ_F16, MKQ_ACT_NONE, h1, stream);
    if (rc != MKQ_OK) return rc;
    return mkq_layernorm(d, M, H, p->ln2_gamma, p->ln2_beta, p->ln_eps, h_out, 1.0f, nullptr, stream);
}
