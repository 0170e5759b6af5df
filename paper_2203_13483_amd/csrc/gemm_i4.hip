// int4 x int4 -> int32 GEMM with fused dequantize / activation / requantize
// epilogue for gfx950 (CDNA4), the hot loop of the W4A4 linear layer.
//
// CDNA4 has no 4-bit integer MFMA, so nibbles are widened to int8 on the way from
// LDS to the matrix core.  The widening used here costs three VALU ops per eight
// codes: for a 32-bit word w of eight two's-complement nibbles,
//     hi = w & 0xF0F0F0F0          -> four int8 lanes equal to 16 * (odd codes)
//     lo = (w << 4) & 0xF0F0F0F0   -> four int8 lanes equal to 16 * (even codes)
// (the nibble's sign bit lands in bit 7 of its byte).  Both operands carry the
// factor 16, so the int32 accumulator holds exactly 256 * sum(a*w) and the true
// sum is recovered with an arithmetic shift by 8.  |sum| <= 64 K, so this is exact
// while 256 * 64 * K < 2^31, i.e. K < 131072.  The lo/hi split permutes k inside
// a word identically for both operands, which a dot product does not see.
//
// Data flow: packed rows of A [M, K/2] and W [N, K/2] (both K-contiguous) are
// copied by 128-bit loads into LDS tiles of RB bytes per row, XOR-swizzled at
// 16-byte granularity so that both the staging writes and the ds_read_b128
// fragment reads are bank-conflict free; each lane reads 16 bytes (32 codes) of
// one row and feeds two v_mfma_i32_16x16x64_i8.  W is the MFMA "A" operand and the
// activations the "B" operand, so a lane ends up with four consecutive output
// channels of one token and stores them as one vector.
#include "mkq_internal.h"

namespace mkq {

typedef int v4i __attribute__((ext_vector_type(4)));

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

// 16-byte-chunk swizzle for a row of CH chunks; r = row % 16.  Chosen so that any
// 8 or 16 consecutive lanes of a fragment read (same chunk, 16 rows) and of a
// staging write (consecutive chunks of consecutive rows) hit distinct bank groups.
template <int CH>
__device__ __forceinline__ int swz(int r);
template <>
__device__ __forceinline__ int swz<4>(int r) { return ((r >> 2) ^ (r & 2)) & 3; }
template <>
__device__ __forceinline__ int swz<8>(int r) { return ((r & 7) ^ (r >> 3)) & 7; }

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
    static constexpr int WTM = BM / WGM, WTN = BN / WGN;  // per-wave tile
    static constexpr int TM = WTM / 16, TN = WTN / 16;    // 16x16 MFMA tiles per wave
    static constexpr int CH = RB / 16;                    // 16-byte chunks per LDS row
    static constexpr int READS = RB / 64;                 // ds_read_b128 per fragment per stage
    static constexpr int STAGE_BYTES = (BM + BN) * RB;
    static constexpr int A_CHUNKS = BM * CH, W_CHUNKS = BN * CH;
    static constexpr int A_PER_T = A_CHUNKS / THREADS, W_PER_T = W_CHUNKS / THREADS;
    static_assert(A_CHUNKS % THREADS == 0 && W_CHUNKS % THREADS == 0, "tile/threads mismatch");
    static_assert(WTM % 16 == 0 && WTN % 16 == 0, "wave tile must be a multiple of 16");
};

template <class Cfg>
__global__ __launch_bounds__(Cfg::THREADS) void gemm_i4_kernel(const GemmI4Params p)
{
    constexpr int BM = Cfg::BM, BN = Cfg::BN, RB = Cfg::RB, CH = Cfg::CH;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, READS = Cfg::READS;
    constexpr int THREADS = Cfg::THREADS;

    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / Cfg::WGN, wn = wave % Cfg::WGN;
    const int lr = lane & 15;  // row inside a 16-row fragment
    const int lg = lane >> 4;  // 16-byte chunk (k group) inside a 64-byte slice

    const int tiles_n = (p.N + BN - 1) / BN;
    const int tile_m = blockIdx.x / tiles_n;
    const int tile_n = blockIdx.x - tile_m * tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int64_t row_bytes = p.K / 2;
    const int kt_count = (int)((row_bytes + RB - 1) / RB);

    // --- staging: which chunks this thread copies each stage ------------------
    uint4 ra[Cfg::A_PER_T], rw[Cfg::W_PER_T];
    const uint8_t *ga[Cfg::A_PER_T];
    const uint8_t *gw[Cfg::W_PER_T];
    int sa[Cfg::A_PER_T], sw[Cfg::W_PER_T], ca[Cfg::A_PER_T], cw[Cfg::W_PER_T];
#pragma unroll
    for (int i = 0; i < Cfg::A_PER_T; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / CH, c = idx % CH;
        int gm = m0 + row;
        gm = gm < p.M ? gm : p.M - 1;  // rows past the edge re-read the last row; never stored
        ga[i] = p.A + (int64_t)gm * row_bytes + c * 16;
        ca[i] = c * 16;
        sa[i] = row * RB + ((c ^ swz<CH>(row & 15)) * 16);
    }
#pragma unroll
    for (int i = 0; i < Cfg::W_PER_T; ++i) {
        const int idx = tid + i * THREADS;
        const int row = idx / CH, c = idx % CH;
        int gn = n0 + row;
        gn = gn < p.N ? gn : p.N - 1;
        gw[i] = p.W + (int64_t)gn * row_bytes + c * 16;
        cw[i] = c * 16;
        sw[i] = BM * RB + row * RB + ((c ^ swz<CH>(row & 15)) * 16);
    }

    auto load_stage = [&](int kt) {
        const int64_t kb = (int64_t)kt * RB;
#pragma unroll
        for (int i = 0; i < Cfg::A_PER_T; ++i)
            ra[i] = (kb + ca[i] < row_bytes) ? *reinterpret_cast<const uint4 *>(ga[i] + kb)
                                             : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < Cfg::W_PER_T; ++i)
            rw[i] = (kb + cw[i] < row_bytes) ? *reinterpret_cast<const uint4 *>(gw[i] + kb)
                                             : make_uint4(0, 0, 0, 0);
    };
    auto store_stage = [&](int buf) {
        uint8_t *base = smem + buf * Cfg::STAGE_BYTES;
#pragma unroll
        for (int i = 0; i < Cfg::A_PER_T; ++i) *reinterpret_cast<uint4 *>(base + sa[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < Cfg::W_PER_T; ++i) *reinterpret_cast<uint4 *>(base + sw[i]) = rw[i];
    };

    v4i acc[TM][TN];
#pragma unroll
    for (int j = 0; j < TM; ++j)
#pragma unroll
        for (int i = 0; i < TN; ++i) acc[j][i] = (v4i){0, 0, 0, 0};

    // fragment read offsets (bytes inside a stage), per ds_read_b128 r
    int offA[TM], offW[TN];
#pragma unroll
    for (int j = 0; j < TM; ++j) offA[j] = (wm * Cfg::WTM + j * 16 + lr) * RB;
#pragma unroll
    for (int i = 0; i < TN; ++i) offW[i] = BM * RB + (wn * Cfg::WTN + i * 16 + lr) * RB;
    const int sz = swz<CH>(lr);

    load_stage(0);
    store_stage(0);
    __syncthreads();

    for (int kt = 0; kt < kt_count; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < kt_count) load_stage(kt + 1);

        const uint8_t *base = smem + buf * Cfg::STAGE_BYTES;
#pragma unroll
        for (int r = 0; r < READS; ++r) {
            const int coff = ((r * 4 + lg) ^ sz) * 16;
            uint4 fw[TN], fa[TM];
#pragma unroll
            for (int i = 0; i < TN; ++i) fw[i] = *reinterpret_cast<const uint4 *>(base + offW[i] + coff);
#pragma unroll
            for (int j = 0; j < TM; ++j) fa[j] = *reinterpret_cast<const uint4 *>(base + offA[j] + coff);
            v4i w0[TN], w1[TN], a0[TM], a1[TM];
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                w0[i] = widen(fw[i].x, fw[i].y);
                w1[i] = widen(fw[i].z, fw[i].w);
            }
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                a0[j] = widen(fa[j].x, fa[j].y);
                a1[j] = widen(fa[j].z, fa[j].w);
            }
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w0[i], a0[j], acc[j][i], 0, 0, 0);
                    acc[j][i] = __builtin_amdgcn_mfma_i32_16x16x64_i8(w1[i], a1[j], acc[j][i], 0, 0, 0);
                }
        }

        if (kt + 1 < kt_count) store_stage(buf ^ 1);
        __syncthreads();
    }

    // --- epilogue ---------------------------------------------------------------
    // MFMA result layout: lane holds D[4*(lane/16) + v][lane%16], v = 0..3, with D
    // rows = output channels (W rows) and D columns = tokens (A rows).
    const bool vec_ok = (p.N % 4) == 0;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m0 + wm * Cfg::WTM + j * 16 + lr;
        if (m >= p.M) continue;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int nb = n0 + wn * Cfg::WTN + i * 16 + lg * 4;
            if (nb >= p.N) continue;
            const int64_t o = (int64_t)m * p.N + nb;
            const int nvalid = (p.N - nb) < 4 ? (p.N - nb) : 4;
            int a[4];
            a[0] = acc[j][i].x >> 8; a[1] = acc[j][i].y >> 8;
            a[2] = acc[j][i].z >> 8; a[3] = acc[j][i].w >> 8;

            if (p.acc_out) {
                if (vec_ok) *reinterpret_cast<int4 *>(p.acc_out + o) = make_int4(a[0], a[1], a[2], a[3]);
                else for (int v = 0; v < nvalid; ++v) p.acc_out[o + v] = a[v];
            }
            if (p.out_dtype < 0 && !p.q_out) continue;

            float y[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int n = (nb + v < p.N) ? nb + v : p.N - 1;
                const float scale = p.s_x * p.s_w[n];
                y[v] = __fmaf_rn((float)a[v], scale, p.bias ? p.bias[n] : 0.0f);
            }
            if (p.residual) {
                if (p.residual_dtype == MKQ_F32) {
                    const float *r = (const float *)p.residual + o;
                    for (int v = 0; v < nvalid; ++v) y[v] = y[v] + r[v];
                } else {
                    const uint16_t *r = (const uint16_t *)p.residual + o;
                    for (int v = 0; v < nvalid; ++v) y[v] = y[v] + half_bits_to_float(r[v]);
                }
            }
            if (p.act == MKQ_ACT_GELU) {
#pragma unroll
                for (int v = 0; v < 4; ++v) y[v] = gelu_erf(y[v]);
            }

            if (p.out_dtype == MKQ_F32) {
                float *dst = (float *)p.out + o;
                if (vec_ok) *reinterpret_cast<float4 *>(dst) = make_float4(y[0], y[1], y[2], y[3]);
                else for (int v = 0; v < nvalid; ++v) dst[v] = y[v];
            } else if (p.out_dtype == MKQ_F16 || p.out_dtype == MKQ_BF16) {
                uint16_t h[4];
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    h[v] = (p.out_dtype == MKQ_F16) ? float_to_half_bits(y[v]) : float_to_bf16_bits(y[v]);
                uint16_t *dst = (uint16_t *)p.out + o;
                if (vec_ok)
                    *reinterpret_cast<uint2 *>(dst) =
                        make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
                else for (int v = 0; v < nvalid; ++v) dst[v] = h[v];
            }
            if (p.out_dtype == MKQ_I4 || p.q_out) {
                // Eq. 1 on the binary32 value; N is even here, nb is a multiple of 4
                uint32_t packed = 0;
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    packed |= ((uint32_t)quantize_code(y[v], p.s_next) & 0xFu) << (4 * v);
                uint8_t *qdst = (p.out_dtype == MKQ_I4 ? (uint8_t *)p.out : p.q_out) + (o >> 1);
                // N even and nb % 4 == 0, so nvalid is 2 or 4 and o is even
                if (nvalid == 4 && (o & 2) == 0) {
                    *reinterpret_cast<uint16_t *>(qdst) = (uint16_t)packed;
                } else {
                    qdst[0] = (uint8_t)packed;
                    if (nvalid == 4) qdst[1] = (uint8_t)(packed >> 8);
                }
            }
        }
    }
}

template <class Cfg>
static int launch_gemm_i4(const GemmI4Params &p, hipStream_t st)
{
    const int64_t tiles = ceil_div(p.M, Cfg::BM) * ceil_div(p.N, Cfg::BN);
    if (tiles > 0x7FFFFFFF) return MKQ_ERR_UNSUPPORTED;
    const size_t lds = 2 * (size_t)Cfg::STAGE_BYTES;
    gemm_i4_kernel<Cfg><<<(unsigned)tiles, Cfg::THREADS, lds, st>>>(p);
    return launch_status();
}

int run_gemm_i4(const GemmI4Params &p, hipStream_t st)
{
    // tile choice: the largest tile that still yields enough workgroups for 256 CUs
    const int64_t t128 = ceil_div(p.M, 128) * ceil_div(p.N, 128);
    if (t128 >= 256) return launch_gemm_i4<GemmI4Cfg<128, 128, 2, 2, 64>>(p, st);
    return launch_gemm_i4<GemmI4Cfg<64, 64, 2, 2, 64>>(p, st);
}

}  // namespace mkq

using namespace mkq;

extern "C" int mkq_quantize(const void *, int, int64_t, int64_t, int64_t, float, uint8_t *, void *);

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
    if (!aligned16(a) || !aligned16(Wq) || (out && !aligned16(out)) ||
        (reinterpret_cast<uintptr_t>(s_w) & 3u) || (reinterpret_cast<uintptr_t>(bias) & 3u))
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
