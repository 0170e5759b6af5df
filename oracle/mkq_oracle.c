/*
 * mkq_oracle.c -- CPU oracle for the W4A4 quantized BERT linear layer of MKQ-BERT.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * GPU library must compute.  It shares no code with the HIP path, is never loaded
 * by the product, and is only called from tests, the smoke check and the
 * cpu_baseline leg of the benchmark.
 *
 * Everything is written as the definition reads: unpacked int8 codes, scalar
 * loops, no blocking, no packing tricks.  OpenMP only spreads independent output
 * rows over cores.  Build with -ffp-contract=off so that the only fused
 * multiply-add is the one spelled fmaf() below.
 *
 * Precision: the quantizer decision and the dequantize epilogue are defined in
 * IEEE binary32 (one correctly rounded divide / one multiply / one fma) so that
 * an integer code decided from a float is decided in the same precision on both
 * sides.  LayerNorm, softmax and GELU are evaluated in binary64 and rounded once
 * to binary32 (the paper keeps them in float32; the oracle gives the best
 * float32 answer).
 *
 * Readings of the paper taken here (section 3.1, Eq. 1 unless noted):
 *   - clamp range for k=4 is the signed nibble range [-8, 7]; the printed
 *     (-2^{k-1}+1, 2^{k-1}) is read as a sign slip.  MKQ_QMIN/MKQ_QMAX are
 *     parameters of every function so the tests can exercise other ranges.
 *   - round() is round-half-to-even.
 *   - clamp is applied before round, as printed in Eq. 1.
 *   - x/s is a true division.
 *   - a "row" of a weight matrix stored [N,K] is one output channel.
 *   - abs-max calibration (section 3.1, third paragraph) divides by qmax.
 *   - attention scores are q k^T / sqrt(d_k) (the printed q v^T is a typo: k is
 *     defined and otherwise unused), section 3.2.
 *   - residual connections and LayerNorm follow the standard post-LN BERT layer;
 *     the paper only says LayerNorm is kept in float32 (section 5).
 *   - GELU is the erf form.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define MKQ_REF_OK 0
#define MKQ_REF_ERR_NULL (-1)
#define MKQ_REF_ERR_SHAPE (-2)
#define MKQ_REF_ERR_SCALE (-4)

/* ------------------------------------------------------------------------- */
/* Eq. 1, integer part: code = round(clamp(x / s, qmin, qmax)).               */
/* NaN maps to code 0 (paper silent).                                          */
static inline int8_t quantize_one(float x, float s, int qmin, int qmax)
{
    float v = x / s;
    if (v != v) return 0;
    if (v < (float)qmin) v = (float)qmin;
    if (v > (float)qmax) v = (float)qmax;
    return (int8_t)nearbyintf(v); /* default rounding mode: nearest, ties to even */
}

static int scale_ok(float s) { return s > 0.0f && s < INFINITY; }

/* Quantize a [M,K] matrix with leading dimension ldx to unpacked int8 codes [M,K]
 * using one scale for the whole tensor (per-tensor scale, section 3.1). */
int mkq_ref_quantize(const float *x, int64_t M, int64_t K, int64_t ldx, float s,
                     int qmin, int qmax, int8_t *codes)
{
    if (!x || !codes) return MKQ_REF_ERR_NULL;
    if (M < 0 || K < 0 || ldx < K) return MKQ_REF_ERR_SHAPE;
    if (!scale_ok(s)) return MKQ_REF_ERR_SCALE;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k)
            codes[m * K + k] = quantize_one(x[m * ldx + k], s, qmin, qmax);
    return MKQ_REF_OK;
}

/* Eq. 1, full: Q[x] = s * code. */
int mkq_ref_dequantize(const int8_t *codes, int64_t n, float s, float *out)
{
    if (!codes || !out) return MKQ_REF_ERR_NULL;
    for (int64_t i = 0; i < n; ++i) out[i] = s * (float)codes[i];
    return MKQ_REF_OK;
}

/* Abs-max calibration: s = max|x| / qmax, per tensor (one value) or per row
 * (M values).  An all-zero tensor/row gets s = 1 (paper silent). */
int mkq_ref_absmax_scale(const float *x, int64_t M, int64_t K, int64_t ldx,
                         int per_row, int qmax, float *s_out)
{
    if (!x || !s_out) return MKQ_REF_ERR_NULL;
    if (M < 0 || K < 0 || ldx < K) return MKQ_REF_ERR_SHAPE;
    float tmax = 0.0f;
    for (int64_t m = 0; m < M; ++m) {
        float rmax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            float a = fabsf(x[m * ldx + k]);
            if (a > rmax) rmax = a; /* NaN never wins the comparison */
        }
        if (per_row) s_out[m] = (rmax > 0.0f) ? rmax / (float)qmax : 1.0f;
        if (rmax > tmax) tmax = rmax;
    }
    if (!per_row) s_out[0] = (tmax > 0.0f) ? tmax / (float)qmax : 1.0f;
    return MKQ_REF_OK;
}

/* Percentile calibration of an activation step (section 3.1, third paragraph: sampled
 * activations' absolute values are ranked and the value at the top 0.01 % becomes the
 * initial clipping point).  Reading: T = the k-th largest of |x_i| with
 * k = max(1, floor(n * top_ppm / 10^6)) (top_ppm = 100 for 0.01 %), s = T / qmax, and
 * s = 1 when T = 0.  NaN counts as 0.  Written as the definition: sort, then index. */
static int cmp_float_asc(const void *a, const void *b)
{
    float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

int mkq_ref_percentile_scale(const float *x, int64_t n, int64_t top_ppm, int qmax, float *s_out,
                             float *t_out)
{
    if (!x || !s_out) return MKQ_REF_ERR_NULL;
    if (n <= 0 || top_ppm < 0 || top_ppm > 1000000 || qmax <= 0) return MKQ_REF_ERR_SHAPE;
    float *a = (float *)malloc(sizeof(float) * (size_t)n);
    if (!a) return MKQ_REF_ERR_NULL;
    for (int64_t i = 0; i < n; ++i) {
        float v = fabsf(x[i]);
        a[i] = (v != v) ? 0.0f : v;
    }
    qsort(a, (size_t)n, sizeof(float), cmp_float_asc);
    int64_t k = n * top_ppm / 1000000;
    if (k < 1) k = 1;
    const float T = a[n - k];
    free(a);
    if (t_out) *t_out = T;
    *s_out = (T > 0.0f) ? T / (float)qmax : 1.0f;
    return MKQ_REF_OK;
}

/* Per-row (per output channel) weight quantization.  If s_w_in is NULL the
 * scales come from abs-max calibration, otherwise they are taken as given. */
int mkq_ref_quantize_weights(const float *W, int64_t N, int64_t K,
                             const float *s_w_in, int qmin, int qmax,
                             float *s_w_out, int8_t *codes)
{
    if (!W || !s_w_out || !codes) return MKQ_REF_ERR_NULL;
    if (N < 0 || K < 0) return MKQ_REF_ERR_SHAPE;
    if (s_w_in) {
        for (int64_t n = 0; n < N; ++n) {
            if (!scale_ok(s_w_in[n])) return MKQ_REF_ERR_SCALE;
            s_w_out[n] = s_w_in[n];
        }
    } else {
        int rc = mkq_ref_absmax_scale(W, N, K, K, 1, qmax, s_w_out);
        if (rc) return rc;
    }
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k)
            codes[n * K + k] = quantize_one(W[n * K + k], s_w_out[n], qmin, qmax);
    return MKQ_REF_OK;
}

/* Canonical nibble packing (the paper gives none; this is the library's
 * interchange format): element k of a row is the low nibble of byte k/2 when k
 * is even and the high nibble when k is odd, two's complement. */
int mkq_ref_pack_nibbles(const int8_t *codes, int64_t rows, int64_t K, uint8_t *out)
{
    if (!codes || !out) return MKQ_REF_ERR_NULL;
    if (rows < 0 || K < 0 || (K & 1)) return MKQ_REF_ERR_SHAPE;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            unsigned lo = (unsigned)codes[r * K + 2 * j] & 0xFu;
            unsigned hi = (unsigned)codes[r * K + 2 * j + 1] & 0xFu;
            out[r * (K / 2) + j] = (uint8_t)(lo | (hi << 4));
        }
    return MKQ_REF_OK;
}

int mkq_ref_unpack_nibbles(const uint8_t *packed, int64_t rows, int64_t K, int8_t *codes)
{
    if (!packed || !codes) return MKQ_REF_ERR_NULL;
    if (rows < 0 || K < 0 || (K & 1)) return MKQ_REF_ERR_SHAPE;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t j = 0; j < K / 2; ++j) {
            int lo = packed[r * (K / 2) + j] & 0xF;
            int hi = packed[r * (K / 2) + j] >> 4;
            codes[r * K + 2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            codes[r * K + 2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
    return MKQ_REF_OK;
}

/* The integer matrix product of the quantized linear layer (x W of section 3.2
 * with both operands replaced by their codes):
 *   acc[m,n] = sum_k a[m,k] * w[n,k], exact in int32. */
int mkq_ref_gemm_codes(const int8_t *a, const int8_t *w, int64_t M, int64_t N,
                       int64_t K, int32_t *acc)
{
    if (!a || !w || !acc) return MKQ_REF_ERR_NULL;
    if (M < 0 || N < 0 || K < 0) return MKQ_REF_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int32_t sum = 0;
            for (int64_t k = 0; k < K; ++k)
                sum += (int32_t)a[m * K + k] * (int32_t)w[n * K + k];
            acc[m * N + n] = sum;
        }
    return MKQ_REF_OK;
}

/* GELU(x) = x/2 (1 + erf(x / sqrt 2)), evaluated in binary64, rounded once. */
static inline float gelu_f32(float x)
{
    double d = (double)x;
    return (float)(0.5 * d * (1.0 + erf(d * 0.70710678118654752440)));
}

/* Dequantize epilogue: Q[x] Q[w] summed over k equals acc * s_x * s_w[n]
 * (both factors of Eq. 1 pulled out of the sum), then the layer's bias
 * (section 3.2), optional residual, optional GELU (FFN, section 3.2):
 *   scale = s_x * s_w[n]            one binary32 multiply
 *   y     = fma((float)acc, scale, bias[n])
 *   y    += residual[m,n]           (if given)
 *   y     = gelu(y)                 (if act == 1)
 * (float)acc is exact: |acc| <= 64 K. */
int mkq_ref_epilogue(const int32_t *acc, int64_t M, int64_t N, float s_x,
                     const float *s_w, const float *bias, const float *residual,
                     int act, float *y)
{
    if (!acc || !s_w || !y) return MKQ_REF_ERR_NULL;
    if (M < 0 || N < 0) return MKQ_REF_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_REF_ERR_SCALE;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            float scale = s_x * s_w[n];
            float v = fmaf((float)acc[m * N + n], scale, bias ? bias[n] : 0.0f);
            if (residual) v = v + residual[m * N + n];
            if (act == 1) v = gelu_f32(v);
            y[m * N + n] = v;
        }
    return MKQ_REF_OK;
}

/* ------------------------------------------------------------------------- */
/* Narrowing to the 16-bit storage formats, round-to-nearest-even, returned as
 * the binary32 value that the narrow number represents.                       */
static inline float round_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) { /* Inf/NaN: keep class */
        if (u & 0x007FFFFFu) u |= 0x00400000u;
        u &= 0xFFFF0000u;
    } else {
        uint32_t lsb = (u >> 16) & 1u;
        u += 0x7FFFu + lsb;
        u &= 0xFFFF0000u;
    }
    memcpy(&f, &u, 4);
    return f;
}

static inline float round_to_f16(float f)
{
    /* binary16: 10 fraction bits, exponent range [-14, 15], subnormal step 2^-24.
     * Work on the magnitude in binary64 (every binary32 is exact there). */
    if (f != f) return f;
    double a = fabs((double)f);
    double r;
    if (a >= 65520.0) { /* halfway between max finite 65504 and 2^16 rounds to Inf */
        r = INFINITY;
    } else if (a < 6.103515625e-05) { /* below 2^-14: fixed step 2^-24 */
        r = nearbyint(a * 16777216.0) / 16777216.0;
    } else {
        int e;
        frexp(a, &e); /* a = m * 2^e, m in [0.5, 1) */
        double step = ldexp(1.0, e - 11); /* 11 significant bits */
        r = nearbyint(a / step) * step;
    }
    return (float)(f < 0 ? -r : r);
}

/* dtype: 0 = binary32 (identity), 1 = binary16, 2 = bfloat16 */
int mkq_ref_round_storage(float *x, int64_t n, int dtype)
{
    if (!x) return MKQ_REF_ERR_NULL;
    if (dtype == 0) return MKQ_REF_OK;
    for (int64_t i = 0; i < n; ++i)
        x[i] = (dtype == 1) ? round_to_f16(x[i]) : round_to_bf16(x[i]);
    return MKQ_REF_OK;
}

/* ------------------------------------------------------------------------- */
/* The whole quantized linear layer on float inputs:
 *   codes(x; s_x) x codes(W; s_w) -> acc -> epilogue -> optional requantization
 * with the next layer's step (Eq. 1 applied to the binary32 epilogue value,
 * before any narrowing).  Any output pointer may be NULL.
 *   a_codes [M,K], w_codes [N,K] : int8 codes (already quantized)
 *   acc_out [M,N] int32, y_out [M,N] float (narrowed to out_dtype),
 *   q_out [M,N] int8 codes of y under s_next, clamped to [qmin, qmax]. */
int mkq_ref_linear_int4(const int8_t *a_codes, float s_x, const int8_t *w_codes,
                        const float *s_w, const float *bias, int64_t M, int64_t N,
                        int64_t K, const float *residual, int act, int out_dtype,
                        float s_next, int qmin, int qmax, int32_t *acc_out, float *y_out,
                        int8_t *q_out)
{
    if (!a_codes || !w_codes || !s_w) return MKQ_REF_ERR_NULL;
    if (M < 0 || N < 0 || K < 0) return MKQ_REF_ERR_SHAPE;
    if (!scale_ok(s_x)) return MKQ_REF_ERR_SCALE;
    if (q_out && !scale_ok(s_next)) return MKQ_REF_ERR_SCALE;
    int32_t *acc = acc_out ? acc_out : (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * N));
    float *y = (float *)malloc(sizeof(float) * (size_t)(M * N));
    int rc = mkq_ref_gemm_codes(a_codes, w_codes, M, N, K, acc);
    if (!rc) rc = mkq_ref_epilogue(acc, M, N, s_x, s_w, bias, residual, act, y);
    if (!rc && q_out) rc = mkq_ref_quantize(y, M, N, N, s_next, qmin, qmax, q_out);
    if (!rc && y_out) {
        memcpy(y_out, y, sizeof(float) * (size_t)(M * N));
        mkq_ref_round_storage(y_out, M * N, out_dtype);
    }
    free(y);
    if (!acc_out) free(acc);
    return rc;
}

/* fp16 baseline linear: inputs are given as binary32 arrays that already hold
 * binary16-representable values; products summed in binary64. */
int mkq_ref_linear_float(const float *a, const float *W, const float *bias, int64_t M,
                         int64_t N, int64_t K, const float *residual, int act,
                         int out_dtype, float *y_out)
{
    if (!a || !W || !y_out) return MKQ_REF_ERR_NULL;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double sum = 0.0;
            for (int64_t k = 0; k < K; ++k) sum += (double)a[m * K + k] * (double)W[n * K + k];
            float v = (float)(sum + (bias ? (double)bias[n] : 0.0));
            if (residual) v = v + residual[m * N + n];
            if (act == 1) v = gelu_f32(v);
            y_out[m * N + n] = v;
        }
    return mkq_ref_round_storage(y_out, M * N, out_dtype);
}

/* LayerNorm over the last dimension, binary64 statistics, one rounding to
 * binary32 (section 5: LayerNorm is kept in float32). */
int mkq_ref_layernorm(const float *x, int64_t M, int64_t D, const float *gamma,
                      const float *beta, float eps, float *y)
{
    if (!x || !y) return MKQ_REF_ERR_NULL;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double mean = 0.0, var = 0.0;
        for (int64_t d = 0; d < D; ++d) mean += (double)x[m * D + d];
        mean /= (double)D;
        for (int64_t d = 0; d < D; ++d) {
            double c = (double)x[m * D + d] - mean;
            var += c * c;
        }
        var /= (double)D;
        double rstd = 1.0 / sqrt(var + (double)eps);
        for (int64_t d = 0; d < D; ++d) {
            double g = gamma ? (double)gamma[d] : 1.0;
            double b = beta ? (double)beta[d] : 0.0;
            y[m * D + d] = (float)(((double)x[m * D + d] - mean) * rstd * g + b);
        }
    }
    return MKQ_REF_OK;
}

/* Multi-head self-attention core (section 3.2): for every sequence b and head a,
 *   A = softmax(q k^T / sqrt(d_k)),  OA = A v
 * qkv is [B*S, 3*H] with q | k | v side by side, head a owning columns
 * [a*d_k, (a+1)*d_k) of each third.  Scores and softmax in binary64;
 * if p_dtype != 0 the probabilities are narrowed to that storage format before
 * multiplying v (the GPU feeds them to a 16-bit matrix unit).  Output [B*S, H]. */
int mkq_ref_attention(const float *qkv, int64_t B, int64_t S, int64_t H, int64_t heads,
                      int p_dtype, float *ctx)
{
    if (!qkv || !ctx) return MKQ_REF_ERR_NULL;
    if (heads <= 0 || H % heads) return MKQ_REF_ERR_SHAPE;
    const int64_t dk = H / heads;
    const double inv = 1.0 / sqrt((double)dk);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t a = 0; a < heads; ++a) {
            double *p = (double *)malloc(sizeof(double) * (size_t)S);
            for (int64_t i = 0; i < S; ++i) {
                const float *q = qkv + (b * S + i) * 3 * H + a * dk;
                double mx = -INFINITY;
                for (int64_t j = 0; j < S; ++j) {
                    const float *k = qkv + (b * S + j) * 3 * H + H + a * dk;
                    double s = 0.0;
                    for (int64_t d = 0; d < dk; ++d) s += (double)q[d] * (double)k[d];
                    p[j] = s * inv;
                    if (p[j] > mx) mx = p[j];
                }
                double den = 0.0;
                for (int64_t j = 0; j < S; ++j) {
                    p[j] = exp(p[j] - mx);
                    den += p[j];
                }
                for (int64_t j = 0; j < S; ++j) {
                    float pf = (float)(p[j] / den);
                    if (p_dtype == 1) pf = round_to_f16(pf);
                    else if (p_dtype == 2) pf = round_to_bf16(pf);
                    p[j] = (double)pf;
                }
                for (int64_t d = 0; d < dk; ++d) {
                    double o = 0.0;
                    for (int64_t j = 0; j < S; ++j)
                        o += p[j] * (double)qkv[(b * S + j) * 3 * H + 2 * H + a * dk + d];
                    ctx[(b * S + i) * H + a * dk + d] = (float)o;
                }
            }
            free(p);
        }
    return MKQ_REF_OK;
}

/* One post-LN BERT encoder layer with all six linears W4A4 (section 3.2 + 5).
 * Weights come as codes + per-channel scales; activations between kernels are
 * stored in `act_dtype` (0 = binary32, 1 = binary16).
 *
 *   c0  = codes(h; sx_qkv)
 *   qkv = store(Lin_qkv(c0))
 *   ctx = attention(qkv)                      (probabilities stored in act_dtype)
 *   c1  = codes(ctx; sx_ao)
 *   u   = store(Lin_ao(c1) + h)
 *   h1f = LN1(u);  h1 = store(h1f);  c2 = codes(h1f; sx_up)
 *   c3  = codes(GELU(Lin_up(c2)); sx_down)
 *   d   = store(Lin_down(c3) + h1)
 *   out = store(LN2(d))
 *
 * Intermediates are returned through the optional pointers of `dbg`
 * (any may be NULL) so that tests can compare stage by stage. */
typedef struct {
    int8_t *c0;      /* [M,H]   */
    float *qkv;      /* [M,3H]  */
    float *ctx;      /* [M,H] binary32, not narrowed */
    int8_t *c1;      /* [M,H]   */
    float *u;        /* [M,H]   */
    float *h1;       /* [M,H]   */
    int8_t *c2;      /* [M,H]   */
    int8_t *c3;      /* [M,F]   */
    float *d;        /* [M,H]   */
    float *g_pre;    /* [M,F] GELU output in binary32 before requantization */
} mkq_ref_layer_debug;

typedef struct {
    int64_t batch, seq, hidden, heads, ffn;
    const int8_t *w_qkv, *w_ao, *w_up, *w_down; /* codes [3H,H] [H,H] [F,H] [H,F] */
    const float *sw_qkv, *sw_ao, *sw_up, *sw_down;
    const float *b_qkv, *b_ao, *b_up, *b_down;
    float sx_qkv, sx_ao, sx_up, sx_down;
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    float ln_eps;
    int qmin, qmax; /* clamp range of every activation quantizer in the layer */
} mkq_ref_layer_params;

int mkq_ref_bert_layer_int4(const mkq_ref_layer_params *p, const float *h_in,
                            const int8_t *c0_given, int act_dtype, float *h_out,
                            mkq_ref_layer_debug *dbg)
{
    if (!p || !h_in || !h_out) return MKQ_REF_ERR_NULL;
    const int64_t M = p->batch * p->seq, H = p->hidden, F = p->ffn;
    const int lo = p->qmin, hi = p->qmax;
    int rc = 0;
    int8_t *c0 = (int8_t *)malloc((size_t)(M * H));
    int8_t *c1 = (int8_t *)malloc((size_t)(M * H));
    int8_t *c2 = (int8_t *)malloc((size_t)(M * H));
    int8_t *c3 = (int8_t *)malloc((size_t)(M * F));
    float *qkv = (float *)malloc(sizeof(float) * (size_t)(M * 3 * H));
    float *ctx = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *u = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *h1 = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *g = (float *)malloc(sizeof(float) * (size_t)(M * F));
    float *d = (float *)malloc(sizeof(float) * (size_t)(M * H));

    if (c0_given) memcpy(c0, c0_given, (size_t)(M * H));
    else rc = mkq_ref_quantize(h_in, M, H, H, p->sx_qkv, lo, hi, c0);
    if (!rc) rc = mkq_ref_linear_int4(c0, p->sx_qkv, p->w_qkv, p->sw_qkv, p->b_qkv, M, 3 * H, H,
                                      NULL, 0, act_dtype, 0.0f, lo, hi, NULL, qkv, NULL);
    if (!rc) rc = mkq_ref_attention(qkv, p->batch, p->seq, H, p->heads, act_dtype, ctx);
    if (!rc) rc = mkq_ref_quantize(ctx, M, H, H, p->sx_ao, lo, hi, c1);
    if (!rc) rc = mkq_ref_linear_int4(c1, p->sx_ao, p->w_ao, p->sw_ao, p->b_ao, M, H, H, h_in, 0,
                                      act_dtype, 0.0f, lo, hi, NULL, u, NULL);
    if (!rc) rc = mkq_ref_layernorm(u, M, H, p->ln1_gamma, p->ln1_beta, p->ln_eps, h1);
    if (!rc) rc = mkq_ref_quantize(h1, M, H, H, p->sx_up, lo, hi, c2);
    if (!rc) rc = mkq_ref_round_storage(h1, M * H, act_dtype);
    if (!rc) rc = mkq_ref_linear_int4(c2, p->sx_up, p->w_up, p->sw_up, p->b_up, M, F, H, NULL, 1,
                                      0, p->sx_down, lo, hi, NULL, g, c3);
    if (!rc) rc = mkq_ref_linear_int4(c3, p->sx_down, p->w_down, p->sw_down, p->b_down, M, H, F,
                                      h1, 0, act_dtype, 0.0f, lo, hi, NULL, d, NULL);
    if (!rc) rc = mkq_ref_layernorm(d, M, H, p->ln2_gamma, p->ln2_beta, p->ln_eps, h_out);
    /* h_out is left in binary32 here; the caller narrows it (and may first
     * take next-layer codes from the binary32 value). */
    if (!rc && dbg) {
        if (dbg->c0) memcpy(dbg->c0, c0, (size_t)(M * H));
        if (dbg->qkv) memcpy(dbg->qkv, qkv, sizeof(float) * (size_t)(M * 3 * H));
        if (dbg->ctx) memcpy(dbg->ctx, ctx, sizeof(float) * (size_t)(M * H));
        if (dbg->c1) memcpy(dbg->c1, c1, (size_t)(M * H));
        if (dbg->u) memcpy(dbg->u, u, sizeof(float) * (size_t)(M * H));
        if (dbg->h1) memcpy(dbg->h1, h1, sizeof(float) * (size_t)(M * H));
        if (dbg->c2) memcpy(dbg->c2, c2, (size_t)(M * H));
        if (dbg->c3) memcpy(dbg->c3, c3, (size_t)(M * F));
        if (dbg->d) memcpy(dbg->d, d, sizeof(float) * (size_t)(M * H));
        if (dbg->g_pre) memcpy(dbg->g_pre, g, sizeof(float) * (size_t)(M * F));
    }
    free(c0); free(c1); free(c2); free(c3);
    free(qkv); free(ctx); free(u); free(h1); free(g); free(d);
    return rc;
}

/* The same layer in the 16-bit float baseline: no quantizers, weights given as
 * binary32 arrays holding binary16 values. */
typedef struct {
    int64_t batch, seq, hidden, heads, ffn;
    const float *w_qkv, *w_ao, *w_up, *w_down;
    const float *b_qkv, *b_ao, *b_up, *b_down;
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    float ln_eps;
} mkq_ref_layer_params_float;

int mkq_ref_bert_layer_float(const mkq_ref_layer_params_float *p, const float *h_in,
                             int act_dtype, float *h_out)
{
    if (!p || !h_in || !h_out) return MKQ_REF_ERR_NULL;
    const int64_t M = p->batch * p->seq, H = p->hidden, F = p->ffn;
    float *qkv = (float *)malloc(sizeof(float) * (size_t)(M * 3 * H));
    float *ctx = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *u = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *h1 = (float *)malloc(sizeof(float) * (size_t)(M * H));
    float *g = (float *)malloc(sizeof(float) * (size_t)(M * F));
    float *d = (float *)malloc(sizeof(float) * (size_t)(M * H));
    int rc = mkq_ref_linear_float(h_in, p->w_qkv, p->b_qkv, M, 3 * H, H, NULL, 0, act_dtype, qkv);
    if (!rc) rc = mkq_ref_attention(qkv, p->batch, p->seq, H, p->heads, act_dtype, ctx);
    if (!rc) rc = mkq_ref_round_storage(ctx, M * H, act_dtype);
    if (!rc) rc = mkq_ref_linear_float(ctx, p->w_ao, p->b_ao, M, H, H, h_in, 0, act_dtype, u);
    if (!rc) rc = mkq_ref_layernorm(u, M, H, p->ln1_gamma, p->ln1_beta, p->ln_eps, h1);
    if (!rc) rc = mkq_ref_round_storage(h1, M * H, act_dtype);
    if (!rc) rc = mkq_ref_linear_float(h1, p->w_up, p->b_up, M, F, H, NULL, 1, act_dtype, g);
    if (!rc) rc = mkq_ref_linear_float(g, p->w_down, p->b_down, M, H, F, h1, 0, act_dtype, d);
    if (!rc) rc = mkq_ref_layernorm(d, M, H, p->ln2_gamma, p->ln2_beta, p->ln_eps, h_out);
    free(qkv); free(ctx); free(u); free(h1); free(g); free(d);
    return rc;
}

/* Scale gradients of section 4.1 for one tensor and one scale (used only to pin
 * the quantizer against the paper's worked example):
 *   STE : sum_i ( -x_i/s + round(x_i/s) )
 *   MSE : 2 sum_i ( Q[x_i] - x_i ) round(x_i/s)
 * with round() including the clamp of Eq. 1.  Evaluated in binary64. */
int mkq_ref_scale_gradients(const float *x, int64_t n, float s, int qmin, int qmax,
                            double *g_ste, double *g_mse)
{
    if (!x || !g_ste || !g_mse) return MKQ_REF_ERR_NULL;
    if (!scale_ok(s)) return MKQ_REF_ERR_SCALE;
    double ste = 0.0, mse = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double c = (double)quantize_one(x[i], s, qmin, qmax);
        ste += -(double)x[i] / (double)s + c;
        mse += 2.0 * ((double)s * c - (double)x[i]) * c;
    }
    *g_ste = ste;
    *g_mse = mse;
    return MKQ_REF_OK;
}

/* Number of OpenMP threads the loops above will use (reported beside timings). */
int mkq_ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
