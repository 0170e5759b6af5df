/*
 * Memory / undefined-behaviour check of the CPU oracle (test infrastructure): built together with
 * mkq_oracle.c under -fsanitize=address,undefined and run by the CPU test tier.  It calls every entry point of
 * the oracle on small inputs in exactly-sized heap buffers (ragged sizes, size 0 and 1, both clamp ranges), so
 * that an access one element past a buffer, a signed overflow or a bad shift aborts the run.  It checks no
 * values: the pins in the Python tests do that.
 */
#include "mkq_oracle.c"

#include <stdio.h>

static unsigned long long lcg = 88172645463325252ull;
static float rnd(void)  /* roughly uniform on [-3, 3) */
{
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return (float)((double)(lcg >> 11) / 9007199254740992.0 * 6.0 - 3.0);
}
static float *floats(int64_t n, float scale)
{
    float *p = (float *)malloc(sizeof(float) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) p[i] = scale * rnd();
    return p;
}
#define CHECK(call) do { int rc_ = (call); if (rc_ != MKQ_REF_OK) { printf("%s -> %d\n", #call, rc_); return 1; } } while (0)

static int linear_case(int64_t M, int64_t N, int64_t K, int qmin, int qmax)
{
    float *X = floats(M * K, 1.0f), *W = floats(N * K, 0.05f), *b = floats(N, 0.1f), *res = floats(M * N, 1.0f);
    int8_t *a = (int8_t *)malloc((size_t)(M * K) + 1), *w = (int8_t *)malloc((size_t)(N * K) + 1);
    float *sw = floats(N, 1.0f), s_x = 0.4f;
    CHECK(mkq_ref_absmax_scale(X, M, K, K, 0, qmax, &s_x));
    CHECK(mkq_ref_quantize(X, M, K, K, s_x, qmin, qmax, a));
    CHECK(mkq_ref_quantize_weights(W, N, K, NULL, qmin, qmax, sw, w));
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)(M * N) + 4);
    float *y = floats(M * N, 0.0f);
    int8_t *q = (int8_t *)malloc((size_t)(M * N) + 1);
    CHECK(mkq_ref_gemm_codes(a, w, M, N, K, acc));
    CHECK(mkq_ref_epilogue(acc, M, N, s_x, sw, b, res, 1, y));
    for (int od = 0; od < 3; ++od)
        CHECK(mkq_ref_linear_int4(a, s_x, w, sw, b, M, N, K, od ? res : NULL, od == 1, od, 0.3f, qmin, qmax, acc, y, q));
    CHECK(mkq_ref_linear_float(X, W, b, M, N, K, res, 1, 1, y));
    float *d = floats(M * K, 0.0f);
    CHECK(mkq_ref_dequantize(a, M * K, s_x, d));
    if (K % 2 == 0 && qmax == 7) {
        uint8_t *packed = (uint8_t *)malloc((size_t)(M * K / 2) + 1);
        CHECK(mkq_ref_pack_nibbles(a, M, K, packed));
        CHECK(mkq_ref_unpack_nibbles(packed, M, K, a));
        free(packed);
    }
    free(X); free(W); free(b); free(res); free(a); free(w); free(sw); free(acc); free(y); free(q); free(d);
    return 0;
}

static int layer_case(int64_t B, int64_t S, int64_t H, int64_t heads, int64_t F, int qmin, int qmax)
{
    const int64_t M = B * S;
    float *Wf[4], *bias[4], *sw[4];
    int8_t *wc[4];
    const int64_t Ns[4] = {3 * H, H, F, H}, Ks[4] = {H, H, H, F};
    for (int i = 0; i < 4; ++i) {
        Wf[i] = floats(Ns[i] * Ks[i], 0.05f);
        bias[i] = floats(Ns[i], 0.05f);
        sw[i] = floats(Ns[i], 1.0f);
        wc[i] = (int8_t *)malloc((size_t)(Ns[i] * Ks[i]));
        CHECK(mkq_ref_quantize_weights(Wf[i], Ns[i], Ks[i], NULL, qmin, qmax, sw[i], wc[i]));
    }
    float *g1 = floats(H, 0.3f), *b1 = floats(H, 0.1f), *g2 = floats(H, 0.3f), *b2 = floats(H, 0.1f);
    float *h = floats(M * H, 1.0f), *out = floats(M * H, 0.0f);
    mkq_ref_layer_params p;
    memset(&p, 0, sizeof p);
    p.batch = B; p.seq = S; p.hidden = H; p.heads = heads; p.ffn = F;
    p.w_qkv = wc[0]; p.w_ao = wc[1]; p.w_up = wc[2]; p.w_down = wc[3];
    p.sw_qkv = sw[0]; p.sw_ao = sw[1]; p.sw_up = sw[2]; p.sw_down = sw[3];
    p.b_qkv = bias[0]; p.b_ao = bias[1]; p.b_up = bias[2]; p.b_down = bias[3];
    const float unit = qmax == 7 ? 1.0f : 7.0f / 127.0f;
    p.sx_qkv = 0.34f * unit; p.sx_ao = 0.05f * unit; p.sx_up = 0.34f * unit; p.sx_down = 0.05f * unit;
    p.ln1_gamma = g1; p.ln1_beta = b1; p.ln2_gamma = g2; p.ln2_beta = b2;
    p.ln_eps = 1e-12f; p.qmin = qmin; p.qmax = qmax;
    mkq_ref_layer_debug dbg;
    memset(&dbg, 0, sizeof dbg);
    dbg.c0 = (int8_t *)malloc((size_t)(M * H)); dbg.c1 = (int8_t *)malloc((size_t)(M * H));
    dbg.c2 = (int8_t *)malloc((size_t)(M * H)); dbg.c3 = (int8_t *)malloc((size_t)(M * F));
    dbg.qkv = floats(M * 3 * H, 0.0f); dbg.ctx = floats(M * H, 0.0f); dbg.u = floats(M * H, 0.0f);
    dbg.h1 = floats(M * H, 0.0f); dbg.d = floats(M * H, 0.0f); dbg.g_pre = floats(M * F, 0.0f);
    for (int act_dtype = 0; act_dtype < 2; ++act_dtype) {
        CHECK(mkq_ref_bert_layer_int4(&p, h, NULL, act_dtype, out, &dbg));
        CHECK(mkq_ref_bert_layer_int4(&p, h, dbg.c0, act_dtype, out, NULL));
    }
    mkq_ref_layer_params_float pf;
    memset(&pf, 0, sizeof pf);
    pf.batch = B; pf.seq = S; pf.hidden = H; pf.heads = heads; pf.ffn = F;
    pf.w_qkv = Wf[0]; pf.w_ao = Wf[1]; pf.w_up = Wf[2]; pf.w_down = Wf[3];
    pf.b_qkv = bias[0]; pf.b_ao = bias[1]; pf.b_up = bias[2]; pf.b_down = bias[3];
    pf.ln1_gamma = g1; pf.ln1_beta = b1; pf.ln2_gamma = g2; pf.ln2_beta = b2; pf.ln_eps = 1e-12f;
    CHECK(mkq_ref_bert_layer_float(&pf, h, 1, out));
    for (int pd = 0; pd < 2; ++pd) CHECK(mkq_ref_attention(dbg.qkv, B, S, H, heads, pd, dbg.ctx));
    CHECK(mkq_ref_layernorm(h, M, H, NULL, NULL, 1e-5f, out));
    for (int i = 0; i < 4; ++i) { free(Wf[i]); free(bias[i]); free(sw[i]); free(wc[i]); }
    free(g1); free(b1); free(g2); free(b2); free(h); free(out);
    free(dbg.c0); free(dbg.c1); free(dbg.c2); free(dbg.c3); free(dbg.qkv); free(dbg.ctx); free(dbg.u);
    free(dbg.h1); free(dbg.d); free(dbg.g_pre);
    return 0;
}

int main(void)
{
    const int64_t shapes[][3] = {{1, 1, 2}, {3, 5, 8}, {17, 33, 64}, {0, 4, 8}, {5, 1, 30}, {9, 7, 2}};
    for (size_t i = 0; i < sizeof shapes / sizeof shapes[0]; ++i) {
        if (linear_case(shapes[i][0], shapes[i][1], shapes[i][2], -8, 7)) return 1;
        if (linear_case(shapes[i][0], shapes[i][1], shapes[i][2], -128, 127)) return 1;
    }
    if (layer_case(2, 5, 16, 2, 24, -8, 7) || layer_case(1, 1, 8, 1, 8, -128, 127) || layer_case(3, 7, 24, 3, 40, -8, 7))
        return 1;
    /* scale machinery, rounding helpers, special values */
    float *x = floats(1000, 2.0f), s = 0.0f, t = 0.0f;
    x[3] = INFINITY; x[4] = -INFINITY; x[5] = NAN; x[6] = 3.0e38f; x[7] = -3.0e38f; x[8] = 1e-45f;
    int8_t *c = (int8_t *)malloc(1000);
    CHECK(mkq_ref_quantize(x, 10, 100, 100, 1e-30f, -8, 7, c));
    CHECK(mkq_ref_quantize(x, 10, 100, 100, 3.0e38f, -128, 127, c));
    CHECK(mkq_ref_quantize(x, 4, 50, 100, 0.37f, -8, 7, c));  /* strided rows */
    x[3] = x[4] = x[5] = 0.5f;
    for (int64_t ppm = 0; ppm <= 1000000; ppm += 250000) CHECK(mkq_ref_percentile_scale(x, 1000, ppm, 7, &s, &t));
    CHECK(mkq_ref_percentile_scale(x, 1, 100, 127, &s, NULL));
    double g0 = 0, g1 = 0;
    CHECK(mkq_ref_scale_gradients(x, 1000, 0.3f, -8, 7, &g0, &g1));
    CHECK(mkq_ref_scale_gradients(x, 0, 0.3f, -128, 127, &g0, &g1));
    for (int dt = 0; dt < 3; ++dt) CHECK(mkq_ref_round_storage(x, 1000, dt));
    float per_row[10];
    CHECK(mkq_ref_absmax_scale(x, 10, 100, 100, 1, 7, per_row));
    free(x); free(c);
    printf("oracle sanitizer driver: ok (%d threads)\n", mkq_ref_num_threads());
    return 0;
}
