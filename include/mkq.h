/*
 * mkq.h -- C ABI of libmkq: the 4-bit (W4A4) quantized BERT linear layer of
 * MKQ-BERT (arXiv 2203.13483) for AMD MI355X (gfx950).
 *
 * Conventions that hold for every entry point unless it says otherwise
 *   - returns an int status: MKQ_OK (0) or a negative MKQ_ERR_* code; nothing
 *     throws, nothing prints;
 *   - every pointer is a DEVICE pointer owned by the caller (the library keeps
 *     no reference after the call is enqueued), except arguments whose names
 *     end in _host and the parameter structs themselves, which are read on the
 *     host during the call;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream); the call does not synchronise and does not allocate;
 *   - matrices are row-major and dense (row stride = number of columns) unless
 *     a leading dimension is given; device pointers must be 16-byte aligned;
 *   - argument errors are detected on the host before anything is enqueued, so
 *     a failing call has no effect on device memory.
 *
 * Packed int4 ("I4") tensors use the canonical nibble packing: element k of a
 * row is the low nibble of byte k/2 when k is even, the high nibble when k is
 * odd, two's complement, rows of K/2 bytes.
 */
#ifndef MKQ_H
#define MKQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MKQ_OK = 0,
    MKQ_ERR_NULL = -1,        /* a required pointer is NULL */
    MKQ_ERR_SHAPE = -2,       /* a dimension is negative / not a supported multiple */
    MKQ_ERR_ALIGN = -3,       /* a device pointer is not 16-byte aligned */
    MKQ_ERR_SCALE = -4,       /* a host-side step size is <= 0, NaN or Inf */
    MKQ_ERR_DTYPE = -5,       /* unknown / unsupported MKQ_* dtype or activation enum */
    MKQ_ERR_WORKSPACE = -6,   /* workspace NULL or smaller than the *_workspace_bytes value */
    MKQ_ERR_UNSUPPORTED = -7, /* valid request outside what the kernels cover (e.g. K >= 131072) */
    MKQ_ERR_HIP = -8          /* the HIP runtime reported an error at launch */
};

enum { MKQ_F32 = 0, MKQ_F16 = 1, MKQ_BF16 = 2, MKQ_I4 = 3, MKQ_I8 = 4 };
enum { MKQ_ACT_NONE = 0, MKQ_ACT_GELU = 1 };

const char *mkq_status_string(int status);
int mkq_version(void);

/* Quantizer of section 3.1, Eq. 1, integer part, 4 bits, one step for the whole
 * tensor (per-tensor scale):  code = round(clamp(x / s_x, -8, 7)), binary32
 * divide, round half to even, NaN -> 0.
 *   x      [M, K] of x_dtype (MKQ_F32 or MKQ_F16), row stride ldx elements
 *   q_out  [M, K/2] bytes, canonical packing
 * K must be a multiple of 32.  M == 0 is a no-op.
 * Errors: NULL, SHAPE (M<0, K<0, K%32, ldx<K), ALIGN, SCALE, DTYPE, HIP. */
int mkq_quantize(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s_x,
                 uint8_t *q_out, void *stream);

/* Abs-max calibration of section 3.1 (third paragraph):  s = max|x| / 7, written
 * to s_out[0] (per_row == 0) or s_out[m] for every row (per_row != 0).  An
 * all-zero tensor / row gets s = 1.  x_dtype MKQ_F32 or MKQ_F16.
 * Errors: NULL, SHAPE, ALIGN, DTYPE, HIP. */
int mkq_absmax_scale(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, int per_row,
                     float *s_out, void *stream);

/* Scale gradients of one tensor under one step (section 4.1):
 *     g_out[0] = sum_i ( round(x_i/s) - x_i/s )                 STE-based (4.1.1)
 *     g_out[1] = 2 sum_i ( Q[x_i] - x_i ) round(x_i/s)          MSE-based (4.1.2)
 * where round() is the code of Eq. 1 (clamp to the `bits`-bit range included, decided in
 * binary32 like the quantizer) and Q[x] = s * code.  Terms and sums are binary64; the
 * order of the partial sums is not fixed, so results agree to rounding only.
 *   x      [M, K] of x_dtype (MKQ_F32 or MKQ_F16), row stride ldx; K % 8 == 0, M > 0
 *   bits   4 or 8;  g_out  two doubles on the device (overwritten)
 * Errors: NULL, SHAPE, ALIGN, SCALE, DTYPE (x_dtype, bits), HIP. */
int mkq_scale_gradients(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s,
                        int bits, double *g_out, void *stream);

/* Percentile calibration of an activation step (section 3.1, third paragraph): the
 * clipping point T is the k-th largest |x_i|, k = max(1, floor(M*K * top_ppm / 10^6))
 * (top_ppm = 100 for the top 0.01 %), found exactly by radix selection over the bit
 * patterns of |x| (three counting passes over x); s_out[0] = T / (2^(bits-1) - 1), or 1
 * when T = 0.  NaN ranks as 0.  top_ppm = 0 gives abs-max calibration.
 *   workspace  at least mkq_percentile_scale_workspace_bytes() bytes, 16-byte aligned
 * M*K < 2^32.  Errors: NULL, SHAPE, ALIGN, DTYPE, WORKSPACE, UNSUPPORTED, HIP. */
size_t mkq_percentile_scale_workspace_bytes(void);
int mkq_percentile_scale(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx,
                         int64_t top_ppm, int bits, float *s_out, void *workspace,
                         size_t workspace_bytes, void *stream);

/* Offline weight preparation (Eq. 1 with one step per row = per output channel;
 * abs-max calibration when s_w_in is NULL).
 *   W        [N, K] binary32, row n = output channel n
 *   s_w_in   [N] steps to use, or NULL to calibrate  s_w[n] = max_k |W[n,k]| / 7
 *            (all-zero row -> 1).  Given steps must be > 0 and finite (precondition;
 *            they live on the device and are not checked).
 *   s_w_out  [N] the steps actually used (may alias s_w_in)
 *   Wq_out   mkq_packed_weight_bytes(N, K) bytes in the layout the GEMM reads
 *            (currently the canonical packing, rows of K/2 bytes)
 * K must be a multiple of 32.
 * Errors: NULL, SHAPE, ALIGN, HIP. */
size_t mkq_packed_weight_bytes(int64_t N, int64_t K);
int mkq_pack_weights_int4(const float *W, int64_t N, int64_t K, const float *s_w_in,
                          float *s_w_out, uint8_t *Wq_out, void *stream);

/* Reduction lengths that are not a multiple of 32 (the 4-layer student of section 5.2 has hidden size
 * 312 and FFN size 1200): both operands are stored with rows padded to mkq_padded_k(K) codes, the
 * smallest multiple of 128 >= K (whole 64-byte stages of the tile kernels), the padding codes being
 * zero, which adds nothing to any dot product.  The padded variants of the quantizer and of the weight
 * preparation take K % 8 == 0, compute exactly what their plain counterparts compute on the K real
 * columns (abs-max over the real columns only) and write rows of mkq_padded_k(K) / 2 bytes;
 * mkq_linear_int4 is then called with K = mkq_padded_k(K) on pre-quantized activations.  Same errors
 * as the plain variants (SHAPE on K % 8 instead of K % 32). */
int64_t mkq_padded_k(int64_t K);
int mkq_quantize_padded(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s_x,
                        uint8_t *q_out, void *stream);
int mkq_pack_weights_int4_padded(const float *W, int64_t N, int64_t K, const float *s_w_in,
                                 float *s_w_out, uint8_t *Wq_out, void *stream);

/* Packs already-quantized int8 codes (values in [-8, 7]; higher bits are
 * discarded) of a [rows, K] matrix into the weight / activation layout. */
int mkq_pack_codes_int4(const int8_t *codes, int64_t rows, int64_t K, uint8_t *q_out, void *stream);

/* Inverse of the weight layout: int8 codes [N, K] (for tests and inspection). */
int mkq_unpack_weights_int4(const uint8_t *Wq, int64_t N, int64_t K, int8_t *codes_out,
                            void *stream);

/* Optional parts of the linear's epilogue. */
typedef struct mkq_epilogue {
    int act;              /* MKQ_ACT_*; applied after bias and residual (GELU: erf form, FFN of section 3.2) */
    const void *residual; /* NULL or [M, N] added after the bias */
    int residual_dtype;   /* MKQ_F32 or MKQ_F16 */
    float s_next;         /* step of the next layer's activation quantizer; used when out_dtype == MKQ_I4
                             or q_out != NULL */
    uint8_t *q_out;       /* NULL, or [M, N/2] packed codes of the binary32 result under s_next, written
                             in addition to a float `out` */
    int32_t *acc_out;     /* NULL, or [M, N] raw int32 accumulators (for parity checks) */
    void *splitk_scratch; /* NULL, or a scratch area prepared by mkq_splitk_scratch_init (see there): lets a
                             linear with few tokens split K across workgroups to fill the chip */
    size_t splitk_scratch_bytes;
    int64_t q_pitch;      /* codes per row of the code outputs (`out` of MKQ_I4 / MKQ_I8, q_out); 0 = N.  A
                             consumer whose reduction length is padded (mkq_padded_k) takes rows of that
                             many codes: give the padded length here; the columns N .. q_pitch - 1 of every
                             row are written as zero codes.  >= N, a multiple of 8, and N % 8 == 0. */
} mkq_epilogue;

/* Scratch of a K split across workgroups.  Few tokens against a weight matrix with few output channels
 * give too few workgroups to fill 256 compute units; the reduction over K is then cut into slices that
 * different workgroups sum (int32 addition is associative: the accumulators are the same bit for bit),
 * their partial sums meeting in this area.  It is device memory owned by the caller, at least
 * mkq_splitk_scratch_bytes() bytes (a constant: 16 KiB of ticket counters, then 16 MiB for partial sums),
 * 16-byte aligned.  mkq_splitk_scratch_init clears the counters and must have run once (on any stream,
 * ordered before the first linear that uses the area) after the area was allocated; every linear leaves the
 * counters cleared again.  Two linears that may run at the same time need two areas.  A linear given no
 * area, or whose partial sums would not fit, runs without the split -- same results, fewer workgroups.
 * Errors: NULL, ALIGN, WORKSPACE (area too small), HIP. */
size_t mkq_splitk_scratch_bytes(void);
int mkq_splitk_scratch_init(void *scratch, size_t scratch_bytes, void *stream);

/* Once-per-device setup of every kernel of the library (dynamic LDS limits, occupancy queries) for the
 * device that is current.  Optional: each kernel is otherwise set up, under a lock, the first time it is
 * launched on a device.  Call it before capturing launches into a HIP graph if no eager call has run yet.
 * Errors: HIP. */
int mkq_init(void);

/* The quantized linear layer  y = x W^T + b  with both operands in 4 bits
 * (the int4 matrix multiplication of sections 1 and 5.4 applied to the linears
 * of section 3.2):
 *     acc[m,n] = sum_k a[m,k] * w[n,k]                      (int32, exact)
 *     y[m,n]   = fma((float)acc, s_x * s_w[n], bias[n])     (binary32)
 *     y       += residual;  y = act(y)                      (optional)
 *     out      = narrow(y)  or  codes(y; s_next) packed     (Eq. 1 again)
 *   a        [M, K]: packed codes (a_dtype == MKQ_I4, rows of K/2 bytes) or float
 *            activations (MKQ_F32 / MKQ_F16), which are first quantized with s_x
 *            into `workspace` by a launch of mkq_quantize's kernel that precedes the
 *            GEMM (two launches: inside one launch the hand-over between the
 *            quantizing and the multiplying workgroups cost more than the second launch)
 *   Wq, s_w  from mkq_pack_weights_int4;  bias [N] binary32 or NULL
 *   out      [M, N] of out_dtype (F32, F16, BF16) or [M, N/2] bytes (I4); may be
 *            NULL when epi->q_out or epi->acc_out is the only result wanted
 *   epi      NULL = no activation, no residual, no extra outputs
 *   workspace  at least mkq_linear_int4_workspace_bytes(M, N, K, a_dtype) bytes
 *              (0 for packed input: then workspace may be NULL)
 * K % 32 == 0, K < 131072; N even when codes are written.  M == 0 is a no-op.
 * Errors: NULL, SHAPE, ALIGN, SCALE (s_x, s_next), DTYPE, WORKSPACE, UNSUPPORTED, HIP. */
size_t mkq_linear_int4_workspace_bytes(int64_t M, int64_t N, int64_t K, int a_dtype);
int mkq_linear_int4(const void *a, int a_dtype, float s_x, const uint8_t *Wq, const float *s_w,
                    const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                    const mkq_epilogue *epi, void *workspace, size_t workspace_bytes, void *stream);

/* Few tokens (M <= 128): the linear is one pass over the weights and is bound by how fast they stream from
 * HBM.  Canonical rows, K/2 bytes apart, are a poor stream (32 rows fetched side by side, a power-of-two
 * pitch apart, land on the same few memory channels), so weights that serve few tokens can be kept in a
 * second layout in which the bytes that the chip reads at one moment lie next to each other: the 32 channels
 * of panel q (q = 0 .. P-1, P = ceil(N / 32)) and the 64 codes of k position g (g = 0 .. K/64 - 1) form a
 * block of 1 KiB = 64 pieces of 16 bytes; the block is number g P' + q, where P' = P if P is odd, else P + 1
 * (all panels of one k position, one unused block when P is even, then the next k position: an odd pitch keeps
 * the k positions that a wave has in flight off each other's memory channels); piece l of a block is bytes
 * [32 g + 16 (l / 32), + 16) of the canonical row of channel 32 q + r(l % 32), where
 * r(i) = 16 (i / 16) + 8 ((i / 4) % 2) + 4 ((i / 8) % 2) + i % 4; channels past N and the unused block are
 * zero.  mkq_stream_weight_bytes(N, K) = 32 P' K / 2.
 *   mkq_repack_weights_int4_stream   canonical (from mkq_pack_weights_int4) -> streaming layout; K % 64 == 0
 *   mkq_linear_int4_stream           mkq_linear_int4 on weights in the streaming layout: same arguments, same
 *                                    results bit for bit; M <= 128 and K % 256 == 0 (else UNSUPPORTED)
 * Errors: as mkq_linear_int4. */
size_t mkq_stream_weight_bytes(int64_t N, int64_t K);
int mkq_repack_weights_int4_stream(const uint8_t *Wq, int64_t N, int64_t K, uint8_t *Wq_stream_out, void *stream);
int mkq_linear_int4_stream(const void *a, int a_dtype, float s_x, const uint8_t *Wq_stream, const float *s_w,
                           const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                           const mkq_epilogue *epi, void *workspace, size_t workspace_bytes, void *stream);

/* For callers that cannot allocate device memory or carry a scratch area around -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: mkq_linear_int4_stream on packed codes
 * (a is [M, K/2] bytes; no workspace) with the scratch of the K split taken from an area that is part of
 * the library's code object (16 KiB of ticket counters + 16 MiB for partial sums, per GPU, held until the
 * process ends) instead of epi->splitk_scratch, which is ignored.  Nothing is allocated or freed.  Same
 * results as mkq_linear_int4_stream, bit for bit.  A problem whose K split would need more room for partial
 * sums than the area has (ceil(N / 128) * slices * 16 KiB * ceil(M / 32) rounded up to 1, 2 or 4 > 16 MiB,
 * or N > 524288) is refused with MKQ_ERR_UNSUPPORTED and nothing runs.  All calls on one GPU share the area:
 * calls that may overlap in time on one GPU (two streams, two threads) race; calls ordered on one stream
 * do not.  Other errors: as mkq_linear_int4. */
int mkq_linear_int4_stream_static(const uint8_t *a, float s_x, const uint8_t *Wq_stream, const float *s_w,
                                  const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                                  const mkq_epilogue *epi, void *stream);

/* The same linear with both operands in 8 bits (the int8 column of Table 2 in
 * section 5.4; the 8-bit layers of the mixed 4/8-bit models of section 4.2).  Eq. 1
 * with k = 8: codes in [-128, 127], one byte each, row-major, K-contiguous.
 *   mkq_quantize_int8      x [M, K] (F32 / F16, row stride ldx) -> int8 [M, K], per-tensor
 *                          step s_x; NaN -> 0.  K % 16 == 0.
 *   mkq_pack_weights_int8  W [N, K] binary32 -> int8 [N, K] and per-channel steps
 *                          s_w[n] = max_k |W[n,k]| / 127 (all-zero row -> 1) unless
 *                          s_w_in gives them.  K % 16 == 0.
 *   mkq_linear_int8        acc[m,n] = sum_k a[m,k] w[n,k] (int32, exact; |acc| <= K * 2^14),
 *                          y = fma((float)acc, s_x * s_w[n], bias[n]), then residual and
 *                          activation as in mkq_linear_int4.  a is int8 codes [M, K]
 *                          (quantize first; there is no workspace), out [M, N] of
 *                          F32 / F16 / BF16, or int8 codes of y under epi->s_next (MKQ_I8),
 *                          or NULL with epi->acc_out.  4-bit code outputs (out_dtype
 *                          MKQ_I4, epi->q_out) are not offered: UNSUPPORTED.
 *                          K % 64 == 0, K < 65536.  M == 0 is a no-op.
 * Errors: NULL, SHAPE, ALIGN, SCALE, DTYPE, UNSUPPORTED, HIP. */
int mkq_quantize_int8(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s_x,
                      int8_t *q_out, void *stream);
int mkq_pack_weights_int8(const float *W, int64_t N, int64_t K, const float *s_w_in,
                          float *s_w_out, int8_t *Wq_out, void *stream);
int mkq_linear_int8(const int8_t *a, float s_x, const int8_t *Wq, const float *s_w,
                    const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                    const mkq_epilogue *epi, void *stream);

/* Experimental: the 4-bit linear through the 6-bit float path of the matrix core.  Every code in [-8, 8]
 * is an E3M2 value (sign, 3 exponent bits with bias 3, 2 mantissa bits), products and sums of codes are
 * exact in binary32 while |sum| < 2^24, so the result is the same exact integer contraction as
 * mkq_linear_int4 -- with no widening and half the matrix instructions per k.  Operands are "containers":
 * 6 bits per code, rows of 3K/4 bytes made of groups of 64 codes = 48 bytes; the 32 codes of half h of a
 * group are a 192-bit little-endian stream (code i in bits [6i, 6i + 6)) stored as bytes [16h, 16h + 16)
 * and then [32 + 8h, 40 + 8h) of the group.  K % 64 == 0 for the containers, K % 128 == 0 and
 * K < 262144 for the linear.  The quantizer and the weight preparation are those of
 * mkq_quantize / mkq_pack_weights_int4 (Eq. 1, per-tensor / per-channel steps), written as containers;
 * mkq_pack_codes_e3m2 takes int8 codes in [-8, 8].  mkq_linear_int4_e3m2: arguments and epilogue as
 * mkq_linear_int4 with both operands given as containers (no workspace).
 * Errors: NULL, SHAPE, ALIGN, SCALE, DTYPE, UNSUPPORTED, HIP. */
int mkq_quantize_e3m2(const void *x, int x_dtype, int64_t M, int64_t K, int64_t ldx, float s_x,
                      uint8_t *q_out, void *stream);
int mkq_pack_codes_e3m2(const int8_t *codes, int64_t rows, int64_t K, uint8_t *q_out, void *stream);
int mkq_pack_weights_e3m2(const float *W, int64_t N, int64_t K, const float *s_w_in, float *s_w_out,
                          uint8_t *Wq_out, void *stream);
int mkq_linear_int4_e3m2(const uint8_t *a, float s_x, const uint8_t *Wq, const float *s_w,
                         const float *bias, int64_t M, int64_t N, int64_t K, void *out, int out_dtype,
                         const mkq_epilogue *epi, void *stream);

/* 16-bit float baseline linear (same epilogue, no quantizers):
 *   a [M, K] binary16, W [N, K] binary16, bias [N] binary32 or NULL, binary32
 *   accumulation, out [M, N] of out_dtype (F32 or F16), residual binary16 or NULL.
 * K % 64 == 0.  Errors: NULL, SHAPE, ALIGN, DTYPE, UNSUPPORTED, HIP. */
int mkq_linear_fp16(const void *a, const void *W, const float *bias, int64_t M, int64_t N,
                    int64_t K, void *out, int out_dtype, int act, const void *residual,
                    void *stream);

/* One post-LN BERT encoder layer (multi-head attention and feed-forward network
 * of section 3.2) with all six linears W4A4; LayerNorm, softmax and GELU are
 * computed in binary32 (section 5), the attention products in binary16 with
 * binary32 accumulation, hidden states are stored in binary16.
 *
 *   c0  = codes(h; sx_qkv)                      (or q_in, if the caller has them)
 *   qkv = Lin_qkv(c0)                           [M, 3*hidden], q | k | v
 *   ctx = softmax(q k^T / sqrt(d_k)) v          per sequence and head, d_k = hidden/heads
 *   u   = Lin_ao(codes(ctx; sx_ao)) + h
 *   h1  = LayerNorm1(u)
 *   d   = Lin_down(codes(GELU(Lin_up(codes(h1; sx_up))); sx_down)) + h1
 *   out = LayerNorm2(d)
 *
 * The struct lives on the host; the pointers inside are device pointers. */
typedef struct mkq_bert_layer_params {
    int64_t batch, seq, hidden, heads, ffn;
    const uint8_t *Wq_qkv, *Wq_ao, *Wq_up, *Wq_down; /* packed; qkv is [3*hidden, hidden] */
    const float *sw_qkv, *sw_ao, *sw_up, *sw_down;   /* per-output-channel steps */
    const float *b_qkv, *b_ao, *b_up, *b_down;       /* biases, binary32 */
    float sx_qkv, sx_ao, sx_up, sx_down;             /* learned per-tensor activation steps */
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    float ln_eps;
    float s_out_next; /* > 0: also write codes(out; s_out_next) to q_out_next */
    int next_bits;    /* width of those codes: 4 (packed, [M, hidden/2] bytes), 8 ([M, hidden] bytes), or 0 =
                         this layer's own width; lets 4-bit and 8-bit layers follow each other in a mixed
                         model (section 4.2) */
    /* Padding-free batches (the "valid tokens" of Table 2, section 5.4): cu_seqlens is NULL, or a device
     * array [batch + 1] of row offsets, sequence b being rows cu_seqlens[b] .. cu_seqlens[b+1] - 1 of the
     * total_tokens rows of h_in / h_out; seq is then an upper bound of the lengths (<= 128, any value);
     * a longer sequence is a precondition violation (its rows beyond the bound are not computed). */
    const int32_t *cu_seqlens;
    int64_t total_tokens;
} mkq_bert_layer_params;

/* Byte offsets of the layer's intermediates inside its workspace (all 256-byte
 * aligned); tests read them back stage by stage. */
typedef struct mkq_bert_layer_workspace_layout {
    size_t c0;   /* [M, hidden/2]   codes of the input                     */
    size_t qkv;  /* [M, 3*hidden]   binary16                                */
    size_t c1;   /* [M, hidden/2]   codes of the attention context          */
    size_t u;    /* [M, hidden]     binary16, attention output + residual   */
    size_t h1;   /* [M, hidden]     binary16, LayerNorm1 output             */
    size_t c2;   /* [M, hidden/2]   codes of h1                             */
    size_t c3;   /* [M, ffn/2]      codes of GELU(FFN-up)                   */
    size_t d;    /* [M, hidden]     binary16, FFN output + residual         */
    size_t total;
} mkq_bert_layer_workspace_layout;

int mkq_bert_layer_workspace(const mkq_bert_layer_params *p_host,
                             mkq_bert_layer_workspace_layout *layout_host);

/*   h_in   [M, hidden] binary16 (h_dtype == MKQ_F16) or binary32, M = batch*seq
 *   q_in   NULL, or packed codes of h_in under sx_qkv (skips the first quantizer)
 *   h_out  [M, hidden] binary16
 *   q_out_next  [M, hidden/2] bytes (or [M, hidden] when next_bits == 8), required iff s_out_next > 0
 * hidden % 8 == 0, ffn % 8 == 0, hidden % heads == 0 (else SHAPE); d_k = hidden / heads even and <= 64,
 * seq <= 4096, hidden <= 8192 (else UNSUPPORTED).
 * A hidden or FFN size that is no multiple of 32 (the 4-layer student of section 5.2: 312 and 1200) is
 * carried padded: every 4-bit code buffer whose rows feed a linear of that reduction length -- q_in,
 * q_out_next, the workspace's c0..c3 -- has rows of mkq_padded_k(size) / 2 bytes with zero codes past the
 * real columns (every kernel of the layer that writes codes writes the padding too), and the weights come from
 * mkq_pack_weights_int4_padded.  Sizes that are a multiple of 32 are stored as they are.
 * Errors: NULL, SHAPE, ALIGN, SCALE, DTYPE, WORKSPACE, UNSUPPORTED, HIP. */
int mkq_bert_layer_int4(const mkq_bert_layer_params *p_host, const void *h_in, int h_dtype,
                        const uint8_t *q_in, void *h_out, uint8_t *q_out_next, void *workspace,
                        size_t workspace_bytes, void *stream);

/* The same layer in the 16-bit float baseline (no quantizers). */
typedef struct mkq_bert_layer_params_fp16 {
    int64_t batch, seq, hidden, heads, ffn;
    const void *W_qkv, *W_ao, *W_up, *W_down; /* binary16 [N, K] */
    const float *b_qkv, *b_ao, *b_up, *b_down;
    const float *ln1_gamma, *ln1_beta, *ln2_gamma, *ln2_beta;
    float ln_eps;
    const int32_t *cu_seqlens; /* as in mkq_bert_layer_params */
    int64_t total_tokens;
} mkq_bert_layer_params_fp16;

size_t mkq_bert_layer_fp16_workspace_bytes(const mkq_bert_layer_params_fp16 *p_host);
int mkq_bert_layer_fp16(const mkq_bert_layer_params_fp16 *p_host, const void *h_in /* binary16 */,
                        void *h_out /* binary16 */, void *workspace, size_t workspace_bytes,
                        void *stream);

/* The same encoder layer with every linear W8A8 (an 8-bit layer of a mixed 4/8-bit model,
 * section 4.2; the int8 column of Table 2): the params struct is the one above with
 * Wq_* = int8 codes [N, K] from mkq_pack_weights_int8 and sx_* the steps of the 8-bit
 * range; every code buffer (q_in, q_out_next, the c* intermediates) holds one byte per
 * code, so the workspace layout has c0, c1, c2 of M*hidden bytes and c3 of M*ffn bytes.
 * Shape limits and errors of mkq_bert_layer_int4, but hidden % 64 == 0 and ffn % 64 == 0 (no padding). */
int mkq_bert_layer_int8_workspace(const mkq_bert_layer_params *p_host,
                                  mkq_bert_layer_workspace_layout *layout_host);
int mkq_bert_layer_int8(const mkq_bert_layer_params *p_host, const void *h_in, int h_dtype,
                        const int8_t *q_in, void *h_out, int8_t *q_out_next, void *workspace,
                        size_t workspace_bytes, void *stream);

/* Building blocks of the layer, exported for stage-wise parity checks.
 * LayerNorm over the last dimension in binary32 (section 5); x binary16 [M, D];
 * y binary16 [M, D] (may be NULL); q_out (NULL or [M, D/2]) receives
 * codes(y_binary32; s_next).  D % 8 == 0, D <= 8192. */
int mkq_layernorm(const void *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                  float eps, void *y, float s_next, uint8_t *q_out, void *stream);

/* Attention core of section 3.2 on a fused binary16 qkv buffer [batch*seq, 3*hidden]:
 * ctx binary16 [batch*seq, hidden] (may be NULL) and/or q_out packed codes under s_next.
 * Scores are scaled by 1/sqrt(d_k), d_k = hidden / heads; the softmax runs in binary32 and its normalized
 * probabilities are narrowed to binary16 before they multiply v.
 * d_k even and <= 64, hidden % 8 == 0, seq <= 4096 (anything else: UNSUPPORTED).  d_k == 64 with
 * seq <= 128 takes a kernel that holds all keys of a (sequence, head) at once; everything else one that
 * walks the keys in blocks of 128, twice (row maximum and denominator, then the weighted sum). */
int mkq_attention(const void *qkv, int64_t batch, int64_t seq, int64_t hidden, int64_t heads,
                  void *ctx, float s_next, uint8_t *q_out, void *stream);

/* Attention over a padding-free batch: qkv [total_tokens, 3*hidden], sequence b = rows
 * cu_seqlens[b] .. cu_seqlens[b+1] - 1 (device array [batch + 1]), each at most max_seq <= 4096 rows
 * (any length; an empty sequence is skipped).  q_out: codes of q_bits (4: [total, hidden/2] bytes,
 * 8: [total, hidden] bytes) or NULL.  Errors as mkq_attention, plus DTYPE for q_bits. */
int mkq_attention_varlen(const void *qkv, const int32_t *cu_seqlens, int64_t batch, int64_t max_seq,
                         int64_t hidden, int64_t heads, void *ctx, float s_next, void *q_out,
                         int q_bits, void *stream);

/* The two building blocks with 8-bit code output: q_out int8 [M, D] / [batch*seq, hidden]. */
int mkq_layernorm_int8(const void *x, int64_t M, int64_t D, const float *gamma, const float *beta,
                       float eps, void *y, float s_next, int8_t *q_out, void *stream);
int mkq_attention_int8(const void *qkv, int64_t batch, int64_t seq, int64_t hidden, int64_t heads,
                       void *ctx, float s_next, int8_t *q_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MKQ_H */
