"""GPU parity of the 8-bit linear (W8A8; the int8 comparison column of Table 2 and the
8-bit layers of the mixed-precision models of section 4.2) against the oracle run with the
clamp range [-128, 127]: codes and int32 accumulators bit-exact, float outputs to the
1e-3 / 1e-2 rule (and in fact identical: every epilogue op is one correctly rounded
binary32 op on both sides)."""
import numpy as np
import pytest

import oracle
from layer_checks import LayerBuffers, attention_code_band, check_layer_stagewise, codes_match
from helpers import RTOL, assert_codes_match_with_tie_band, assert_float_close, to_dev, to_np

pytestmark = pytest.mark.gpu
Q8 = dict(qmin=-128, qmax=127)


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m


def _codes_case(M, N, K, seed):
    rng = np.random.default_rng(seed)
    A = rng.integers(-128, 128, (M, K), dtype=np.int8)
    Wc = rng.integers(-128, 128, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.0001, 0.003, N).astype(np.float32)
    bias = rng.normal(0, 0.5, N).astype(np.float32)
    return A, Wc, s_w, np.float32(0.02), bias


@pytest.mark.parametrize("x_dtype", ["f32", "f16"])
@pytest.mark.parametrize("M,K", [(1, 16), (7, 48), (130, 768), (1024, 3072)])
def test_quantize_int8_bit_exact(mkq, M, K, x_dtype):
    rng = np.random.default_rng(M + K)
    s = np.float32(0.0173)
    X = (rng.standard_normal((M, K)) * 1.5).astype(np.float32)
    X.flat[:: 97] *= 8  # some values beyond +-127 steps
    X.flat[5 % X.size] = np.nan
    if x_dtype == "f16":
        X = X.astype(np.float16)
    got = to_np(mkq.mkq_quantize_int8(to_dev(X), float(s)))
    ref = oracle.quantize(X.astype(np.float32), s, **Q8)
    assert ref.min() == -128 or M * K < 100
    assert np.array_equal(got, ref)


def test_quantize_int8_strided_rows_and_empty(mkq):
    import torch
    rng = np.random.default_rng(3)
    X = rng.standard_normal((33, 256)).astype(np.float32)
    xd = to_dev(X)[:, 64:192]  # row stride 256, K = 128
    got = to_np(mkq.mkq_quantize_int8(xd, 0.01))
    assert np.array_equal(got, oracle.quantize(np.ascontiguousarray(X[:, 64:192]), np.float32(0.01), **Q8))
    empty = mkq.mkq_quantize_int8(torch.empty((0, 64), device="cuda"), 0.01)
    assert empty.shape == (0, 64)


def test_pack_weights_int8_bit_exact(mkq):
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((300, 832)) * 0.02).astype(np.float32)
    W[17] = 0
    Wq, s_w = mkq.mkq_pack_weights_int8(to_dev(W))
    codes, s_ref = oracle.quantize_weights(W, **Q8)
    assert np.array_equal(to_np(s_w), s_ref) and s_ref[17] == 1.0
    assert np.array_equal(to_np(Wq), codes)
    given = rng.uniform(1e-4, 1e-3, 300).astype(np.float32)
    Wq2, s2 = mkq.mkq_pack_weights_int8(to_dev(W), s_w_in=to_dev(given))
    codes2, _ = oracle.quantize_weights(W, given, **Q8)
    assert np.array_equal(to_np(s2), given) and np.array_equal(to_np(Wq2), codes2)


SHAPES = [(128, 768, 768), (1, 32, 64), (16, 16, 64), (200, 328, 832), (257, 130, 192),
          (64, 2304, 768), (1024, 768, 3072), (300, 300, 2048), (2050, 1100, 128), (4100, 2100, 256)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_accumulators_and_f32_output(mkq, M, N, K):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M + N + K)
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_F32,
                            want_acc=True)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, **Q8)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert_float_close(to_np(r["out"]), ref["y"], RTOL[0], "f32 out")
    assert np.array_equal(to_np(r["out"]), ref["y"])


@pytest.mark.parametrize("K", [64, 4096, 65472])
def test_accumulator_extremes(mkq, K):
    M, N = 48, 80
    lo = np.full((M, K), -128, np.int8)
    ones = np.ones(N, np.float32)
    r = mkq.mkq_linear_int8(to_dev(lo), 1.0, to_dev(np.full((N, K), -128, np.int8)), to_dev(ones), None,
                            mkq.MKQ_F32, want_acc=True)
    assert np.all(to_np(r["acc"]) == (1 << 14) * K)
    r = mkq.mkq_linear_int8(to_dev(lo), 1.0, to_dev(np.full((N, K), 127, np.int8)), to_dev(ones), None,
                            mkq.MKQ_F32, want_acc=True)
    assert np.all(to_np(r["acc"]) == -128 * 127 * K)


@pytest.mark.parametrize("out_dtype", [1, 2])
@pytest.mark.parametrize("M,N,K", [(128, 768, 768), (200, 328, 832), (2050, 1100, 128)])
def test_narrow_outputs(mkq, M, N, K, out_dtype):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=out_dtype + M)
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), out_dtype)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=out_dtype, **Q8)
    got = to_np(r["out"]).astype(np.float32)
    assert_float_close(got, ref["y"], RTOL[out_dtype], "narrow out")
    assert np.array_equal(got, ref["y"])


@pytest.mark.parametrize("res_dtype", ["f32", "f16"])
def test_residual_and_gelu(mkq, res_dtype):
    M, N, K = 260, 392, 320
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=8)
    rng = np.random.default_rng(9)
    res = rng.standard_normal((M, N)).astype(np.float16 if res_dtype == "f16" else np.float32)
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_F32,
                            residual=to_dev(res))
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res.astype(np.float32), **Q8)
    assert np.array_equal(to_np(r["out"]), ref["y"])
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_F16,
                            act=mkq.MKQ_ACT_GELU)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU, out_dtype=oracle.F16, **Q8)
    assert_float_close(to_np(r["out"]).astype(np.float32), ref["y"], RTOL[1], "gelu f16")


def test_float_in_to_float_out_through_both_quantizers(mkq):
    """quantize -> linear on calibrated operands, the way an 8-bit layer of a mixed model runs."""
    rng = np.random.default_rng(10)
    M, K, N = 512, 768, 3072
    X = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.01).astype(np.float32)
    s_x = oracle.absmax_scale(X.astype(np.float32), qmax=127)
    Wq, s_w = mkq.mkq_pack_weights_int8(to_dev(W))
    a = mkq.mkq_quantize_int8(to_dev(X), float(s_x))
    r = mkq.mkq_linear_int8(a, float(s_x), Wq, s_w, to_dev(b), mkq.MKQ_F16)
    wc, sw = oracle.quantize_weights(W, **Q8)
    ref = oracle.linear_int4(oracle.quantize(X.astype(np.float32), s_x, **Q8), s_x, wc, sw, b,
                             out_dtype=oracle.F16, **Q8)
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    # and the 8-bit result sits close to the unquantized product
    exact = X.astype(np.float64) @ W.astype(np.float64).T + b
    assert np.sqrt(np.mean((ref["y"] - exact) ** 2)) < 0.02 * np.sqrt(np.mean(exact ** 2))


def test_large_m_sampled_rows_bf16(mkq):
    """The tile configuration used at benchmark sizes (256 x 128 tiles, two workgroups per CU)."""
    import torch
    M, K, N = 16384, 1024, 4096
    A, Wc, s_w, s_x, _ = _codes_case(M, N, K, seed=11)
    out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), None, mkq.MKQ_BF16, out=out)
    torch.cuda.synchronize()
    rng = np.random.default_rng(12)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, 257, M - 257, M - 256, M - 1], rng.integers(0, M, 40)]))
    got = to_np(out[torch.from_numpy(rows).cuda()]).astype(np.float32)
    ref = oracle.linear_int4(A[rows], s_x, Wc, s_w, None, out_dtype=oracle.BF16, **Q8)
    assert np.array_equal(got, ref["y"])


def test_argument_checks(mkq):
    import torch
    a = torch.zeros((4, 64), dtype=torch.int8, device="cuda")
    w = torch.zeros((8, 64), dtype=torch.int8, device="cuda")
    s = torch.ones(8, device="cuda")
    with pytest.raises(mkq.MkqError) as e:
        mkq.mkq_linear_int8(a[:, :32].contiguous(), 1.0, w[:, :32].contiguous(), s, None)
    assert e.value.status == mkq.MKQ_ERR_SHAPE  # K % 64
    with pytest.raises(mkq.MkqError) as e:
        mkq.mkq_linear_int8(a, 0.0, w, s, None)
    assert e.value.status == mkq.MKQ_ERR_SCALE
    with pytest.raises(mkq.MkqError) as e:
        mkq.mkq_linear_int8(a, 1.0, w, s, None, mkq.MKQ_I4, out=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == mkq.MKQ_ERR_UNSUPPORTED
    empty = mkq.mkq_linear_int8(a[:0], 1.0, w, s, None)
    assert empty["out"].shape == (0, 8)


# --- the 8-bit encoder layer ----------------------------------------------------------

def _f16(a):
    return np.asarray(a, np.float32).astype(np.float16)


def test_layernorm_and_attention_int8_codes(mkq):
    rng = np.random.default_rng(21)
    M, D = 130, 768
    x = _f16(rng.normal(0.2, 1.5, (M, D)))
    g = rng.normal(1, 0.2, D).astype(np.float32)
    b = rng.normal(0, 0.2, D).astype(np.float32)
    s_next = 0.02  # clips beyond +-2.5
    y, q = mkq.mkq_layernorm_int8(to_dev(x), to_dev(g), to_dev(b), 1e-12, s_next)
    ref = oracle.layernorm(x.astype(np.float32), g, b, 1e-12)
    assert_float_close(to_np(y).astype(np.float32), oracle.round_storage(ref, oracle.F16), RTOL[1], "layernorm")
    refq = oracle.quantize(ref, s_next, **Q8)
    assert refq.min() == -128 and refq.max() == 127
    assert_codes_match_with_tie_band(to_np(q), refq, ref, s_next, band=2.0 ** -7, max_frac=2e-3, what="layernorm codes")

    B, S, heads = 2, 96, 4
    H = heads * 64
    qkv = _f16(rng.normal(0, 1.0, (B * S, 3 * H)))
    s_next = 0.004
    ctx, q = mkq.mkq_attention_int8(to_dev(qkv), B, S, H, heads, s_next)
    ref = oracle.attention(qkv.astype(np.float32), B, S, H, heads, p_dtype=oracle.F16)
    assert_float_close(to_np(ctx).astype(np.float32), ref, RTOL[1], "attention")
    for b in range(B):  # per-element band: what one binary16 unit of every probability can move the context by
        rows = slice(b * S, (b + 1) * S)
        codes_match(to_np(q)[rows], oracle.quantize(ref[rows], s_next, **Q8), ref[rows], s_next,
                    attention_code_band(qkv[rows].astype(np.float32), S, H, heads, s_next), "attention codes")


def test_linear_int8_code_output_with_gelu(mkq):
    M, N, K = 300, 520, 256
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=23)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU, s_next=0.05, **Q8)
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_I8,
                            act=mkq.MKQ_ACT_GELU, s_next=0.05)
    assert_codes_match_with_tie_band(to_np(r["out"]), ref["q"], ref["y"], 0.05, band=2.0 ** -7, max_frac=2e-3,
                                     what="gelu codes")
    # without the transcendental the codes are decided by correctly rounded binary32 ops: exact
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, s_next=0.07, **Q8)
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_I8, s_next=0.07)
    assert np.array_equal(to_np(r["out"]), ref["q"])
    assert ref["q"].min() == -128 and ref["q"].max() == 127


# Few tokens (M <= 64, K % 128 == 0) take the weight-streaming kernel: eight waves split K, ragged N, K that does not
# divide evenly over the waves, the accumulator extremes, every kind of output
@pytest.mark.parametrize("M", [1, 16, 33, 64])
@pytest.mark.parametrize("N,K", [(200, 128), (40, 512), (768, 768), (328, 4096), (96, 2304), (72, 8192), (3072, 768)])
def test_few_token_linear_int8(mkq, M, N, K):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M * 3 + N + K)
    if N == 40:  # the extremes: |acc| = K * 128 * 128
        A[:] = -128
        Wc[: N // 2] = -128
        Wc[N // 2:] = 127
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, **Q8)
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_F32, want_acc=True)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]), ref["y"])
    # (the library's own route takes the tile kernels for 33 .. 64 tokens against small weights: the streaming
    # kernel is also asked for by number)
    r30 = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_F32, want_acc=True,
                              config=30)
    assert np.array_equal(to_np(r30["acc"]), ref["acc"]) and np.array_equal(to_np(r30["out"]), ref["y"])
    if N == 40:
        assert ref["acc"].max() == K * 128 * 128 and ref["acc"].min() == -K * 128 * 127
    res = np.random.default_rng(N).normal(0, 1, (M, N)).astype(np.float16)
    ref16 = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res.astype(np.float32), out_dtype=oracle.F16, **Q8)
    r16 = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_F16, residual=to_dev(res))
    assert np.array_equal(to_np(r16["out"]).astype(np.float32), ref16["y"])
    s_next = float(np.float32(max(np.abs(ref["y"]).max(), 1e-3) / 100))
    refq = oracle.linear_int4(A, s_x, Wc, s_w, bias, s_next=s_next, **Q8)
    rq = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_I8, s_next=s_next)
    assert np.array_equal(to_np(rq["out"]), refq["q"])
    refg = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU, s_next=s_next, **Q8)
    rg = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_I8,
                             act=mkq.MKQ_ACT_GELU, s_next=s_next)
    assert_codes_match_with_tie_band(to_np(rg["out"]), refg["q"], refg["y"], s_next, band=2.0 ** -7, max_frac=2e-3,
                                     what="gelu codes")


@pytest.mark.parametrize("B,S,hidden,heads,ffn", [(2, 64, 128, 2, 256), (2, 128, 768, 12, 3072), (1, 300, 512, 16, 1024), (1, 512, 256, 4, 512)])
def test_bert_layer_int8_stagewise_and_end_to_end(mkq, B, S, hidden, heads, ffn):
    import torch
    from paper_2203_13483_amd import workloads as wl
    p = wl.bert_layer_weights(hidden, heads, ffn, 51)
    rng = np.random.default_rng(58)
    for ln in ("ln1", "ln2"):
        p[ln + "_gamma"] = rng.normal(1, 0.1, hidden).astype(np.float32)
        p[ln + "_beta"] = rng.normal(0, 0.1, hidden).astype(np.float32)
    h = _f16(wl.hidden_states(B, S, hidden, 52))
    hf = h.astype(np.float32)
    M = B * S
    # activation steps calibrated on the float layer (abs-max over 127, tails clipped by 2x)
    qkv_f = oracle.linear_float(hf, p["W_qkv"], p["b_qkv"])
    ctx_f = oracle.attention(qkv_f, B, S, hidden, heads)
    u_f = oracle.linear_float(ctx_f, p["W_ao"], p["b_ao"], residual=hf)
    h1_f = oracle.layernorm(u_f, p["ln1_gamma"], p["ln1_beta"], p["ln_eps"])
    g_f = oracle.linear_float(h1_f, p["W_up"], p["b_up"], act=oracle.ACT_GELU)
    q = {k: p[k] for k in ("hidden", "heads", "ffn", "ln_eps", "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    q["batch"], q["seq"] = B, S
    packed, sx = {}, {}
    for nm, act_in in (("qkv", hf), ("ao", ctx_f), ("up", h1_f), ("down", g_f)):
        q["w_" + nm], q["sw_" + nm] = oracle.quantize_weights(p["W_" + nm], **Q8)
        q["b_" + nm] = p["b_" + nm]
        q["sx_" + nm] = float(np.float32(oracle.absmax_scale(act_in, qmax=127) * 0.5))
        Wq, s_w = mkq.mkq_pack_weights_int8(to_dev(p["W_" + nm]))
        assert np.array_equal(to_np(s_w), q["sw_" + nm]) and np.array_equal(to_np(Wq), q["w_" + nm])
        packed[nm] = (Wq, s_w, to_dev(p["b_" + nm]))
        sx[nm] = q["sx_" + nm]
    ln = {k: to_dev(p[k]) for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    s_out_next = 0.02
    layer = mkq.BertLayerInt8(B, S, hidden, heads, ffn, packed, sx, ln, p["ln_eps"], s_out_next)
    ws = torch.zeros(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
    q_next = torch.empty((M, hidden), dtype=torch.int8, device="cuda")
    h_out = layer(to_dev(h), ws, q_out_next=q_next)
    torch.cuda.synchronize()
    L = layer.layout
    wsn = to_np(ws)

    def codes(off, cols):
        return wsn[off: off + M * cols].view(np.int8).reshape(M, cols)

    def f16buf(off, cols):
        return wsn[off: off + M * cols * 2].view(np.float16).reshape(M, cols).astype(np.float32)

    c0, c1, c2, c3 = codes(L.c0, hidden), codes(L.c1, hidden), codes(L.c2, hidden), codes(L.c3, ffn)
    qkv, u, h1, d = f16buf(L.qkv, 3 * hidden), f16buf(L.u, hidden), f16buf(L.h1, hidden), f16buf(L.d, hidden)
    tie = dict(band=2.0 ** -7, max_frac=2e-3)

    assert np.array_equal(c0, oracle.quantize(hf, q["sx_qkv"], **Q8))
    r = oracle.linear_int4(c0, q["sx_qkv"], q["w_qkv"], q["sw_qkv"], q["b_qkv"], out_dtype=oracle.F16, **Q8)
    assert np.array_equal(qkv, r["y"])
    ctx_ref = oracle.attention(qkv, B, S, hidden, heads, p_dtype=oracle.F16)
    for b in range(B):
        rows = slice(b * S, (b + 1) * S)
        codes_match(c1[rows], oracle.quantize(ctx_ref[rows], q["sx_ao"], **Q8), ctx_ref[rows], q["sx_ao"],
                    attention_code_band(qkv[rows], S, hidden, heads, q["sx_ao"]), "context codes")
    r = oracle.linear_int4(c1, q["sx_ao"], q["w_ao"], q["sw_ao"], q["b_ao"], residual=hf, out_dtype=oracle.F16, **Q8)
    assert np.array_equal(u, r["y"])
    h1_ref = oracle.layernorm(u, p["ln1_gamma"], p["ln1_beta"], p["ln_eps"])
    assert_float_close(h1, oracle.round_storage(h1_ref, oracle.F16), RTOL[1], "h1")
    assert_codes_match_with_tie_band(c2, oracle.quantize(h1_ref, q["sx_up"], **Q8), h1_ref, q["sx_up"],
                                     what="h1 codes", **tie)
    r = oracle.linear_int4(c2, q["sx_up"], q["w_up"], q["sw_up"], q["b_up"], act=oracle.ACT_GELU,
                           s_next=q["sx_down"], **Q8)
    assert_codes_match_with_tie_band(c3, r["q"], r["y"], q["sx_down"], what="ffn codes", **tie)
    r = oracle.linear_int4(c3, q["sx_down"], q["w_down"], q["sw_down"], q["b_down"], residual=h1,
                           out_dtype=oracle.F16, **Q8)
    assert np.array_equal(d, r["y"])
    out_ref = oracle.layernorm(d, p["ln2_gamma"], p["ln2_beta"], p["ln_eps"])
    got_out = to_np(h_out).astype(np.float32)
    assert_float_close(got_out, oracle.round_storage(out_ref, oracle.F16), RTOL[1], "layer out (teacher-forced)")
    assert_codes_match_with_tie_band(to_np(q_next), oracle.quantize(out_ref, s_out_next, **Q8), out_ref, s_out_next,
                                     what="next-layer codes", **tie)

    # end to end against the oracle's own 8-bit layer, and against the unquantized layer
    ref_out, _ = oracle.bert_layer_int4(q, hf, act_dtype=oracle.F16, **Q8)
    err = got_out - ref_out
    assert np.sqrt((err ** 2).mean()) < 0.02 * np.sqrt((ref_out ** 2).mean())


def test_mixed_4bit_and_8bit_layers_follow_each_other(mkq):
    """Section 4.2 deploys models with 8-bit and 4-bit layers mixed: a layer writes the codes of its
    output at the width of the layer that follows.  Each layer's output codes are checked against the
    oracle's quantizer at that width, and the next layer, fed those codes, against the oracle's layer."""
    import torch
    from paper_2203_13483_amd import workloads as wl
    B, S, hidden, heads, ffn = 2, 64, 128, 2, 256
    M = B * S
    h = _f16(wl.hidden_states(B, S, hidden, 61))
    layers = []
    for i, bits in enumerate((8, 4, 8)):
        p = wl.bert_layer_weights(hidden, heads, ffn, 70 + i)
        rng_q = Q8 if bits == 8 else dict(qmin=-8, qmax=7)
        q = {k: p[k] for k in ("hidden", "heads", "ffn", "ln_eps", "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
        q["batch"], q["seq"] = B, S
        packed, sx = {}, {}
        steps4 = {"qkv": 0.34, "ao": 0.05, "up": 0.34, "down": 0.05}
        for nm in ("qkv", "ao", "up", "down"):
            q["w_" + nm], q["sw_" + nm] = oracle.quantize_weights(p["W_" + nm], **rng_q)
            q["b_" + nm] = p["b_" + nm]
            q["sx_" + nm] = float(np.float32(steps4[nm] * (7.0 / 127.0 if bits == 8 else 1.0)))
            pack = mkq.mkq_pack_weights_int8 if bits == 8 else mkq.mkq_pack_weights_int4
            Wq, s_w = pack(to_dev(p["W_" + nm]))
            packed[nm] = (Wq, s_w, to_dev(p["b_" + nm]))
            sx[nm] = q["sx_" + nm]
        layers.append((bits, p, q, packed, sx, rng_q))
    x = to_dev(h)
    q_in = None
    c_prev = None
    x_ref = h.astype(np.float32)
    for i, (bits, p, q, packed, sx, rng_q) in enumerate(layers):
        nxt = layers[i + 1] if i + 1 < len(layers) else None
        next_bits = nxt[0] if nxt else 0
        s_next = nxt[2]["sx_qkv"] if nxt else 0.0
        ln = {k: to_dev(p[k]) for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
        cls = mkq.BertLayerInt8 if bits == 8 else mkq.BertLayerInt4
        layer = cls(B, S, hidden, heads, ffn, packed, sx, ln, p["ln_eps"], s_next, next_bits=next_bits)
        ws = torch.zeros(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
        q_next = None
        if nxt:
            q_next = (torch.empty((M, hidden), dtype=torch.int8, device="cuda") if next_bits == 8
                      else torch.empty((M, hidden // 2), dtype=torch.uint8, device="cuda"))
        out = layer(x, ws, q_in=q_in, q_out_next=q_next)
        torch.cuda.synchronize()
        got = to_np(out).astype(np.float32)
        # the oracle's layer on the GPU's own input (binary16 values): closeness end to end
        ref_out, _ = oracle.bert_layer_int4(q, x_ref, act_dtype=oracle.F16, **rng_q)
        err = got - ref_out
        assert np.sqrt((err ** 2).mean()) < 0.03 * np.sqrt((ref_out ** 2).mean()), i
        # every stage, and the codes handed to the next layer at ITS width, against the oracle fed the GPU's
        # own previous stage (the codes are decided from the binary32 LayerNorm output, which the oracle
        # recomputes from the GPU's binary16 input of that LayerNorm)
        buf = LayerBuffers(to_np(ws), layer.layout, M, hidden, ffn, bits)
        codes_next = None
        if nxt:
            codes_next = to_np(q_next) if next_bits == 8 else oracle.unpack_nibbles(to_np(q_next), hidden)
        check_layer_stagewise(buf, q, x_ref, got, [(b * S, S) for b in range(B)], c0_in=c_prev, q_next=codes_next,
                              s_out_next=float(np.float32(s_next)) if nxt else 0.0, next_bits=next_bits,
                              what=f"layer {i} ({bits} bits)")
        c_prev = codes_next
        x, q_in, x_ref = out, q_next, got


@pytest.mark.parametrize("s", [0.021, 1.0 / 3.0, 0.1, 2.0 ** -20, 300.0])
def test_quantize_int8_around_every_rounding_boundary(mkq, s):
    """Values a few ulps either side of every boundary (k + 1/2) s of the 8-bit range: the kernel decides
    most codes from a reciprocal and must agree with the division."""
    s32 = np.float32(s)
    b = (np.arange(-131, 131) + 0.5)[:, None] * np.float64(s32)
    x = (b * (1.0 + np.arange(-6, 7)[None, :] * 2.0 ** -24)).astype(np.float32).ravel()
    x = np.concatenate([x, np.nextafter(x, np.float32(np.inf)), np.nextafter(x, np.float32(-np.inf))])
    x = np.concatenate([x, np.zeros((-x.size) % 64, np.float32)]).reshape(1, -1)
    q = to_np(mkq.mkq_quantize_int8(to_dev(x), float(s32)))
    assert np.array_equal(q, oracle.quantize(x, s32, **Q8))


# The fused 8-bit code decision at and next to exact ties (see the 4-bit case in test_gpu_linear.py): acc * s_x is
# exact, a step of 2 * s_x makes every odd accumulator a tie, steps an ulp either side or without an exact binary32
# form leave the quotient an ulp off it.  Codes must equal the oracle's, no band.
@pytest.mark.parametrize("config", [None, 28, 29, 18])
@pytest.mark.parametrize("s_x", [1.0, 0.25])
def test_fused_code_decision_int8_at_and_next_to_exact_ties(mkq, s_x, config):
    M, N, K = 300, 264, 128
    rng = np.random.default_rng(77)
    A = (rng.integers(-9, 10, (M, K)) * (rng.random((M, K)) < 0.2)).astype(np.int8)
    Wc = (rng.integers(-9, 10, (N, K)) * (rng.random((N, K)) < 0.3)).astype(np.int8)
    ones = np.ones(N, np.float32)
    two = np.float32(2.0 * s_x)
    ties = 0
    for s_next in [two, np.nextafter(two, np.float32(np.inf)), np.nextafter(two, np.float32(0)), np.float32(two / 3),
                   np.float32(two * 0.4), np.float32(two * 0.1)]:
        ref = oracle.linear_int4(A, s_x, Wc, ones, None, s_next=float(s_next), **Q8)
        assert np.array_equal(ref["y"], ref["acc"].astype(np.float32) * np.float32(s_x))
        q = ref["y"].astype(np.float64) / np.float64(s_next)
        ties += int(((np.abs(q - np.floor(q) - 0.5) < 1e-6) & (np.abs(q) < 127)).sum())
        r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(ones), None, mkq.MKQ_I8, s_next=float(s_next),
                                config=config)
        assert np.array_equal(to_np(r["out"]), ref["q"]), f"s_next={s_next!r}"
    assert ties > 1000


# int8 code outputs with a row pitch: real columns at the pitch, zero codes in the padding, through the direct
# epilogue of the small tiles and the row epilogue of the large ones (forced configurations); stale buffers show
# that the padding is written
@pytest.mark.parametrize("M,N,K,pitch,config", [(100, 200, 128, 256, None), (300, 328, 256, 384, 29),
                                                (520, 264, 128, 320, 18), (64, 72, 512, 128, None),
                                                (16, 200, 128, 256, None), (1, 328, 256, 384, None)])
def test_int8_code_outputs_with_a_row_pitch(mkq, M, N, K, pitch, config):
    import torch
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M + pitch)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, s_next=0.07, **Q8)
    want = np.zeros((M, pitch), np.int8)
    want[:, :N] = ref["q"]
    out = torch.full((M, pitch), 0x5A, dtype=torch.int8, device="cuda")
    r = mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_I8, s_next=0.07,
                            out=out, q_pitch=pitch, config=config)
    assert np.array_equal(to_np(r["out"]), want)
    with pytest.raises(mkq.MkqError):
        mkq.mkq_linear_int8(to_dev(A), float(s_x), to_dev(Wc), to_dev(s_w), to_dev(bias), mkq.MKQ_I8, s_next=0.07,
                            out=out, q_pitch=N - 8, config=config)
