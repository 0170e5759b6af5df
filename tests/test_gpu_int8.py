"""GPU parity of the 8-bit linear (W8A8; the int8 comparison column of Table 2 and the
8-bit layers of the mixed-precision models of section 4.2) against the oracle run with the
clamp range [-128, 127]: codes and int32 accumulators bit-exact, float outputs to the
1e-3 / 1e-2 rule (and in fact identical: every epilogue op is one correctly rounded
binary32 op on both sides)."""
import numpy as np
import pytest

import oracle
from helpers import RTOL, assert_float_close, to_dev, to_np

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
