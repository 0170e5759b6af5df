"""GPU parity of the 4-bit linear at reduction lengths that are not a multiple of 32 -- the hidden size 312
and FFN size 1200 of the 4-layer student (section 5.2): operands are stored with zero codes up to the next
multiple of 128, the oracle works on the real K columns."""
import numpy as np
import pytest

import oracle
from paper_2203_13483_amd import workloads as wl
from helpers import to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m


def _padded_reference(codes, Kp):
    out = np.zeros((codes.shape[0], Kp), np.int8)
    out[:, :codes.shape[1]] = codes
    return oracle.pack_nibbles(out)


@pytest.mark.parametrize("M,K", [(37, 312), (5, 1200), (64, 8), (3, 40)])
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_padded_quantizer_and_weights_bit_exact(mkq, M, K, dtype):
    rng = np.random.default_rng(M + K)
    Kp = mkq.mkq_padded_k(K)
    assert Kp % 128 == 0 and 0 <= Kp - K < 128
    X = (rng.standard_normal((M, K)) * 1.3).astype(dtype)
    s = np.float32(0.37)
    got = to_np(mkq.mkq_quantize_padded(to_dev(X), float(s)))
    assert got.shape == (M, Kp // 2)
    assert np.array_equal(got, _padded_reference(oracle.quantize(X.astype(np.float32), s), Kp))
    W = (rng.standard_normal((M, K)) * 0.02).astype(np.float32)
    Wq, s_w = mkq.mkq_pack_weights_int4_padded(to_dev(W))
    wc, sw = oracle.quantize_weights(W)
    assert np.array_equal(to_np(s_w), sw)
    assert np.array_equal(to_np(Wq).reshape(M, Kp // 2), _padded_reference(wc, Kp))


# the four linears of a TinyBERT4 layer (hidden 312, FFN 1200) at ragged token counts
@pytest.mark.parametrize("M,K,N", [(440, 312, 936), (537, 312, 312), (1691, 312, 1200), (681, 1200, 312),
                                   (16, 312, 1200), (4096, 1200, 312)])
def test_linear_matches_the_oracle_on_the_real_columns(mkq, M, K, N):
    rng = np.random.default_rng(K + N + M)
    X = wl.outlier_activations(rng, M, K, 0.01, "x8").astype(np.float16)
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    Kp = mkq.mkq_padded_k(K)
    a = mkq.mkq_quantize_padded(to_dev(X), s_x)
    Wq, s_w = mkq.mkq_pack_weights_int4_padded(to_dev(W))
    r = mkq.mkq_linear_int4(a, s_x, Wq, s_w, to_dev(b), N, Kp, mkq.MKQ_F32, want_acc=True)
    codes = oracle.quantize(X.astype(np.float32), s_x)
    wc, sw = oracle.quantize_weights(W)
    ref = oracle.linear_int4(codes, s_x, wc, sw, b)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]), ref["y"])
    r = mkq.mkq_linear_int4(a, s_x, Wq, s_w, to_dev(b), N, Kp, mkq.MKQ_F16)
    ref = oracle.linear_int4(codes, s_x, wc, sw, b, out_dtype=oracle.F16)
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
