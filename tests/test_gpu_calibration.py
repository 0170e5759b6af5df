"""GPU parity of the scale machinery (sections 3.1 and 4.1) against the oracle: the
percentile step is an exact order statistic (bit-exact); the scale-gradient sums are
binary64 sums whose order differs, compared to 1e-10 of the sum of the terms' magnitudes."""
import numpy as np
import pytest

import oracle
from helpers import to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m


def _activations(M, K, seed, dtype):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    x.flat[:: 101] *= 8  # outliers beyond the clamp
    return x.astype(dtype)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("M,K,bits,s", [(1, 8, 4, 0.5), (37, 200, 4, 0.34), (1024, 768, 4, 0.34),
                                         (1024, 768, 8, 0.02), (4096, 3072, 4, 0.21)])
def test_scale_gradients(mkq, M, K, bits, s, dtype):
    x = _activations(M, K, M + K + bits, dtype)
    g = to_np(mkq.mkq_scale_gradients(to_dev(x), s, bits))
    qmin, qmax = (-8, 7) if bits == 4 else (-128, 127)
    xf = x.astype(np.float32)
    ste, mse = oracle.scale_gradients(xf, s, qmin, qmax)
    c = oracle.quantize(xf, np.float32(s), qmin, qmax).astype(np.float64)
    xd, sd = xf.astype(np.float64), float(np.float32(s))
    mag_ste = np.abs(-xd / sd + c).sum()
    mag_mse = np.abs(2 * (sd * c - xd) * c).sum()
    assert abs(g[0] - ste) <= 1e-10 * mag_ste + 1e-12
    assert abs(g[1] - mse) <= 1e-10 * mag_mse + 1e-12


def test_scale_gradients_worked_example_and_strided_rows(mkq):
    # section 4.1: x = (0.2, 0.9), s = 1 -> -0.1 and +0.2 (padded with on-grid zeros, which add nothing)
    x = np.zeros((1, 8), np.float32)
    x[0, :2] = (0.2, 0.9)
    g = to_np(mkq.mkq_scale_gradients(to_dev(x), 1.0))
    assert g[0] == pytest.approx(-0.1, abs=1e-6) and g[1] == pytest.approx(0.2, abs=1e-6)
    big = _activations(64, 512, 5, np.float32)
    view = to_dev(big)[:, 128:384]
    g = to_np(mkq.mkq_scale_gradients(view, 0.3))
    ste, mse = oracle.scale_gradients(np.ascontiguousarray(big[:, 128:384]), 0.3)
    assert g[0] == pytest.approx(ste, rel=1e-9) and g[1] == pytest.approx(mse, rel=1e-9)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("M,K", [(1, 8), (13, 72), (1024, 768), (4096, 3072)])
def test_percentile_scale_bit_exact(mkq, M, K, dtype):
    x = _activations(M, K, 3 * M + K, dtype)
    if M * K > 100:
        x.flat[7] = np.nan
    for ppm, bits in ((100, 8), (100, 4), (20000, 4), (0, 4), (1000000, 8), (500000, 4)):
        s = float(to_np(mkq.mkq_percentile_scale(to_dev(x), ppm, bits))[0])
        ref, _ = oracle.percentile_scale(x.astype(np.float32), ppm, 7 if bits == 4 else 127)
        assert s == ref, (ppm, bits)


def test_percentile_scale_ties_zeros_and_absmax(mkq):
    ties = np.array([[3, -3, 3, 1, 0, -3, 0, 0]], np.float32)
    for ppm in (0, 250000, 375000, 500000, 625000, 1000000):
        s = float(to_np(mkq.mkq_percentile_scale(to_dev(ties), ppm))[0])
        assert s == oracle.percentile_scale(ties, ppm)[0]
    z = np.zeros((4, 16), np.float32)
    assert float(to_np(mkq.mkq_percentile_scale(to_dev(z)))[0]) == 1.0
    x = _activations(128, 768, 9, np.float16)
    s0 = float(to_np(mkq.mkq_percentile_scale(to_dev(x), 0))[0])
    assert s0 == float(to_np(mkq.mkq_absmax_scale(to_dev(x)))[0])


def test_percentile_step_feeds_the_quantizer(mkq):
    """Calibrate, then quantize with the calibrated step: about top_ppm of the codes clip."""
    x = _activations(2048, 768, 11, np.float16)
    s = float(to_np(mkq.mkq_percentile_scale(to_dev(x), 20000))[0])  # top 2 %
    codes = oracle.unpack_nibbles(to_np(mkq.mkq_quantize(to_dev(x), s)), 768)
    ref = oracle.quantize(x.astype(np.float32), np.float32(s))
    assert np.array_equal(codes, ref)
    clipped = (np.abs(x.astype(np.float32)) >= 7 * s).mean()
    assert 0.015 < clipped < 0.025
