"""Pins of the oracle's scale machinery: the two scale gradients of section 4.1 beyond the
paper's worked example (closed forms, numerical derivative of the quantization error, numpy
re-evaluation) and the percentile calibration of section 3.1 (numpy's order statistics,
closed forms on ranked data, reduction to abs-max)."""
import numpy as np
import pytest

import oracle


# --- scale gradients (section 4.1) ---------------------------------------------------

def test_gradients_vanish_on_the_grid():
    # x exactly on the quantization grid: Q[x] = x, so both sums are 0
    x = (np.arange(-8, 8) * 0.25).astype(np.float32)
    ste, mse = oracle.scale_gradients(x, 0.25)
    assert ste == 0.0 and mse == 0.0


def test_gradients_on_clipped_values_closed_form():
    # every element beyond the clamp: round(clamp(x/s)) = 7, Q[x] = 7s
    s = 0.5
    x = np.array([5.0, 6.0, 10.0], np.float32)
    ste, mse = oracle.scale_gradients(x, s)
    assert ste == pytest.approx(sum(-v / s + 7 for v in (5.0, 6.0, 10.0)), rel=1e-12)
    assert mse == pytest.approx(sum(2 * (7 * s - v) * 7 for v in (5.0, 6.0, 10.0)), rel=1e-12)
    # and on the negative side the code is -8
    ste, mse = oracle.scale_gradients(-x, s)
    assert mse == pytest.approx(sum(2 * (-8 * s + v) * -8 for v in (5.0, 6.0, 10.0)), rel=1e-12)


def test_mse_gradient_is_the_derivative_of_the_squared_error():
    """Section 4.1.2 defines it as d/ds sum (Q[x]-x)^2 with the codes held fixed: away from rounding
    boundaries that is the true derivative, so a central difference must reproduce it."""
    rng = np.random.default_rng(31)
    x = rng.normal(0, 1.0, 4000).astype(np.float32)
    s = 0.31
    v = x.astype(np.float64) / s
    frac = np.abs(v - np.floor(v) - 0.5)
    x = x[frac > 1e-3]  # keep clear of the ties so the codes do not change under s +- h
    h = 1e-7

    def err(sv):
        c = np.rint(np.clip(x.astype(np.float64) / sv, -8, 7))
        return np.sum((sv * c - x) ** 2)

    _, mse = oracle.scale_gradients(x, s)
    assert mse == pytest.approx((err(s + h) - err(s - h)) / (2 * h), rel=1e-5)


@pytest.mark.parametrize("qmin,qmax", [(-8, 7), (-128, 127)])
def test_gradients_match_numpy_float64(qmin, qmax):
    rng = np.random.default_rng(32)
    x = (rng.standard_t(3, 20000) * 0.7).astype(np.float32)
    s = np.float32(0.21 if qmax == 7 else 0.013)
    c = oracle.quantize(x[None, :], s, qmin, qmax)[0].astype(np.float64)
    xd, sd = x.astype(np.float64), float(s)
    ste, mse = oracle.scale_gradients(x, s, qmin, qmax)
    assert ste == pytest.approx(np.sum(-xd / sd + c), rel=1e-11, abs=1e-9)
    assert mse == pytest.approx(np.sum(2 * (sd * c - xd) * c), rel=1e-11, abs=1e-9)
    # the STE sum of in-range elements is a sum of rounding residuals, each at most 1/2
    inside = (xd / sd > qmin) & (xd / sd < qmax)
    assert np.abs(-xd[inside] / sd + c[inside]).max() <= 0.5 + 1e-6


# --- percentile calibration (section 3.1) --------------------------------------------

def test_percentile_on_ranked_data_closed_form():
    # |x| = 1 .. 20000 shuffled, signs mixed: the k-th largest is n + 1 - k
    n = 20000
    rng = np.random.default_rng(33)
    x = rng.permutation(np.arange(1, n + 1)).astype(np.float32) * rng.choice([-1.0, 1.0], n).astype(np.float32)
    for ppm, k in ((100, 2), (1000, 20), (500000, 10000), (1000000, 20000), (1, 1), (0, 1)):
        s, t = oracle.percentile_scale(x, ppm)
        assert t == n + 1 - k
        assert s == np.float32(np.float32(t) / np.float32(7))


@pytest.mark.parametrize("n", [1, 7, 9999, 10000, 250001])
def test_percentile_matches_numpy_partition(n):
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n).astype(np.float32)
    if n > 10:
        x[3] = np.nan  # ranked as 0
    for ppm, qmax in ((100, 127), (100, 7), (20000, 7)):
        k = max(1, n * ppm // 10 ** 6)
        a = np.nan_to_num(np.abs(x), nan=0.0)
        expect = np.partition(a, n - k)[n - k]
        s, t = oracle.percentile_scale(x, ppm, qmax)
        assert t == expect and s == np.float32(expect / np.float32(qmax))


def test_percentile_reduces_to_absmax_and_handles_ties_and_zeros():
    rng = np.random.default_rng(34)
    x = rng.standard_normal((50, 64)).astype(np.float32)
    s, t = oracle.percentile_scale(x, 1)  # k = max(1, 0) = 1: the maximum
    assert s == oracle.absmax_scale(x) and t == np.abs(x).max()
    ties = np.array([3, -3, 3, 1, 0, -3], np.float32)
    assert oracle.percentile_scale(ties, 500000)[1] == 3.0   # k = 3: third largest is still 3
    assert oracle.percentile_scale(ties, 700000)[1] == 3.0   # k = 4
    assert oracle.percentile_scale(ties, 900000)[1] == 1.0   # k = 5
    assert oracle.percentile_scale(np.zeros(10, np.float32), 100) == (1.0, 0.0)
