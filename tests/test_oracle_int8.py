"""Pins of the oracle at the 8-bit range (Eq. 1 with k = 8, the int8 comparison column of
Table 2): the same oracle functions with qmin, qmax = -128, 127, checked against exact
rational arithmetic, closed forms and numpy integer arithmetic."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

Q8 = dict(qmin=-128, qmax=127)


def _exact_code8(x: float, s: float) -> int:
    v = Fraction(float(np.float32(np.float64(Fraction(x) / Fraction(s)))))
    v = max(Fraction(-128), min(Fraction(127), v))
    fl = v.numerator // v.denominator
    r = v - fl
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return int(fl)


def test_quantize8_against_rational_arithmetic():
    rng = np.random.default_rng(15)
    for s in (1.0, 0.031, 0.0009):
        s32 = float(np.float32(s))
        x = (rng.uniform(-140, 140, 600) * s32).astype(np.float32)
        edges = ((np.arange(-128, 127) + 0.5) * s32).astype(np.float32)
        x = np.concatenate([x, edges, np.nextafter(edges, np.float32(np.inf)),
                            np.nextafter(edges, np.float32(-np.inf))])
        got = oracle.quantize(x[None, :], np.float32(s32), **Q8)[0]
        ref = np.array([_exact_code8(float(xi), s32) for xi in x], np.int8)
        assert np.array_equal(got, ref)


def test_quantize8_saturates_and_is_identity_on_the_grid():
    grid = np.arange(-128, 128, dtype=np.float32)
    assert np.array_equal(oracle.quantize(grid[None, :], np.float32(1.0), **Q8)[0], grid.astype(np.int8))
    far = np.array([[-1e9, -128.6, 127.4, 127.6, 1e9, np.nan]], np.float32)
    assert oracle.quantize(far, np.float32(1.0), **Q8)[0].tolist() == [-128, -128, 127, 127, 127, 0]
    # ties to even, both signs
    ties = np.array([[0.5, 1.5, 2.5, -0.5, -1.5, 126.5, -127.5]], np.float32)
    assert oracle.quantize(ties, np.float32(1.0), **Q8)[0].tolist() == [0, 2, 2, 0, -2, 126, -128]


def test_weight_steps_8bit_closed_form():
    rng = np.random.default_rng(16)
    W = rng.normal(0, 0.02, (40, 64)).astype(np.float32)
    codes, s_w = oracle.quantize_weights(W, **Q8)
    np.testing.assert_array_equal(s_w, (np.abs(W).max(axis=1) / np.float32(127)).astype(np.float32))
    idx = np.argmax(np.abs(W), axis=1)
    assert np.all(np.abs(codes[np.arange(40), idx].astype(np.int32)) == 127)
    # no code below -127: abs-max calibration is symmetric
    assert codes.min() >= -127 and codes.max() <= 127
    # an 8-bit grid is 127/7 times finer: reconstruction error at most half a step
    assert np.all(np.abs(codes * s_w[:, None] - W) <= s_w[:, None] * 0.5000001)


@pytest.mark.parametrize("M,N,K", [(5, 7, 64), (33, 17, 320)])
def test_gemm_full_byte_range_matches_numpy_int64(M, N, K):
    rng = np.random.default_rng(M * K)
    a = rng.integers(-128, 128, (M, K), dtype=np.int8)
    w = rng.integers(-128, 128, (N, K), dtype=np.int8)
    ref = a.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(oracle.gemm_codes(a, w), ref)


@pytest.mark.parametrize("K", [64, 4096, 65472])
def test_accumulator_bound_8bit(K):
    lo = np.full((2, K), -128, np.int8)
    hi = np.full((3, K), 127, np.int8)
    assert np.all(oracle.gemm_codes(lo, lo) == (1 << 14) * K)  # < 2^31 for K < 131072
    assert np.all(oracle.gemm_codes(lo, hi) == -128 * 127 * K)


def test_linear_8bit_is_the_composition_of_its_pieces_and_closer_to_float():
    rng = np.random.default_rng(17)
    M, K, N = 24, 256, 40
    X = rng.standard_normal((M, K)).astype(np.float32)
    W = (rng.standard_normal((N, K)) * 0.05).astype(np.float32)
    b = rng.standard_normal(N).astype(np.float32)
    s_x8 = oracle.absmax_scale(X, qmax=127)
    a8 = oracle.quantize(X, s_x8, **Q8)
    w8, s_w8 = oracle.quantize_weights(W, **Q8)
    r8 = oracle.linear_int4(a8, s_x8, w8, s_w8, b, **Q8)
    assert np.array_equal(r8["acc"], a8.astype(np.int64) @ w8.astype(np.int64).T)
    assert np.array_equal(r8["y"], oracle.epilogue(r8["acc"], s_x8, s_w8, b))
    exact = X.astype(np.float64) @ W.astype(np.float64).T + b
    s_x4 = oracle.absmax_scale(X)
    w4, s_w4 = oracle.quantize_weights(W)
    r4 = oracle.linear_int4(oracle.quantize(X, s_x4), s_x4, w4, s_w4, b)
    e8 = np.sqrt(np.mean((r8["y"] - exact) ** 2))
    e4 = np.sqrt(np.mean((r4["y"] - exact) ** 2))
    assert e8 < e4 / 8  # steps are 127/7 = 18x finer in both operands
