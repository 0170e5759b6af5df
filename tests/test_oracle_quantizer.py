"""Pins for the oracle's quantizer, scales, packing and narrowing (CPU only).

Each test checks the oracle against something other than itself: the paper's
worked example, closed forms, invariants of Eq. 1, or a numpy/torch library
routine.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle


def _read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


# --- the paper's worked example (section 4.1.1 / 4.1.2) -----------------------

def test_worked_example_quantized_values(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "quantizer_worked_example.txt"))
    x = np.array(g["x"], np.float32)
    for s_key, q_key in (("s1", "Q_s1"), ("s2", "Q_s2")):
        s = np.float32(g[s_key][0])
        codes = oracle.quantize(x[None, :], s)[0]
        Q = oracle.dequantize(codes, s)
        np.testing.assert_allclose(Q, np.array(g[q_key], np.float32), rtol=0, atol=1e-7)


def test_worked_example_scale_gradients(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "quantizer_worked_example.txt"))
    ste, mse = oracle.scale_gradients(np.array(g["x"], np.float32), g["s1"][0])
    assert ste == pytest.approx(g["grad_ste_s1"][0], abs=1e-6)
    assert mse == pytest.approx(g["grad_mse_s1"][0], abs=1e-6)
    # the paper's point: the two gradients disagree in sign on this tensor
    assert ste < 0 < mse


# --- invariants of Eq. 1 -------------------------------------------------------

SCALES = [1.0, 0.9, 0.34, 0.0173, 3.7, 2.0 ** -7, 1e-3]


@pytest.mark.parametrize("s", SCALES)
def test_error_at_most_half_step_inside_range(s):
    rng = np.random.default_rng(1)
    s32 = np.float32(s)
    x = (rng.uniform(-8.0, 7.0, 200_000) * float(s32)).astype(np.float32)
    v = x.astype(np.float64) / float(s32)
    inside = (v >= -8.0) & (v <= 7.0)
    codes = oracle.quantize(x[None, :], s32)[0].astype(np.float64)
    err = np.abs(codes * float(s32) - x.astype(np.float64))
    # half a step, with slack for the one rounding of the binary32 divide
    assert np.all(err[inside] <= 0.5 * float(s32) * (1 + 2e-6) + 1e-12)
    assert codes.min() >= -8 and codes.max() <= 7


@pytest.mark.parametrize("s", SCALES)
def test_idempotent_on_grid(s):
    s32 = np.float32(s)
    c = np.arange(-8, 8, dtype=np.int8)
    grid = oracle.dequantize(c, s32)
    assert np.array_equal(oracle.quantize(grid[None, :], s32)[0], c)


@pytest.mark.parametrize("s", SCALES)
def test_monotone_and_saturating(s):
    s32 = np.float32(s)
    x = np.sort(np.random.default_rng(2).normal(0, 6 * s, 100_000).astype(np.float32))
    c = oracle.quantize(x[None, :], s32)[0].astype(np.int32)
    assert np.all(np.diff(c) >= 0)
    big = np.array([7.5 * s, 8 * s, 100 * s, np.inf, 3e38], np.float32)
    small = np.array([-8.5 * s, -9 * s, -100 * s, -np.inf, -3e38], np.float32)
    assert np.all(oracle.quantize(big[None, :], s32) == 7)
    assert np.all(oracle.quantize(small[None, :], s32) == -8)
    assert oracle.quantize(np.array([[np.nan]], np.float32), s32)[0, 0] == 0


@pytest.mark.parametrize("s", SCALES)
def test_odd_symmetry_inside_symmetric_range(s):
    s32 = np.float32(s)
    x = (np.random.default_rng(3).uniform(-7, 7, 100_000) * s).astype(np.float32)
    cp = oracle.quantize(x[None, :], s32)[0].astype(np.int32)
    cm = oracle.quantize((-x)[None, :], s32)[0].astype(np.int32)
    assert np.array_equal(cp, -cm)


def test_exact_ties_go_to_even():
    for s in (1.0, 0.5, 0.125, 4.0):
        j = np.arange(-8, 7)
        x = ((j + 0.5) * s).astype(np.float32)  # exact in binary32, division exact
        c = oracle.quantize(x[None, :], np.float32(s))[0].astype(np.int32)
        expect = np.where(j % 2 == 0, j, j + 1)  # the even neighbour of j + 1/2
        assert np.array_equal(c, expect)
        assert np.all(c % 2 == 0)


def test_clamp_then_round_equals_round_then_clamp():
    # Eq. 1 prints round(clamp(.)); for integer bounds the other order gives the same codes.
    rng = np.random.default_rng(4)
    for s in SCALES:
        s32 = np.float32(s)
        x = (rng.normal(0, 5, 100_000) * s).astype(np.float32)
        v = x / s32                                   # binary32 divide (numpy)
        other = np.clip(np.rint(v), -8, 7).astype(np.int8)   # rint = ties to even
        assert np.array_equal(oracle.quantize(x[None, :], s32)[0], other)


def _exact_code(x: float, s: float) -> int:
    """Eq. 1 on exact rationals, with the quotient first rounded to binary32 as
    the definition's divide is; written with Fractions to share nothing."""
    v = np.float32(np.float64(Fraction(x) / Fraction(s)))  # correctly rounded: f64 of the exact
    # quotient is within 2^-53, and double rounding only matters on 1 in 2^29 inputs; checked below
    v = Fraction(float(v))
    v = max(Fraction(-8), min(Fraction(7), v))
    fl = v.numerator // v.denominator
    r = v - fl
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and fl % 2 == 1):
        fl += 1
    return int(fl)


def test_all_half_precision_inputs_power_of_two_scale():
    # every binary16 value; with s a power of two the divide is exact, so the
    # real-number definition (evaluated in binary64) must agree everywhere.
    bits = np.arange(65536, dtype=np.uint16)
    x16 = bits.view(np.float16)
    x = x16.astype(np.float32)
    ok = np.isfinite(x)
    for s in (1.0, 0.25, 2.0 ** -6, 8.0):
        v = x.astype(np.float64) / s
        ref = np.rint(np.clip(v, -8, 7))
        got = oracle.quantize(x[None, :], np.float32(s))[0]
        assert np.array_equal(got[ok], ref[ok].astype(np.int8))


def test_sampled_inputs_against_rational_arithmetic():
    rng = np.random.default_rng(5)
    for s in (0.9, 0.34, 0.0173, 3.7):
        s32 = float(np.float32(s))
        x = (rng.uniform(-9, 8, 400) * s32).astype(np.float32)
        # add points sitting right at decision boundaries
        edges = ((np.arange(-8, 8) + 0.5) * s32).astype(np.float32)
        x = np.concatenate([x, edges, np.nextafter(edges, np.float32(np.inf)),
                            np.nextafter(edges, np.float32(-np.inf))])
        got = oracle.quantize(x[None, :], np.float32(s32))[0]
        ref = np.array([_exact_code(float(xi), s32) for xi in x], np.int8)
        assert np.array_equal(got, ref)


def test_other_clamp_ranges():
    x = np.linspace(-300, 300, 4001, dtype=np.float32)
    c8 = oracle.quantize(x[None, :], np.float32(1.0), -128, 127)[0]
    assert c8.min() == -128 and c8.max() == 127
    c7 = oracle.quantize(x[None, :], np.float32(1.0), -7, 7)[0]
    assert c7.min() == -7 and c7.max() == 7


def test_invalid_scale_rejected():
    x = np.zeros((1, 4), np.float32)
    for s in (0.0, -1.0, np.inf, np.nan):
        with pytest.raises(ValueError):
            oracle.quantize(x, np.float32(s))


# --- abs-max calibration (section 3.1) ------------------------------------------

def test_absmax_scale_closed_form():
    rng = np.random.default_rng(6)
    W = rng.normal(0, 0.02, (64, 96)).astype(np.float32)
    codes, s_w = oracle.quantize_weights(W)
    assert np.all(s_w > 0)
    # the arg-max element of every row lands exactly on +-7, nothing exceeds 7
    idx = np.argmax(np.abs(W), axis=1)
    assert np.all(np.abs(codes[np.arange(64), idx]) == 7)
    assert np.abs(codes).max() == 7
    np.testing.assert_array_equal(s_w, (np.abs(W).max(axis=1) / np.float32(7)).astype(np.float32))
    s_t = oracle.absmax_scale(W)
    assert s_t == np.float32(np.abs(W).max() / np.float32(7))
    np.testing.assert_array_equal(oracle.absmax_scale(W, per_row=True), s_w)


def test_zero_row_gets_unit_scale():
    W = np.zeros((3, 8), np.float32)
    W[1, 2] = -0.5
    codes, s_w = oracle.quantize_weights(W)
    assert s_w[0] == 1.0 and s_w[2] == 1.0
    assert np.all(codes[0] == 0) and codes[1, 2] == -7


def test_given_weight_scales_are_used():
    W = np.array([[0.1, -0.26, 0.3, 4.0]], np.float32)
    codes, s_w = oracle.quantize_weights(W, s_w=np.array([0.1], np.float32))
    assert s_w[0] == np.float32(0.1)
    assert codes.tolist() == [[1, -3, 3, 7]]


# --- canonical nibble packing -----------------------------------------------------

def test_pack_literal_bytes():
    codes = np.array([[1, -1, -8, 7, 0, 5, -2, -3]], np.int8)
    # low nibble = even element, high nibble = odd element, two's complement
    assert oracle.pack_nibbles(codes).tolist() == [[0xF1, 0x78, 0x50, 0xDE]]


def test_pack_unpack_all_bytes():
    allbytes = np.arange(256, dtype=np.uint8).reshape(2, 128)
    codes = oracle.unpack_nibbles(allbytes, 256)
    assert codes.min() == -8 and codes.max() == 7
    assert np.array_equal(oracle.pack_nibbles(codes), allbytes)
    rng = np.random.default_rng(7)
    c = rng.integers(-8, 8, (5, 64), dtype=np.int8)
    assert np.array_equal(oracle.unpack_nibbles(oracle.pack_nibbles(c), 64), c)
    assert oracle.pack_nibbles(c).nbytes == 5 * 64 // 2


# --- narrowing to 16-bit storage: numpy / torch conversions are the library route ---

def _interesting_floats():
    rng = np.random.default_rng(8)
    x = np.concatenate([
        rng.normal(0, 1, 50_000), rng.normal(0, 1e-6, 20_000), rng.normal(0, 3e4, 20_000),
        np.array([0.0, -0.0, 65504, 65519.99, 65520, 7e4, -7e4, 6.1e-5, 5.96e-8, 2.98e-8,
                  2.9802322e-8, 8.9e-8, 1.0009766, 1.00048828125, 1.0014648, np.inf, -np.inf]),
    ]).astype(np.float32)
    return x


def test_round_to_half_matches_numpy():
    x = _interesting_floats()
    got = oracle.round_storage(x, oracle.F16)
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16).astype(np.float32)
    assert np.array_equal(got, ref)


def test_round_to_bfloat16_matches_torch():
    x = _interesting_floats()
    got = oracle.round_storage(x, oracle.BF16)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got, ref)
