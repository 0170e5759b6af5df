"""Host check of the bound behind the division-free code decision of the GEMM epilogues: with rs = RN(1/s)
and q = RN(x * rs) in binary32, whenever clamp(q) lies farther than the margin from every rounding boundary
k + 1/2, the correctly rounded quotient x / s gives the same code.  Checked on random values and on values
placed a few ulps around every boundary, for steps across the range the fast path accepts.  The same for the
biased form the packed eight-value quantizer uses: v = fma(x, rs, 2^(bits-1)) with one rounding, rounded, then
clamped to [0, 2^bits - 1]."""
import numpy as np
import pytest


def _codes(v, lo, hi):
    v = np.where(np.isnan(v), np.float32(0), v)
    return np.rint(np.clip(v, np.float32(lo), np.float32(hi))).astype(np.int32)


@pytest.mark.parametrize("bits,lo,hi,margin", [(4, -8, 7, 4.0e-6), (8, -128, 127, 5.0e-5)])
def test_far_from_a_boundary_the_reciprocal_decides_like_the_division(bits, lo, hi, margin):
    rng = np.random.default_rng(bits)
    steps = np.concatenate([rng.uniform(1e-3, 2.0, 40), 2.0 ** rng.uniform(-99, 99, 40),
                            [0.3, 1.0 / 3.0, 0.1, 7.0, 2.0 ** -100, 2.0 ** 100]]).astype(np.float32)
    thr = np.float32(0.5) - np.float32(margin)
    flagged = total = 0
    with np.errstate(over="ignore", invalid="ignore", under="ignore"):
        for s in steps:
            rs = np.float32(1.0) / s
            # random quotients over and beyond the clamp range, and values around every boundary
            q = rng.uniform(lo - 2, hi + 2, 20000)
            b = np.arange(lo - 1, hi + 1) + 0.5
            near = (b[:, None] + np.linspace(-8, 8, 33)[None, :] * 2.0 ** -22 * np.maximum(1, np.abs(b))[:, None]).ravel()
            x = (np.concatenate([q, near]) * np.float64(s)).astype(np.float32)
            x = np.concatenate([x, np.nextafter(x, np.float32(np.inf)), np.nextafter(x, np.float32(-np.inf)),
                                np.float32([0.0, np.inf, -np.inf, np.nan, 3e38, -3e38])])
            v = np.clip(np.where(np.isnan(x * rs), np.float32(0), x * rs), np.float32(lo), np.float32(hi))
            far = np.abs(v - np.rint(v)) <= thr
            exact = _codes(x / s, lo, hi)
            assert np.array_equal(np.rint(v).astype(np.int32)[far], exact[far]), f"s={s}"
            flagged += int((~far).sum())
            total += x.size
    assert flagged < total  # the fast path decides almost everything; the rest takes the division


def _fma32(x, rs, bias):
    """fma(x, rs, bias) in binary32 with a single rounding, for binary32 x and rs and a small integer bias: the
    product is exact in binary64 (48 bits), the sum is split into its binary64 value and its exact residual
    (two-sum), and where the binary64 value sits exactly half way between two binary32 numbers the residual
    decides the direction."""
    p = x.astype(np.float64) * np.float64(rs)
    b = np.float64(bias)
    s = p + b
    bb = s - p
    err = (p - (s - bb)) + (b - bb)
    v = s.astype(np.float32)
    d = s - v.astype(np.float64)                       # exact
    fin = np.isfinite(v) & np.isfinite(s)
    up = np.nextafter(v, np.float32(np.inf)).astype(np.float64)
    dn = np.nextafter(v, np.float32(-np.inf)).astype(np.float64)
    # the conversion was a tie that went to even although the true sum lies beyond the midpoint
    tie_up = fin & (d > 0) & (d == (up - v.astype(np.float64)) / 2) & (err > 0)
    tie_dn = fin & (d < 0) & (-d == (v.astype(np.float64) - dn) / 2) & (err < 0)
    # ... or it was not a tie but the residual moves the sum onto or across the midpoint: cannot happen, the
    # residual is below half an ulp of binary64 and the midpoints are binary64 numbers
    v = np.where(tie_up, up.astype(np.float32), v)
    v = np.where(tie_dn, dn.astype(np.float32), v)
    return v


def test_fma32_emulation_against_exact_rationals():
    from fractions import Fraction
    rng = np.random.default_rng(5)
    x = (rng.uniform(-3, 3, 300) * 2.0 ** rng.integers(-30, 3, 300)).astype(np.float32)
    rs = np.float32(1.0) / np.float32(0.3)
    got = _fma32(x, rs, 8.0)
    for xi, gi in zip(x, got):
        exact = Fraction(float(xi)) * Fraction(float(rs)) + 8
        lo, hi = np.nextafter(gi, np.float32(-np.inf)), np.nextafter(gi, np.float32(np.inf))
        assert abs(Fraction(float(gi)) - exact) <= min(abs(Fraction(float(lo)) - exact), abs(Fraction(float(hi)) - exact))


@pytest.mark.parametrize("bits,lo,hi,margin", [(4, -8, 7, 4.0e-6), (8, -128, 127, 5.0e-5)])
def test_biased_fma_form_decides_like_the_division(bits, lo, hi, margin):
    rng = np.random.default_rng(100 + bits)
    steps = np.concatenate([rng.uniform(1e-3, 2.0, 40), 2.0 ** rng.uniform(-99, 99, 40),
                            [0.3, 1.0 / 3.0, 0.1, 7.0, 2.0 ** -100, 2.0 ** 100]]).astype(np.float32)
    thr = np.float32(0.5) - np.float32(margin)
    bias, top = np.float32(2 ** (bits - 1)), np.float32(2 ** bits - 1)
    flagged = total = 0
    with np.errstate(over="ignore", invalid="ignore", under="ignore"):
        for s in steps:
            rs = np.float32(1.0) / s
            q = rng.uniform(lo - 2, hi + 2, 20000)
            b = np.arange(lo - 1, hi + 1) + 0.5
            near = (b[:, None] + np.linspace(-8, 8, 33)[None, :] * 2.0 ** -22 * np.maximum(1, np.abs(b))[:, None]).ravel()
            x = (np.concatenate([q, near]) * np.float64(s)).astype(np.float32)
            x = np.concatenate([x, np.nextafter(x, np.float32(np.inf)), np.nextafter(x, np.float32(-np.inf)),
                                np.float32([0.0, -0.0, np.inf, -np.inf, np.nan, 3e38, -3e38])])
            v = _fma32(x, rs, bias)
            r = np.rint(v)
            far = np.abs(v - r) <= thr                 # False for NaN and for infinities (inf - inf)
            code = (np.clip(r, np.float32(0), top) - bias)
            exact = _codes(x / s, lo, hi)
            assert np.array_equal(code[far].astype(np.int32), exact[far]), f"s={s}"
            assert not far[np.isnan(x) | np.isinf(x)].any()
            flagged += int((~far).sum())
            total += x.size
    assert flagged < total // 4
