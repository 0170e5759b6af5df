"""Host check of the bound behind the division-free code decision of the GEMM epilogues: with rs = RN(1/s)
and q = RN(x * rs) in binary32, whenever clamp(q) lies farther than the margin from every rounding boundary
k + 1/2, the correctly rounded quotient x / s gives the same code.  Checked on random values and on values
placed a few ulps around every boundary, for steps across the range the fast path accepts."""
import numpy as np
import pytest


def _codes(v, lo, hi):
    v = np.where(np.isnan(v), np.float32(0), v)
    return np.rint(np.clip(v, np.float32(lo), np.float32(hi))).astype(np.int32)


@pytest.mark.parametrize("bits,lo,hi,margin", [(4, -8, 7, 2.0e-6), (8, -128, 127, 3.0e-5)])
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
