"""Shared helpers for the GPU parity tests (no method arithmetic here)."""
import numpy as np

RTOL = {0: 1e-3, 1: 1e-2, 2: 1e-2}  # by MKQ dtype code: binary32 / binary16 / bfloat16


def to_dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def to_np(t):
    import torch
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy()


def assert_float_close(gpu, ref, rtol, what=""):
    """|gpu - ref| <= rtol*|ref| + rtol*rms(ref), element-wise."""
    gpu = np.asarray(gpu, np.float64)
    ref = np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
    bad = np.abs(gpu - ref) > rtol * np.abs(ref) + rtol * rms
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} outside tolerance; "
                           f"max abs err {np.abs(gpu - ref).max():.3e}, rms(ref) {rms:.3e}")


def assert_codes_match_with_tie_band(gpu_codes, ref_codes, pre_round, s, band=2.0 ** -10, max_frac=1e-4,
                                     what=""):
    """Codes decided from a float that went through a transcendental (GELU) may
    differ by one step only where the pre-rounding value sits within `band` of a
    rounding boundary; such cases must be rare."""
    gpu_codes = np.asarray(gpu_codes, np.int32)
    ref_codes = np.asarray(ref_codes, np.int32)
    diff = gpu_codes != ref_codes
    if not diff.any():
        return 0
    v = np.asarray(pre_round, np.float64) / float(s)
    frac = np.abs(v - np.floor(v) - 0.5)
    ok = (np.abs(gpu_codes - ref_codes) <= 1) & (frac <= band)
    assert not (diff & ~ok).any(), f"{what}: {int((diff & ~ok).sum())} codes differ outside the tie band"
    assert diff.mean() <= max_frac, f"{what}: {diff.mean():.2e} of codes differ (tie band)"
    return int(diff.sum())
