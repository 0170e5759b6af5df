"""GPU parity: quantizer, calibration and weight packing vs the CPU oracle (bit-exact)."""
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


def _special_values(rng, M, K, s):
    x = rng.normal(0, 3 * s, (M, K)).astype(np.float32)
    flat = x.reshape(-1)
    ties = ((np.arange(-9, 9) + 0.5) * s).astype(np.float32)
    flat[: ties.size] = ties
    flat[ties.size: ties.size + 6] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-30]
    edges = np.nextafter(ties, np.float32(np.inf))
    flat[40: 40 + edges.size] = edges
    return x


@pytest.mark.parametrize("M,K", [(1, 32), (128, 768), (77, 1056), (1024, 3072), (5, 64)])
@pytest.mark.parametrize("s", [0.34, 0.5, 0.0173])
def test_quantize_f32_bit_exact(mkq, M, K, s):
    rng = np.random.default_rng(M + K)
    x = _special_values(rng, M, K, s) if M * K >= 64 else rng.normal(0, 1, (M, K)).astype(np.float32)
    q = to_np(mkq.mkq_quantize(to_dev(x), s))
    ref = oracle.pack_nibbles(oracle.quantize(x, np.float32(s)))
    assert np.array_equal(q, ref)


@pytest.mark.parametrize("M,K", [(128, 768), (33, 96)])
def test_quantize_f16_bit_exact(mkq, M, K):
    rng = np.random.default_rng(7)
    x = rng.normal(0, 1.5, (M, K)).astype(np.float16)
    q = to_np(mkq.mkq_quantize(to_dev(x), 0.34))
    ref = oracle.pack_nibbles(oracle.quantize(x.astype(np.float32), np.float32(0.34)))
    assert np.array_equal(q, ref)


def test_quantize_all_half_values(mkq):
    x = np.arange(65536, dtype=np.uint16).view(np.float16).reshape(64, 1024)
    for s in (1.0, 0.34, 0.0173):
        q = to_np(mkq.mkq_quantize(to_dev(x), s))
        ref = oracle.pack_nibbles(oracle.quantize(x.astype(np.float32), np.float32(s)))
        assert np.array_equal(q, ref)


def test_quantize_strided_rows_and_empty(mkq):
    import torch
    rng = np.random.default_rng(3)
    big = rng.normal(0, 1, (16, 256)).astype(np.float32)
    xd = to_dev(big)[:, :128]  # ldx = 256, K = 128
    q = to_np(mkq.mkq_quantize(xd, 0.3))
    assert np.array_equal(q, oracle.pack_nibbles(oracle.quantize(big[:, :128], np.float32(0.3))))
    empty = torch.empty((0, 64), dtype=torch.float32, device="cuda")
    assert mkq.mkq_quantize(empty, 0.3).shape == (0, 32)


@pytest.mark.parametrize("M,K", [(128, 768), (1, 8), (300, 1000), (2048, 3072)])
def test_absmax_scale_bit_exact(mkq, M, K):
    rng = np.random.default_rng(M)
    x = rng.normal(0, 1, (M, K)).astype(np.float32)
    s = to_np(mkq.mkq_absmax_scale(to_dev(x)))[0]
    assert s == np.float32(oracle.absmax_scale(x))
    sr = to_np(mkq.mkq_absmax_scale(to_dev(x), per_row=True))
    assert np.array_equal(sr, oracle.absmax_scale(x, per_row=True))
    z = np.zeros((4, 64), np.float32)
    assert to_np(mkq.mkq_absmax_scale(to_dev(z)))[0] == 1.0


@pytest.mark.parametrize("N,K", [(768, 768), (100, 96), (3072, 768), (768, 3072), (1, 32)])
def test_pack_weights_calibrated(mkq, N, K):
    _, W, _ = wl.gaussian_linear(1, K, N, seed=N + K)
    W[N // 2] = 0.0  # an all-zero output channel
    Wq, s_w = mkq.mkq_pack_weights_int4(to_dev(W))
    codes_ref, s_ref = oracle.quantize_weights(W)
    assert np.array_equal(to_np(s_w), s_ref)
    codes = to_np(mkq.mkq_unpack_weights_int4(Wq, N, K))
    assert np.array_equal(codes, codes_ref)
    assert Wq.numel() == mkq.mkq_packed_weight_bytes(N, K) == N * K // 2


def test_pack_weights_given_scales_and_pack_codes(mkq):
    rng = np.random.default_rng(5)
    W = rng.normal(0, 0.02, (96, 160)).astype(np.float32)
    s_in = rng.uniform(0.001, 0.01, 96).astype(np.float32)
    Wq, s_w = mkq.mkq_pack_weights_int4(to_dev(W), to_dev(s_in))
    codes_ref, _ = oracle.quantize_weights(W, s_in)
    assert np.array_equal(to_np(s_w), s_in)
    assert np.array_equal(to_np(mkq.mkq_unpack_weights_int4(Wq, 96, 160)), codes_ref)
    assert codes_ref.min() == -8  # learned (smaller) steps reach the lowest code
    c = rng.integers(-8, 8, (50, 224), dtype=np.int8)
    packed = mkq.mkq_pack_codes_int4(to_dev(c))
    assert np.array_equal(to_np(packed), oracle.pack_nibbles(c))
    assert np.array_equal(to_np(mkq.mkq_unpack_weights_int4(packed, 50, 224)), c)


@pytest.mark.parametrize("s", [0.34, 1.0 / 3.0, 0.1, 0.0173, 7.0, 2.0 ** -20, 3.0e4])
def test_quantize_around_every_rounding_boundary(mkq, s):
    """Values a few ulps either side of every boundary (k + 1/2) s, and exact ties where they are
    representable: the kernel decides most codes from a reciprocal and must agree with the division."""
    s32 = np.float32(s)
    b = (np.arange(-10, 10) + 0.5)[:, None] * np.float64(s32)
    x = (b * (1.0 + np.arange(-12, 13)[None, :] * 2.0 ** -24)).astype(np.float32).ravel()
    x = np.concatenate([x, np.nextafter(x, np.float32(np.inf)), np.nextafter(x, np.float32(-np.inf))])
    pad = (-x.size) % 32
    x = np.concatenate([x, np.zeros(pad, np.float32)]).reshape(1, -1)
    q = to_np(mkq.mkq_quantize(to_dev(x), float(s32)))
    assert np.array_equal(q, oracle.pack_nibbles(oracle.quantize(x, s32)))
