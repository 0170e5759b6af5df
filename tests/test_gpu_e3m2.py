"""GPU parity of the experimental 6-bit float (E3M2) route of the 4-bit linear: the containers are checked
bit for bit against a table written here from the format's definition, the accumulators and outputs
against the oracle's int4 linear -- the route must give the same exact integers as the int8 route."""
import numpy as np
import pytest

import oracle
from paper_2203_13483_amd import workloads as wl
from helpers import RTOL, assert_float_close, to_dev, to_np

pytestmark = pytest.mark.gpu

# magnitude m = 0 .. 8 as sign-less E3M2: exponent e (bias 3), mantissa f: value (1 + f/4) * 2^(e - 3)
E3M2_MAG = {0: 0b00000, 1: 0b01100, 2: 0b10000, 3: 0b10010, 4: 0b10100, 5: 0b10101, 6: 0b10110, 7: 0b10111,
            8: 0b11000}


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m


def _containers(codes):
    """Reference packing: a row is groups of 64 codes = 48 bytes; the 32 codes of half h of a group form a
    192-bit little-endian stream (code i in bits [6i, 6i + 6)) whose first 16 bytes are bytes
    [16h, 16h + 16) of the group and whose last 8 bytes are bytes [32 + 8h, 40 + 8h)."""
    rows, K = codes.shape
    e = np.vectorize(lambda c: E3M2_MAG[abs(int(c))] | (0x20 if c < 0 else 0))(codes).astype(np.uint64)
    bits = ((e[:, :, None] >> np.arange(6, dtype=np.uint64)) & 1).astype(np.uint8).reshape(rows, K // 32, 192)
    stream = np.packbits(bits, axis=2, bitorder="little").reshape(rows, K // 64, 2, 24)
    out = np.empty((rows, K // 64, 48), np.uint8)
    for h in (0, 1):
        out[:, :, 16 * h: 16 * h + 16] = stream[:, :, h, :16]
        out[:, :, 32 + 8 * h: 40 + 8 * h] = stream[:, :, h, 16:]
    return out.reshape(rows, K * 3 // 4)


def test_table_is_the_format():
    for m, enc in E3M2_MAG.items():
        e, f = enc >> 2, enc & 3
        val = (f / 4) * 2.0 ** (1 - 3) if e == 0 else (1 + f / 4) * 2.0 ** (e - 3)
        assert val == m


def test_containers_bit_exact(mkq):
    rng = np.random.default_rng(1)
    codes = rng.integers(-8, 9, (37, 192), dtype=np.int8)
    assert np.array_equal(to_np(mkq.mkq_pack_codes_e3m2(to_dev(codes))), _containers(codes))
    X = (rng.standard_normal((50, 256)) * 1.2).astype(np.float32)
    s = np.float32(0.3)
    assert np.array_equal(to_np(mkq.mkq_quantize_e3m2(to_dev(X), float(s))), _containers(oracle.quantize(X, s)))
    W = (rng.standard_normal((40, 128)) * 0.02).astype(np.float32)
    Wq, s_w = mkq.mkq_pack_weights_e3m2(to_dev(W))
    wc, sw = oracle.quantize_weights(W)
    assert np.array_equal(to_np(s_w), sw) and np.array_equal(to_np(Wq), _containers(wc))


@pytest.mark.parametrize("M,N,K", [(256, 128, 128), (300, 200, 128), (1, 8, 128), (1024, 768, 768), (517, 1000, 1024),
                                   (2048, 256, 4096)])
def test_accumulators_and_outputs_match_the_oracle(mkq, M, N, K):
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed=M + K)
    b = np.random.default_rng(N).normal(0, 0.3, N).astype(np.float32)
    a_d, w_d = mkq.mkq_pack_codes_e3m2(to_dev(A)), mkq.mkq_pack_codes_e3m2(to_dev(Wc))
    r = mkq.mkq_linear_int4_e3m2(a_d, s_x, w_d, to_dev(s_w), to_dev(b), mkq.MKQ_F32, want_acc=True)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, b)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]), ref["y"])
    for od in (1, 2):
        r = mkq.mkq_linear_int4_e3m2(a_d, s_x, w_d, to_dev(s_w), to_dev(b), od)
        ref = oracle.linear_int4(A, s_x, Wc, s_w, b, out_dtype=od)
        assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])


@pytest.mark.parametrize("K", [128, 4096, 65536])
def test_accumulator_extremes(mkq, K):
    M, N = 40, 72
    lo = np.full((M, K), -8, np.int8)
    ones = np.ones(N, np.float32)
    for wv, want in ((-8, 64 * K), (7, -56 * K)):
        r = mkq.mkq_linear_int4_e3m2(mkq.mkq_pack_codes_e3m2(to_dev(lo)), 1.0,
                                     mkq.mkq_pack_codes_e3m2(to_dev(np.full((N, K), wv, np.int8))), to_dev(ones), None,
                                     mkq.MKQ_F32, want_acc=True)
        assert np.all(to_np(r["acc"]) == want)


def test_float_in_requant_and_residual(mkq):
    rng = np.random.default_rng(3)
    M, K, N = 700, 768, 520
    X = wl.outlier_activations(rng, M, K, 0.01, "x8").astype(np.float16)
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
    res = rng.standard_normal((M, N)).astype(np.float16)
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    Wq, s_w = mkq.mkq_pack_weights_e3m2(to_dev(W))
    a = mkq.mkq_quantize_e3m2(to_dev(X), s_x)
    wc, sw = oracle.quantize_weights(W)
    codes = oracle.quantize(X.astype(np.float32), s_x)
    r = mkq.mkq_linear_int4_e3m2(a, s_x, Wq, s_w, to_dev(b), mkq.MKQ_I4, residual=to_dev(res), s_next=0.2)
    ref = oracle.linear_int4(codes, s_x, wc, sw, b, residual=res.astype(np.float32), s_next=0.2)
    assert np.array_equal(oracle.unpack_nibbles(to_np(r["out"]), N), ref["q"])


@pytest.mark.parametrize("M,N,K,od,with_bias", [(16384, 4096, 1024, 2, False), (16384, 4096, 128, 1, True),
                                                 (8200, 4104, 256, 0, True), (8200, 4104, 384, 2, False),
                                                 (4099, 8192, 2048, 2, True), (65536, 2048, 256, 2, False)])
@pytest.mark.parametrize("cfg", [41, 42, -1])
def test_large_m_sampled_rows(mkq, cfg, M, N, K, od, with_bias):
    """More tiles than resident workgroups: every workgroup walks several tiles (one-stage tiles, ragged
    edges in both directions, both tile shapes), checked on sampled rows."""
    import torch
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed=9 + K)
    b = np.random.default_rng(K).normal(0, 0.3, N).astype(np.float32) if with_bias else None
    tdt = {0: torch.float32, 1: torch.float16, 2: torch.bfloat16}[od]
    out = torch.empty((M, N), dtype=tdt, device="cuda")
    # 41: 256 x 256 tiles, 42: 256 x 128, -1: the library's own choice
    mkq.mkq_linear_int4_e3m2(mkq.mkq_pack_codes_e3m2(to_dev(A)), s_x, mkq.mkq_pack_codes_e3m2(to_dev(Wc)),
                             to_dev(s_w), None if b is None else to_dev(b), od, out=out, config=cfg)
    torch.cuda.synchronize()
    rows = np.unique(np.concatenate([[0, 255, 256, 257, M - 257, M - 2, M - 1],
                                     np.random.default_rng(2).integers(0, M, 40)]))
    got = to_np(out[torch.from_numpy(rows).cuda()]).astype(np.float32)
    ref = oracle.linear_int4(A[rows], s_x, Wc, s_w, b, out_dtype=od)
    assert np.array_equal(got, ref["y"])
