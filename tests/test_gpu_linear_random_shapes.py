"""Seeded random shapes and epilogues through mkq_linear_int4's own routing (register kernel, ring kernel with
and without a scratch area, every tile kernel and its wave-group split, the register-staged kernel for K that
is no multiple of 128): accumulators and outputs bit for bit against the oracle."""
import numpy as np
import pytest

import oracle
from helpers import assert_codes_match_with_tie_band, to_dev, to_np

pytestmark = pytest.mark.gpu


def _cases(n=96, seed=2203):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        M = int(np.exp(rng.uniform(0, np.log(2500))))
        N = int(np.exp(rng.uniform(np.log(8), np.log(3000))))
        K = 32 * int(np.exp(rng.uniform(0, np.log(128))))
        if i % 3 == 0:
            K = (K + 255) // 256 * 256      # the few-token kernels' granularity
        if i % 4 == 0:
            N = (N + 7) // 8 * 8            # the compile-time epilogues' granularity
        N += N % 2                          # code outputs need an even N
        while M * N * K > 1.5e9:
            M = max(1, M // 2)
        out.append((M, N, K, int(rng.integers(0, 6)), bool(rng.integers(0, 2))))
    return out


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m, m.mkq_splitk_scratch_init()


@pytest.mark.parametrize("M,N,K,kind,with_scratch", _cases())
def test_random_shape(lib, M, N, K, kind, with_scratch):
    mkq, scratch = lib
    rng = np.random.default_rng(M * 31 + N * 7 + K)
    A = rng.integers(-8, 8, (M, K), dtype=np.int8)
    Wc = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.001, 0.05, N).astype(np.float32)
    bias = rng.normal(0, 0.5, N).astype(np.float32)
    s_x = 0.07
    a_d = mkq.mkq_pack_codes_int4(to_dev(A))
    w_d = mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1)
    kw = dict(splitk_scratch=scratch) if with_scratch else {}
    run = lambda dt, **k: mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), to_dev(bias), N, K, dt, **k, **kw)
    if kind == 0:    # binary32 out and raw accumulators
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias)
        r = run(mkq.MKQ_F32, want_acc=True)
        assert np.array_equal(to_np(r["acc"]), ref["acc"])
        assert np.array_equal(to_np(r["out"]), ref["y"])
    elif kind == 1:  # binary16 out
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.F16)
        assert np.array_equal(to_np(run(mkq.MKQ_F16)["out"]).astype(np.float32), ref["y"])
    elif kind == 2:  # bfloat16 out (compared as bits)
        import torch
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.BF16)
        assert np.array_equal(to_np(run(mkq.MKQ_BF16)["out"].float()), ref["y"])
    elif kind == 3:  # binary16 residual, binary16 out, extra codes
        res = rng.normal(0, 1, (M, N)).astype(np.float16)
        ref32 = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res.astype(np.float32))
        s_next = float(np.float32(max(np.abs(ref32["y"]).max(), 1e-3) / 9))
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res.astype(np.float32), out_dtype=oracle.F16, s_next=s_next)
        r = run(mkq.MKQ_F16, residual=to_dev(res), s_next=s_next, want_q=True)
        assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
        assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(ref["q"]))
    elif kind == 4:  # codes out, no activation function: bit-exact
        ref32 = oracle.linear_int4(A, s_x, Wc, s_w, bias)
        s_next = float(np.float32(max(np.abs(ref32["y"]).max(), 1e-3) / 9))
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, s_next=s_next)
        assert np.array_equal(to_np(run(mkq.MKQ_I4, s_next=s_next)["out"]), oracle.pack_nibbles(ref["q"]))
    else:            # GELU, codes out: the float function decides, ties may fall either way
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU, s_next=0.25)
        got = oracle.unpack_nibbles(to_np(run(mkq.MKQ_I4, act=mkq.MKQ_ACT_GELU, s_next=0.25)["out"]), N)
        assert_codes_match_with_tie_band(got, ref["q"], ref["y"], 0.25, what="gelu codes")
