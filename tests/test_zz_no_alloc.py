"""The entry point that allocates nothing: mkq_linear_int4_stream_static (the K split's scratch is a static
device array inside the library) against mkq_linear_int4_stream with a caller-provided scratch area, through
the C ABI, bit for bit, on two calls in a row, the second with a smaller input."""
import ctypes as C

import numpy as np
import pytest

from paper_2203_13483_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _call_pair(mkq, lib, scratch, M, N, K, seed, out_dtype, tdt):
    import torch
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed)
    bias = np.random.default_rng(seed + 1).normal(0, 0.5, N).astype(np.float32)
    a = mkq.mkq_pack_codes_int4(torch.from_numpy(A).cuda())
    w = mkq.mkq_repack_weights_int4_stream(mkq.mkq_pack_codes_int4(torch.from_numpy(Wc).cuda()).reshape(-1), N, K)
    sw, b = torch.from_numpy(s_w).cuda(), torch.from_numpy(bias).cuda()
    outs, accs, qs = [], [], []
    for which in range(2):
        out = torch.full((M, N), float("nan"), dtype=tdt, device="cuda")
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        q = torch.full((M, N // 2), 0xEE, dtype=torch.uint8, device="cuda")
        epi = mkq.Epilogue(act=mkq.MKQ_ACT_NONE, residual=None, residual_dtype=mkq.MKQ_F32, s_next=0.6,
                           q_out=q.data_ptr(), acc_out=acc.data_ptr(),
                           splitk_scratch=scratch.data_ptr() if which == 0 else None,
                           splitk_scratch_bytes=scratch.numel() if which == 0 else 0)
        stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
        if which == 0:
            rc = lib.mkq_linear_int4_stream(C.c_void_p(a.data_ptr()), mkq.MKQ_I4, C.c_float(s_x), C.c_void_p(w.data_ptr()),
                                            C.c_void_p(sw.data_ptr()), C.c_void_p(b.data_ptr()), M, N, K,
                                            C.c_void_p(out.data_ptr()), out_dtype, C.byref(epi), None, 0, stream)
        else:
            rc = lib.mkq_linear_int4_stream_static(C.c_void_p(a.data_ptr()), C.c_float(s_x), C.c_void_p(w.data_ptr()),
                                                   C.c_void_p(sw.data_ptr()), C.c_void_p(b.data_ptr()), M, N, K,
                                                   C.c_void_p(out.data_ptr()), out_dtype, C.byref(epi), stream)
        assert rc == mkq.MKQ_OK, mkq.status_string(rc)
        torch.cuda.synchronize()
        outs.append(out.view(torch.int16 if tdt != torch.float32 else torch.int32).cpu().numpy())
        accs.append(acc.cpu().numpy())
        qs.append(q.cpu().numpy())
    assert np.array_equal(accs[0], accs[1]), "accumulators differ"
    assert np.array_equal(outs[0], outs[1]), "outputs differ"
    assert np.array_equal(qs[0], qs[1]), "codes differ"
    return accs[1], A, Wc


def test_static_scratch_entry_point_matches_caller_scratch_entry_point():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as mkq
    lib = mkq.load()
    scratch = mkq.mkq_splitk_scratch_init()
    # first call: K split over several workgroups per tile (few channel tiles, long K), ragged N
    acc, A, Wc = _call_pair(mkq, lib, scratch, 48, 1000, 8192, 11, mkq.MKQ_F16, torch.float16)
    assert np.array_equal(acc, A.astype(np.int32) @ Wc.astype(np.int32).T)  # both are the exact integer product
    # second call, smaller in every dimension: the area still holds the first call's partial sums
    acc, A, Wc = _call_pair(mkq, lib, scratch, 5, 200, 1024, 12, mkq.MKQ_F32, torch.float32)
    assert np.array_equal(acc, A.astype(np.int32) @ Wc.astype(np.int32).T)
    # and a third, larger again, with 65 .. 128 tokens
    _call_pair(mkq, lib, scratch, 100, 4096, 2048, 13, mkq.MKQ_BF16, torch.bfloat16)
