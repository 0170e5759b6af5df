"""Host-side checks of the C ABI (no GPU): the library loads, exports every symbol the
public header declares, and rejects bad arguments with the documented status codes
before anything is enqueued."""
import ctypes as C
import os
import re

import pytest

import paper_2203_13483_amd as mkq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
P = C.c_void_p(0x1000)      # 16-byte aligned, never dereferenced: validation fails first
ODD = C.c_void_p(0x1004)    # misaligned


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(mkq.LIB_PATH):
        from paper_2203_13483_amd import build
        build.build()
    return mkq.load()


def test_header_symbols_are_exported(lib):
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        found = set(re.findall(r"\b(mkq_[a-z0-9_]+)\s*\(", text))
        assert found, header
        for n in found:
            assert hasattr(lib, n), f"{n} declared in {header} but not exported"
        names |= found
    assert len(names) >= 17
    assert sorted(mkq.EXPORTS) == sorted(names)


def test_status_strings(lib):
    assert mkq.status_string(0) == "ok"
    for code in range(-8, 0):
        assert mkq.status_string(code) not in ("ok", "unknown status")
    assert mkq.status_string(-99) == "unknown status"
    assert mkq.mkq_version() >= 100


def test_quantize_argument_errors(lib):
    q = lib.mkq_quantize
    assert q(None, mkq.MKQ_F32, 4, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_NULL
    assert q(P, mkq.MKQ_F32, 4, 64, 64, 1.0, None, None) == mkq.MKQ_ERR_NULL
    assert q(P, 7, 4, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_DTYPE
    assert q(P, mkq.MKQ_BF16, 4, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_DTYPE
    assert q(P, mkq.MKQ_F32, -1, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_SHAPE
    assert q(P, mkq.MKQ_F32, 4, 48, 48, 1.0, P, None) == mkq.MKQ_ERR_SHAPE   # K % 32
    assert q(P, mkq.MKQ_F32, 4, 64, 32, 1.0, P, None) == mkq.MKQ_ERR_SHAPE   # ldx < K
    assert q(ODD, mkq.MKQ_F32, 4, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_ALIGN
    for s in (0.0, -1.0, float("inf"), float("nan")):
        assert q(P, mkq.MKQ_F32, 4, 64, 64, s, P, None) == mkq.MKQ_ERR_SCALE
    assert q(None, mkq.MKQ_F32, 0, 64, 64, 1.0, None, None) == mkq.MKQ_OK    # empty: no-op


def test_pack_and_scale_argument_errors(lib):
    assert lib.mkq_absmax_scale(None, 0, 4, 64, 64, 0, P, None) == mkq.MKQ_ERR_NULL
    assert lib.mkq_absmax_scale(P, 3, 4, 64, 64, 0, P, None) == mkq.MKQ_ERR_DTYPE
    assert lib.mkq_absmax_scale(P, 0, 0, 64, 64, 0, P, None) == mkq.MKQ_ERR_SHAPE
    assert lib.mkq_pack_weights_int4(None, 8, 64, None, P, P, None) == mkq.MKQ_ERR_NULL
    assert lib.mkq_pack_weights_int4(P, 8, 40, None, P, P, None) == mkq.MKQ_ERR_SHAPE
    assert lib.mkq_pack_weights_int4(P, 8, 64, None, P, ODD, None) == mkq.MKQ_ERR_ALIGN
    assert lib.mkq_packed_weight_bytes(768, 768) == 768 * 768 // 2
    assert lib.mkq_packed_weight_bytes(768, 100) == 0
    assert lib.mkq_pack_codes_int4(None, 4, 64, P, None) == mkq.MKQ_ERR_NULL
    assert lib.mkq_unpack_weights_int4(P, 4, 33, P, None) == mkq.MKQ_ERR_SHAPE


def _linear(lib, a=P, a_dtype=mkq.MKQ_I4, s_x=0.1, Wq=P, s_w=P, bias=P, M=8, N=64, K=64, out=P,
            out_dtype=mkq.MKQ_F32, epi=None, ws=None, ws_bytes=0):
    return lib.mkq_linear_int4(a, a_dtype, s_x, Wq, s_w, bias, M, N, K, out, out_dtype,
                               C.byref(epi) if epi is not None else None, ws, ws_bytes, None)


def test_linear_argument_errors(lib):
    assert _linear(lib, a=None) == mkq.MKQ_ERR_NULL
    assert _linear(lib, Wq=None) == mkq.MKQ_ERR_NULL
    assert _linear(lib, s_w=None) == mkq.MKQ_ERR_NULL
    assert _linear(lib, out=None) == mkq.MKQ_ERR_NULL
    assert _linear(lib, a_dtype=9) == mkq.MKQ_ERR_DTYPE
    assert _linear(lib, a_dtype=mkq.MKQ_BF16) == mkq.MKQ_ERR_DTYPE
    assert _linear(lib, out_dtype=11) == mkq.MKQ_ERR_DTYPE
    assert _linear(lib, K=48) == mkq.MKQ_ERR_SHAPE
    assert _linear(lib, N=0) == mkq.MKQ_ERR_SHAPE
    assert _linear(lib, M=-2) == mkq.MKQ_ERR_SHAPE
    assert _linear(lib, a=ODD) == mkq.MKQ_ERR_ALIGN
    assert _linear(lib, out=ODD) == mkq.MKQ_ERR_ALIGN
    assert _linear(lib, s_x=0.0) == mkq.MKQ_ERR_SCALE
    assert _linear(lib, s_x=float("nan")) == mkq.MKQ_ERR_SCALE
    assert _linear(lib, K=131072) == mkq.MKQ_ERR_UNSUPPORTED
    assert _linear(lib, M=0, a=None, out=None) == mkq.MKQ_OK
    # codes out: N must be even and s_next valid
    e = mkq.Epilogue(act=0, residual=None, residual_dtype=0, s_next=0.0, q_out=None, acc_out=None)
    assert _linear(lib, out_dtype=mkq.MKQ_I4, epi=e) == mkq.MKQ_ERR_SCALE
    e.s_next = 0.5
    assert _linear(lib, out_dtype=mkq.MKQ_I4, N=63, epi=e) == mkq.MKQ_ERR_SHAPE
    e.act = 5
    assert _linear(lib, epi=e) == mkq.MKQ_ERR_DTYPE
    e.act = 0
    e.residual, e.residual_dtype = 0x1000, mkq.MKQ_BF16
    assert _linear(lib, epi=e) == mkq.MKQ_ERR_DTYPE
    # float activations need a workspace of the advertised size
    need = lib.mkq_linear_int4_workspace_bytes(8, 64, 64, mkq.MKQ_F16)
    assert need >= 8 * 32 and lib.mkq_linear_int4_workspace_bytes(8, 64, 64, mkq.MKQ_I4) == 0
    assert _linear(lib, a_dtype=mkq.MKQ_F16) == mkq.MKQ_ERR_WORKSPACE
    assert _linear(lib, a_dtype=mkq.MKQ_F16, ws=P, ws_bytes=need - 1) == mkq.MKQ_ERR_WORKSPACE


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(mkq, "_lib", None)
    monkeypatch.setattr(mkq, "LIB_PATH", "/nonexistent/libmkq.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        mkq.load()


def test_calibration_argument_errors(lib):
    sg = lib.mkq_scale_gradients
    assert sg(None, mkq.MKQ_F32, 4, 64, 64, 1.0, 4, P, None) == mkq.MKQ_ERR_NULL
    assert sg(P, mkq.MKQ_F32, 4, 64, 64, 1.0, 4, None, None) == mkq.MKQ_ERR_NULL
    assert sg(P, mkq.MKQ_BF16, 4, 64, 64, 1.0, 4, P, None) == mkq.MKQ_ERR_DTYPE
    assert sg(P, mkq.MKQ_F32, 4, 64, 64, 1.0, 5, P, None) == mkq.MKQ_ERR_DTYPE
    assert sg(P, mkq.MKQ_F32, 0, 64, 64, 1.0, 4, P, None) == mkq.MKQ_ERR_SHAPE
    assert sg(P, mkq.MKQ_F32, 4, 60, 64, 1.0, 4, P, None) == mkq.MKQ_ERR_SHAPE
    assert sg(P, mkq.MKQ_F32, 4, 64, 64, 0.0, 4, P, None) == mkq.MKQ_ERR_SCALE
    assert sg(ODD, mkq.MKQ_F32, 4, 64, 64, 1.0, 4, P, None) == mkq.MKQ_ERR_ALIGN
    ps = lib.mkq_percentile_scale
    need = lib.mkq_percentile_scale_workspace_bytes()
    assert need >= 3 * 2048 * 4
    assert ps(None, mkq.MKQ_F32, 4, 64, 64, 100, 4, P, P, need, None) == mkq.MKQ_ERR_NULL
    assert ps(P, mkq.MKQ_F32, 4, 64, 64, 100, 4, None, P, need, None) == mkq.MKQ_ERR_NULL
    assert ps(P, mkq.MKQ_F32, 4, 64, 64, -1, 4, P, P, need, None) == mkq.MKQ_ERR_SHAPE
    assert ps(P, mkq.MKQ_F32, 4, 64, 64, 1000001, 4, P, P, need, None) == mkq.MKQ_ERR_SHAPE
    assert ps(P, mkq.MKQ_F32, 4, 64, 64, 100, 3, P, P, need, None) == mkq.MKQ_ERR_DTYPE
    assert ps(P, mkq.MKQ_F32, 4, 64, 64, 100, 4, P, None, need, None) == mkq.MKQ_ERR_WORKSPACE
    assert ps(P, mkq.MKQ_F32, 4, 64, 64, 100, 4, P, P, need - 1, None) == mkq.MKQ_ERR_WORKSPACE
    assert ps(P, mkq.MKQ_F32, 1 << 20, 1 << 13, 1 << 13, 100, 4, P, P, need, None) == mkq.MKQ_ERR_UNSUPPORTED


def test_int8_argument_errors(lib):
    q8 = lib.mkq_quantize_int8
    assert q8(None, mkq.MKQ_F32, 4, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_NULL
    assert q8(P, mkq.MKQ_BF16, 4, 64, 64, 1.0, P, None) == mkq.MKQ_ERR_DTYPE
    assert q8(P, mkq.MKQ_F32, 4, 40, 40, 1.0, P, None) == mkq.MKQ_ERR_SHAPE   # K % 16
    assert q8(P, mkq.MKQ_F32, 4, 64, 64, -1.0, P, None) == mkq.MKQ_ERR_SCALE
    assert q8(P, mkq.MKQ_F32, 0, 64, 64, 1.0, None, None) == mkq.MKQ_OK       # empty
    pw = lib.mkq_pack_weights_int8
    assert pw(None, 8, 64, None, P, P, None) == mkq.MKQ_ERR_NULL
    assert pw(P, 8, 24, None, P, P, None) == mkq.MKQ_ERR_SHAPE
    assert pw(P, 8, 64, None, P, ODD, None) == mkq.MKQ_ERR_ALIGN
    lin = lib.mkq_linear_int8

    def call(a=P, s_x=1.0, Wq=P, s_w=P, bias=None, M=8, N=64, K=64, out=P, out_dtype=mkq.MKQ_F16, epi=None):
        return lin(a, s_x, Wq, s_w, bias, M, N, K, out, out_dtype, epi, None)

    assert call(a=None) == mkq.MKQ_ERR_NULL
    assert call(out=None) == mkq.MKQ_ERR_NULL
    assert call(K=96) == mkq.MKQ_ERR_SHAPE          # K % 64
    assert call(K=65536) == mkq.MKQ_ERR_UNSUPPORTED
    assert call(s_x=0.0) == mkq.MKQ_ERR_SCALE
    assert call(out_dtype=9) == mkq.MKQ_ERR_DTYPE
    assert call(out_dtype=mkq.MKQ_I4) == mkq.MKQ_ERR_UNSUPPORTED
    assert call(out=ODD) == mkq.MKQ_ERR_ALIGN
    assert call(M=0, a=None, out=None) == mkq.MKQ_OK
    e = mkq.Epilogue(act=0, residual=None, residual_dtype=0, s_next=0.0, q_out=None, acc_out=None)
    assert call(out_dtype=mkq.MKQ_I8, epi=C.byref(e)) == mkq.MKQ_ERR_SCALE   # code output needs s_next
    e.q_out = 0x1000
    assert call(epi=C.byref(e)) == mkq.MKQ_ERR_UNSUPPORTED
    lay = mkq.BertLayerParams()
    lay.batch, lay.seq, lay.hidden, lay.heads, lay.ffn = 2, 64, 128, 2, 256
    L4, L8 = mkq.BertLayerWorkspaceLayout(), mkq.BertLayerWorkspaceLayout()
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L4)) == mkq.MKQ_OK
    assert lib.mkq_bert_layer_int8_workspace(C.byref(lay), C.byref(L8)) == mkq.MKQ_OK
    assert L8.qkv - L8.c0 == 2 * (L4.qkv - L4.c0) and L8.total > L4.total
    lay.seq = 5000                                                                    # longest sequence: 4096
    assert lib.mkq_bert_layer_int8_workspace(C.byref(lay), C.byref(L8)) == mkq.MKQ_ERR_UNSUPPORTED
    lay.seq, lay.heads = 160, 1                                                       # d_k = 128
    assert lib.mkq_bert_layer_int8_workspace(C.byref(lay), C.byref(L8)) == mkq.MKQ_ERR_UNSUPPORTED
    # the student's sizes (312 = 12 heads of 26, FFN 1200): padded code rows at 4 bits, refused at 8
    lay.seq, lay.hidden, lay.heads, lay.ffn = 128, 312, 12, 1200
    assert lib.mkq_bert_layer_int8_workspace(C.byref(lay), C.byref(L8)) == mkq.MKQ_ERR_SHAPE
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L4)) == mkq.MKQ_OK
    assert L4.qkv - L4.c0 == 256 * 384 // 2 and L4.d - L4.c3 == 256 * 1280 // 2        # rows of padded_k codes
    lay.heads = 8                                                                     # d_k = 39 is odd
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L4)) == mkq.MKQ_ERR_UNSUPPORTED
    lay.hidden, lay.heads = 316, 2                                                    # hidden % 8
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L4)) == mkq.MKQ_ERR_SHAPE


def test_padding_free_argument_errors(lib):
    av = lib.mkq_attention_varlen
    assert av(P, None, 2, 64, 128, 2, P, 1.0, None, 4, None) == mkq.MKQ_ERR_NULL      # cu_seqlens
    assert av(P, P, 2, 64, 128, 2, P, 1.0, None, 5, None) == mkq.MKQ_ERR_DTYPE        # q_bits
    assert av(P, P, 2, 5000, 128, 2, P, 1.0, None, 4, None) == mkq.MKQ_ERR_UNSUPPORTED  # max_seq > 4096
    assert av(P, P, 2, 200, 256, 2, P, 1.0, None, 4, None) == mkq.MKQ_ERR_UNSUPPORTED   # d_k = 128
    assert av(P, P, 2, 200, 120, 8, P, 1.0, None, 4, None) == mkq.MKQ_ERR_UNSUPPORTED   # d_k = 15 is odd
    assert av(P, P, 2, 200, 36, 2, P, 1.0, None, 4, None) == mkq.MKQ_ERR_SHAPE          # hidden % 8 (code rows)
    assert av(P, P, 2, 70, 128, 3, P, 1.0, None, 4, None) == mkq.MKQ_ERR_SHAPE        # hidden % heads
    assert av(P, P, 0, 70, 128, 2, None, 1.0, None, 4, None) == mkq.MKQ_OK            # empty batch
    lay = mkq.BertLayerParams()
    lay.batch, lay.seq, lay.hidden, lay.heads, lay.ffn = 4, 100, 128, 2, 256          # any length, fixed or bound
    L = mkq.BertLayerWorkspaceLayout()
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L)) == mkq.MKQ_OK
    lay.cu_seqlens, lay.total_tokens = 0x1000, 230
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L)) == mkq.MKQ_OK
    assert L.qkv - L.c0 == 256 * ((230 * 128 // 2 + 255) // 256)
    lay.total_tokens = 401                                                            # more than batch * seq
    assert lib.mkq_bert_layer_workspace(C.byref(lay), C.byref(L)) == mkq.MKQ_ERR_SHAPE
    lay.total_tokens, lay.next_bits = 230, 5
    assert lib.mkq_bert_layer_int4(C.byref(lay), P, mkq.MKQ_F16, None, P, None, P, 1 << 30, None) in (
        mkq.MKQ_ERR_SCALE, mkq.MKQ_ERR_DTYPE)


def test_padded_k_argument_errors(lib):
    assert lib.mkq_padded_k(312) == 384 and lib.mkq_padded_k(1200) == 1280
    assert lib.mkq_padded_k(768) == 768 and lib.mkq_padded_k(8) == 128 and lib.mkq_padded_k(0) == 0
    q = lib.mkq_quantize_padded
    assert q(None, mkq.MKQ_F16, 4, 312, 312, 1.0, P, None) == mkq.MKQ_ERR_NULL
    assert q(P, mkq.MKQ_BF16, 4, 312, 312, 1.0, P, None) == mkq.MKQ_ERR_DTYPE
    assert q(P, mkq.MKQ_F32, 4, 316, 320, 1.0, P, None) == mkq.MKQ_ERR_SHAPE   # K % 8
    assert q(P, mkq.MKQ_F32, 4, 312, 304, 1.0, P, None) == mkq.MKQ_ERR_SHAPE   # ldx < K
    assert q(P, mkq.MKQ_F32, 4, 312, 312, 0.0, P, None) == mkq.MKQ_ERR_SCALE
    assert q(P, mkq.MKQ_F32, 4, 312, 312, 1.0, ODD, None) == mkq.MKQ_ERR_ALIGN
    assert q(None, mkq.MKQ_F32, 0, 312, 312, 1.0, None, None) == mkq.MKQ_OK
    w = lib.mkq_pack_weights_int4_padded
    assert w(None, 8, 312, None, P, P, None) == mkq.MKQ_ERR_NULL
    assert w(P, 8, 316, None, P, P, None) == mkq.MKQ_ERR_SHAPE
    assert w(P, 0, 312, None, P, P, None) == mkq.MKQ_ERR_SHAPE
    assert w(P, 8, 312, None, P, ODD, None) == mkq.MKQ_ERR_ALIGN


def test_static_scratch_entry_point_limits(lib):
    """mkq_linear_int4_stream_static refuses, before anything runs, what its fixed scratch cannot serve."""
    f = lib.mkq_linear_int4_stream_static
    f.argtypes = [C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                  C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
    assert f(P, 1.0, P, P, None, 129, 256, 256, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_UNSUPPORTED   # M > 128
    assert f(P, 1.0, P, P, None, 16, 256, 128, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_UNSUPPORTED    # K % 256
    # 600000 channels: more 128-channel tiles than ticket counters
    assert f(P, 1.0, P, P, None, 16, 600000, 256, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_UNSUPPORTED
    # 128 tokens x 12800 channels x K = 4096: three K slices of 100 tiles x 64 KiB = 18.75 MiB of partial sums
    assert f(P, 1.0, P, P, None, 128, 12800, 4096, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_UNSUPPORTED
    assert f(P, 1.0, P, P, None, -1, 256, 256, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_SHAPE
    assert f(None, 1.0, P, P, None, 16, 256, 256, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_NULL
    assert f(P, 0.0, P, P, None, 16, 256, 256, P, mkq.MKQ_F16, None, None) == mkq.MKQ_ERR_SCALE


def test_splitk_scratch_and_stream_layout_argument_errors(lib):
    assert lib.mkq_splitk_scratch_bytes() == 16384 + (16 << 20)
    assert lib.mkq_splitk_scratch_init(None, 1 << 30, None) == mkq.MKQ_ERR_NULL
    assert lib.mkq_splitk_scratch_init(ODD, 1 << 30, None) == mkq.MKQ_ERR_ALIGN
    assert lib.mkq_splitk_scratch_init(P, 1024, None) == mkq.MKQ_ERR_WORKSPACE
    assert lib.mkq_stream_weight_bytes(100, 256) == 5 * 32 * 128     # 4 panels -> pitch 5
    assert lib.mkq_stream_weight_bytes(96, 256) == 3 * 32 * 128      # 3 panels, already odd
    r = lib.mkq_repack_weights_int4_stream
    assert r(None, 64, 64, P, None) == mkq.MKQ_ERR_NULL
    assert r(P, 64, 96, P, None) == mkq.MKQ_ERR_SHAPE                 # K % 64
    assert r(ODD, 64, 64, P, None) == mkq.MKQ_ERR_ALIGN
    epi = mkq.Epilogue(splitk_scratch=0x1000, splitk_scratch_bytes=4096)
    f = lib.mkq_linear_int4_stream
    assert f(P, mkq.MKQ_I4, 1.0, P, P, None, 16, 256, 256, P, mkq.MKQ_F16, C.byref(epi), None, 0, None) == mkq.MKQ_ERR_WORKSPACE
    assert f(P, mkq.MKQ_I4, 1.0, P, P, None, 129, 256, 256, P, mkq.MKQ_F16, None, None, 0, None) == mkq.MKQ_ERR_UNSUPPORTED
    assert f(P, mkq.MKQ_I4, 1.0, P, P, None, 16, 256, 128, P, mkq.MKQ_F16, None, None, 0, None) == mkq.MKQ_ERR_UNSUPPORTED
    t = lib.mkq_tuning_linear_int4
    # a forced configuration that does not apply is refused before anything is enqueued
    assert t(P, mkq.MKQ_I4, 1.0, P, P, None, 512, 256, 256, P, mkq.MKQ_F16, None, None, 0, None, 50, 0) == mkq.MKQ_ERR_UNSUPPORTED
    assert t(P, mkq.MKQ_I4, 1.0, P, P, None, 512, 256, 96, P, mkq.MKQ_F16, None, None, 0, None, 18, 0) == mkq.MKQ_ERR_UNSUPPORTED
    assert t(P, mkq.MKQ_I4, 1.0, P, P, None, 512, 256, 256, P, mkq.MKQ_F16, None, None, 0, None, 999, 0) == mkq.MKQ_ERR_UNSUPPORTED


def test_ceiling_probe_argument_errors(lib):
    ms = lib.mkq_measure_stream
    ms.restype, ms.argtypes = C.c_int, [C.c_int, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    assert ms(3, P, P, 1024, None) == mkq.MKQ_ERR_DTYPE          # kind
    assert ms(0, None, P, 1024, None) == mkq.MKQ_ERR_NULL        # a read needs a source
    assert ms(1, None, None, 1024, None) == mkq.MKQ_ERR_NULL     # a write needs a destination
    assert ms(2, P, ODD, 1024, None) == mkq.MKQ_ERR_ALIGN
    assert ms(2, P, P, 1000, None) == mkq.MKQ_ERR_SHAPE          # bytes % 16
    assert ms(2, P, P, 0, None) == mkq.MKQ_ERR_SHAPE
    # the size of the operand block and the operation count depend on the device's compute units: without a
    # device both are 0, with one they are checked in the GPU tier
    assert lib.mkq_measure_mfma_i8_ops(0) == 0 and lib.mkq_measure_mfma_i8_ops(-3) == 0
    mm = lib.mkq_measure_mfma_i8
    mm.restype, mm.argtypes = C.c_int, [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p]
    assert mm(None, 1 << 20, 4, P, None) == mkq.MKQ_ERR_NULL
    assert mm(P, 1 << 20, 4, None, None) == mkq.MKQ_ERR_NULL
    assert mm(ODD, 1 << 20, 4, P, None) == mkq.MKQ_ERR_ALIGN
    assert mm(P, 1 << 20, 0, P, None) == mkq.MKQ_ERR_SHAPE


def test_int8_tuning_argument_errors(lib):
    t = lib.mkq_tuning_linear_int8
    t.restype = C.c_int
    t.argtypes = [C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                  C.c_void_p, C.c_int, C.c_void_p, C.c_void_p, C.c_int]
    assert t(P, 0.1, P, P, None, 16, 64, 128, P, mkq.MKQ_F16, None, None, 999) == mkq.MKQ_ERR_UNSUPPORTED   # no such configuration
    assert t(P, 0.1, P, P, None, 16, 64, 96, P, mkq.MKQ_F16, None, None, 30) == mkq.MKQ_ERR_SHAPE           # K % 64 comes first
    assert t(P, 0.1, P, P, None, 16, 64, 192, P, mkq.MKQ_F16, None, None, 30) == mkq.MKQ_ERR_UNSUPPORTED    # streaming: K % 128
    assert t(P, 0.1, P, P, None, 65, 64, 128, P, mkq.MKQ_F16, None, None, 30) == mkq.MKQ_ERR_UNSUPPORTED    # streaming: M <= 64
    assert t(None, 0.1, P, P, None, 16, 64, 128, P, mkq.MKQ_F16, None, None, 30) == mkq.MKQ_ERR_NULL
    assert t(P, 0.0, P, P, None, 16, 64, 128, P, mkq.MKQ_F16, None, None, 27) == mkq.MKQ_ERR_SCALE
