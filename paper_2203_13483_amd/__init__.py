"""Python binding of libmkq (MI355X-native W4A4 BERT linear layer).

Argument marshalling only: every step of the path runs in the HIP kernels of
``libmkq.so``.  PyTorch is used for device memory and streams.  There is no
fallback: if the library has not been built, loading it raises.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmkq.so")

MKQ_OK = 0
MKQ_ERR_NULL, MKQ_ERR_SHAPE, MKQ_ERR_ALIGN, MKQ_ERR_SCALE = -1, -2, -3, -4
MKQ_ERR_DTYPE, MKQ_ERR_WORKSPACE, MKQ_ERR_UNSUPPORTED, MKQ_ERR_HIP = -5, -6, -7, -8
MKQ_F32, MKQ_F16, MKQ_BF16, MKQ_I4, MKQ_I8 = 0, 1, 2, 3, 4
MKQ_ACT_NONE, MKQ_ACT_GELU = 0, 1

EXPORTS = [
    "mkq_status_string", "mkq_version", "mkq_quantize", "mkq_absmax_scale",
    "mkq_packed_weight_bytes", "mkq_pack_weights_int4", "mkq_pack_codes_int4",
    "mkq_padded_k", "mkq_quantize_padded", "mkq_pack_weights_int4_padded",
    "mkq_unpack_weights_int4", "mkq_linear_int4_workspace_bytes", "mkq_linear_int4",
    "mkq_quantize_int8", "mkq_pack_weights_int8", "mkq_linear_int8", "mkq_bert_layer_int8_workspace",
    "mkq_bert_layer_int8", "mkq_layernorm_int8", "mkq_attention_int8",
    "mkq_scale_gradients", "mkq_percentile_scale_workspace_bytes", "mkq_percentile_scale", "mkq_attention_varlen",
    "mkq_quantize_e3m2", "mkq_pack_codes_e3m2", "mkq_pack_weights_e3m2", "mkq_linear_int4_e3m2",
    "mkq_linear_fp16", "mkq_bert_layer_workspace", "mkq_bert_layer_int4",
    "mkq_bert_layer_fp16_workspace_bytes", "mkq_bert_layer_fp16", "mkq_layernorm", "mkq_attention",
    "mkq_splitk_scratch_bytes", "mkq_splitk_scratch_init", "mkq_init",
    "mkq_tuning_linear_int4", "mkq_tuning_linear_int4_e3m2", "mkq_tuning_linear_int4_stream", "mkq_tuning_linear_int8",
    "mkq_stream_weight_bytes", "mkq_repack_weights_int4_stream", "mkq_linear_int4_stream",
    "mkq_linear_int4_stream_static",
    "mkq_measure_stream", "mkq_measure_mfma_i8_operand_bytes", "mkq_measure_mfma_i8_ops", "mkq_measure_mfma_i8",
]


class MkqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class Epilogue(C.Structure):
    _fields_ = [("act", C.c_int), ("residual", C.c_void_p), ("residual_dtype", C.c_int),
                ("s_next", C.c_float), ("q_out", C.c_void_p), ("acc_out", C.c_void_p),
                ("splitk_scratch", C.c_void_p), ("splitk_scratch_bytes", C.c_size_t), ("q_pitch", C.c_int64)]


class BertLayerParams(C.Structure):
    _fields_ = ([(n, C.c_int64) for n in ("batch", "seq", "hidden", "heads", "ffn")]
                + [(n, C.c_void_p) for n in ("Wq_qkv", "Wq_ao", "Wq_up", "Wq_down",
                                             "sw_qkv", "sw_ao", "sw_up", "sw_down",
                                             "b_qkv", "b_ao", "b_up", "b_down")]
                + [(n, C.c_float) for n in ("sx_qkv", "sx_ao", "sx_up", "sx_down")]
                + [(n, C.c_void_p) for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")]
                + [("ln_eps", C.c_float), ("s_out_next", C.c_float), ("next_bits", C.c_int),
                   ("cu_seqlens", C.c_void_p), ("total_tokens", C.c_int64)])


class BertLayerWorkspaceLayout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("c0", "qkv", "c1", "u", "h1", "c2", "c3", "d", "total")]


class BertLayerParamsFp16(C.Structure):
    _fields_ = ([(n, C.c_int64) for n in ("batch", "seq", "hidden", "heads", "ffn")]
                + [(n, C.c_void_p) for n in ("W_qkv", "W_ao", "W_up", "W_down",
                                             "b_qkv", "b_ao", "b_up", "b_down",
                                             "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")]
                + [("ln_eps", C.c_float), ("cu_seqlens", C.c_void_p), ("total_tokens", C.c_int64)])


_lib = None


def load() -> C.CDLL:
    """Loads libmkq.so (built by ``python -m paper_2203_13483_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           f"`python -m paper_2203_13483_amd.build` (there is no fallback path)")
    # torch first: the device memory and streams handed to the library are torch's, so both must sit on the
    # HIP runtime that torch brings; loaded before torch, the library would pull in the system's copy instead
    _torch()
    lib = C.CDLL(LIB_PATH)
    i64, vp, f32, ci, sz = C.c_int64, C.c_void_p, C.c_float, C.c_int, C.c_size_t
    sig = {
        "mkq_status_string": (C.c_char_p, [ci]),
        "mkq_version": (ci, []),
        "mkq_quantize": (ci, [vp, ci, i64, i64, i64, f32, vp, vp]),
        "mkq_absmax_scale": (ci, [vp, ci, i64, i64, i64, ci, vp, vp]),
        "mkq_packed_weight_bytes": (sz, [i64, i64]),
        "mkq_scale_gradients": (ci, [vp, ci, i64, i64, i64, f32, ci, vp, vp]),
        "mkq_percentile_scale_workspace_bytes": (sz, []),
        "mkq_percentile_scale": (ci, [vp, ci, i64, i64, i64, i64, ci, vp, vp, sz, vp]),
        "mkq_pack_weights_int4": (ci, [vp, i64, i64, vp, vp, vp, vp]),
        "mkq_pack_codes_int4": (ci, [vp, i64, i64, vp, vp]),
        "mkq_padded_k": (i64, [i64]),
        "mkq_quantize_padded": (ci, [vp, ci, i64, i64, i64, f32, vp, vp]),
        "mkq_pack_weights_int4_padded": (ci, [vp, i64, i64, vp, vp, vp, vp]),
        "mkq_unpack_weights_int4": (ci, [vp, i64, i64, vp, vp]),
        "mkq_linear_int4_workspace_bytes": (sz, [i64, i64, i64, ci]),
        "mkq_linear_int4": (ci, [vp, ci, f32, vp, vp, vp, i64, i64, i64, vp, ci,
                                 C.POINTER(Epilogue), vp, sz, vp]),
        "mkq_tuning_linear_int4": (ci, [vp, ci, f32, vp, vp, vp, i64, i64, i64, vp, ci,
                                        C.POINTER(Epilogue), vp, sz, vp, ci, ci]),
        "mkq_tuning_linear_int4_e3m2": (ci, [vp, f32, vp, vp, vp, i64, i64, i64, vp, ci, C.POINTER(Epilogue), vp, ci]),
        "mkq_tuning_linear_int4_stream": (ci, [vp, ci, f32, vp, vp, vp, i64, i64, i64, vp, ci,
                                               C.POINTER(Epilogue), vp, sz, vp, ci, ci]),
        "mkq_linear_int4_stream": (ci, [vp, ci, f32, vp, vp, vp, i64, i64, i64, vp, ci,
                                        C.POINTER(Epilogue), vp, sz, vp]),
        "mkq_linear_int4_stream_static": (ci, [vp, f32, vp, vp, vp, i64, i64, i64, vp, ci, C.POINTER(Epilogue), vp]),
        "mkq_measure_stream": (ci, [ci, vp, vp, sz, vp]),
        "mkq_measure_mfma_i8_operand_bytes": (sz, []),
        "mkq_measure_mfma_i8_ops": (i64, [ci]),
        "mkq_measure_mfma_i8": (ci, [vp, sz, ci, vp, vp]),
        "mkq_stream_weight_bytes": (sz, [i64, i64]),
        "mkq_repack_weights_int4_stream": (ci, [vp, i64, i64, vp, vp]),
        "mkq_splitk_scratch_bytes": (sz, []),
        "mkq_splitk_scratch_init": (ci, [vp, sz, vp]),
        "mkq_init": (ci, []),
        "mkq_quantize_int8": (ci, [vp, ci, i64, i64, i64, f32, vp, vp]),
        "mkq_pack_weights_int8": (ci, [vp, i64, i64, vp, vp, vp, vp]),
        "mkq_linear_int8": (ci, [vp, f32, vp, vp, vp, i64, i64, i64, vp, ci, C.POINTER(Epilogue), vp]),
        "mkq_tuning_linear_int8": (ci, [vp, f32, vp, vp, vp, i64, i64, i64, vp, ci, C.POINTER(Epilogue), vp, ci]),
        "mkq_linear_fp16": (ci, [vp, vp, vp, i64, i64, i64, vp, ci, ci, vp, vp]),
        "mkq_quantize_e3m2": (ci, [vp, ci, i64, i64, i64, f32, vp, vp]),
        "mkq_pack_codes_e3m2": (ci, [vp, i64, i64, vp, vp]),
        "mkq_pack_weights_e3m2": (ci, [vp, i64, i64, vp, vp, vp, vp]),
        "mkq_linear_int4_e3m2": (ci, [vp, f32, vp, vp, vp, i64, i64, i64, vp, ci, C.POINTER(Epilogue), vp]),
        "mkq_bert_layer_workspace": (ci, [C.POINTER(BertLayerParams), C.POINTER(BertLayerWorkspaceLayout)]),
        "mkq_bert_layer_int4": (ci, [C.POINTER(BertLayerParams), vp, ci, vp, vp, vp, vp, sz, vp]),
        "mkq_bert_layer_fp16_workspace_bytes": (sz, [C.POINTER(BertLayerParamsFp16)]),
        "mkq_bert_layer_fp16": (ci, [C.POINTER(BertLayerParamsFp16), vp, vp, vp, sz, vp]),
        "mkq_layernorm": (ci, [vp, i64, i64, vp, vp, f32, vp, f32, vp, vp]),
        "mkq_attention": (ci, [vp, i64, i64, i64, i64, vp, f32, vp, vp]),
        "mkq_attention_varlen": (ci, [vp, vp, i64, i64, i64, i64, vp, f32, vp, ci, vp]),
        "mkq_layernorm_int8": (ci, [vp, i64, i64, vp, vp, f32, vp, f32, vp, vp]),
        "mkq_attention_int8": (ci, [vp, i64, i64, i64, i64, vp, f32, vp, vp]),
        "mkq_bert_layer_int8_workspace": (ci, [C.POINTER(BertLayerParams), C.POINTER(BertLayerWorkspaceLayout)]),
        "mkq_bert_layer_int8": (ci, [C.POINTER(BertLayerParams), vp, ci, vp, vp, vp, vp, sz, vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().mkq_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != MKQ_OK:
        raise MkqError(status, where)


def _torch():
    import torch
    return torch


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _dtype_code(t):
    torch = _torch()
    return {torch.float32: MKQ_F32, torch.float16: MKQ_F16, torch.bfloat16: MKQ_BF16}[t.dtype]


def _torch_dtype(code):
    torch = _torch()
    return {MKQ_F32: torch.float32, MKQ_F16: torch.float16, MKQ_BF16: torch.bfloat16}[code]


# ----------------------------------------------------------------------------------
# Same names as the C entry points.  Tensors are torch CUDA tensors; outputs are
# allocated with torch when not passed in.

def mkq_version() -> int:
    return int(load().mkq_version())


def mkq_quantize(x, s_x: float, q_out=None, stream=None):
    """x [M,K] float32/float16 -> packed codes uint8 [M,K/2]."""
    torch = _torch()
    M, K = x.shape
    if q_out is None:
        q_out = torch.empty((M, K // 2), dtype=torch.uint8, device=x.device)
    _check(load().mkq_quantize(_ptr(x), _dtype_code(x), M, K, x.stride(0), float(s_x), _ptr(q_out),
                               _stream(stream)), "mkq_quantize")
    return q_out


def mkq_absmax_scale(x, per_row: bool = False, s_out=None, stream=None):
    torch = _torch()
    M, K = x.shape
    if s_out is None:
        s_out = torch.empty(M if per_row else 1, dtype=torch.float32, device=x.device)
    _check(load().mkq_absmax_scale(_ptr(x), _dtype_code(x), M, K, x.stride(0), int(per_row),
                                   _ptr(s_out), _stream(stream)), "mkq_absmax_scale")
    return s_out


def mkq_scale_gradients(x, s: float, bits: int = 4, g_out=None, stream=None):
    """(STE-based, MSE-based) scale-gradient sums of x [M,K] under step s -> float64 tensor [2]."""
    torch = _torch()
    M, K = x.shape
    if g_out is None:
        g_out = torch.empty(2, dtype=torch.float64, device=x.device)
    _check(load().mkq_scale_gradients(_ptr(x), _dtype_code(x), M, K, x.stride(0), float(s), int(bits), _ptr(g_out),
                                      _stream(stream)), "mkq_scale_gradients")
    return g_out


def mkq_percentile_scale_workspace_bytes() -> int:
    return int(load().mkq_percentile_scale_workspace_bytes())


def mkq_percentile_scale(x, top_ppm: int = 100, bits: int = 4, s_out=None, workspace=None, stream=None):
    """Step from the k-th largest |x| (k = max(1, n*top_ppm // 10**6)) -> float32 tensor [1]."""
    torch = _torch()
    M, K = x.shape
    if s_out is None:
        s_out = torch.empty(1, dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(mkq_percentile_scale_workspace_bytes(), dtype=torch.uint8, device=x.device)
    _check(load().mkq_percentile_scale(_ptr(x), _dtype_code(x), M, K, x.stride(0), int(top_ppm), int(bits),
                                       _ptr(s_out), _ptr(workspace), workspace.numel(), _stream(stream)),
           "mkq_percentile_scale")
    return s_out


def mkq_packed_weight_bytes(N: int, K: int) -> int:
    return int(load().mkq_packed_weight_bytes(N, K))


def mkq_pack_weights_int4(W, s_w_in=None, stream=None):
    """W [N,K] float32 -> (Wq uint8 [packed bytes], s_w float32 [N])."""
    torch = _torch()
    N, K = W.shape
    nbytes = mkq_packed_weight_bytes(N, K)
    Wq = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=W.device)
    s_w = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(load().mkq_pack_weights_int4(_ptr(W), N, K, _ptr(s_w_in), _ptr(s_w), _ptr(Wq),
                                        _stream(stream)), "mkq_pack_weights_int4")
    return Wq, s_w


def mkq_padded_k(K: int) -> int:
    """Smallest multiple of 128 >= K: the row length, in codes, of operands stored with zero padding."""
    return int(load().mkq_padded_k(K))


def mkq_quantize_padded(x, s_x: float, q_out=None, stream=None):
    """x [M,K] float32/float16, K % 8 == 0 -> packed codes uint8 [M, mkq_padded_k(K)/2], zero codes past K."""
    torch = _torch()
    M, K = x.shape
    if q_out is None:
        q_out = torch.empty((M, mkq_padded_k(K) // 2), dtype=torch.uint8, device=x.device)
    _check(load().mkq_quantize_padded(_ptr(x), _dtype_code(x), M, K, x.stride(0), float(s_x), _ptr(q_out),
                                      _stream(stream)), "mkq_quantize_padded")
    return q_out


def mkq_pack_weights_int4_padded(W, s_w_in=None, stream=None):
    """W [N,K] float32, K % 8 == 0 -> (Wq uint8 [N * mkq_padded_k(K)/2], s_w float32 [N])."""
    torch = _torch()
    N, K = W.shape
    Wq = torch.empty(max(N * mkq_padded_k(K) // 2, 1), dtype=torch.uint8, device=W.device)
    s_w = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(load().mkq_pack_weights_int4_padded(_ptr(W), N, K, _ptr(s_w_in), _ptr(s_w), _ptr(Wq),
                                               _stream(stream)), "mkq_pack_weights_int4_padded")
    return Wq, s_w


def mkq_pack_codes_int4(codes, stream=None):
    torch = _torch()
    rows, K = codes.shape
    q = torch.empty((rows, K // 2), dtype=torch.uint8, device=codes.device)
    _check(load().mkq_pack_codes_int4(_ptr(codes), rows, K, _ptr(q), _stream(stream)),
           "mkq_pack_codes_int4")
    return q


def mkq_unpack_weights_int4(Wq, N: int, K: int, stream=None):
    torch = _torch()
    codes = torch.empty((N, K), dtype=torch.int8, device=Wq.device)
    _check(load().mkq_unpack_weights_int4(_ptr(Wq), N, K, _ptr(codes), _stream(stream)),
           "mkq_unpack_weights_int4")
    return codes


def mkq_linear_int4_workspace_bytes(M: int, N: int, K: int, a_dtype: int) -> int:
    return int(load().mkq_linear_int4_workspace_bytes(M, N, K, a_dtype))


def mkq_init() -> None:
    _check(load().mkq_init(), "mkq_init")


def mkq_splitk_scratch_bytes() -> int:
    return int(load().mkq_splitk_scratch_bytes())


def mkq_splitk_scratch_init(scratch=None, device="cuda", stream=None):
    """A scratch area for K splits across workgroups, counters cleared (allocated here when not passed in)."""
    torch = _torch()
    if scratch is None:
        scratch = torch.empty(mkq_splitk_scratch_bytes(), dtype=torch.uint8, device=device)
    _check(load().mkq_splitk_scratch_init(_ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream)),
           "mkq_splitk_scratch_init")
    return scratch


def mkq_linear_int4(a, s_x: float, Wq, s_w, bias, N: int, K: int, out_dtype: int = MKQ_F32, *,
                    a_is_codes: bool | None = None, act: int = MKQ_ACT_NONE, residual=None,
                    s_next: float = 0.0, want_q: bool = False, want_acc: bool = False,
                    out=None, workspace=None, stream=None, splitk_scratch=None,
                    config: int | None = None, k_slices: int = 0, w_stream: bool = False,
                    prefetch_stages: int = 0, q_pitch: int = 0, q_out=None):
    """The quantized linear.  ``a`` is packed codes (uint8 [M,K/2]) or float [M,K].

    Returns a dict with ``out`` (float tensor, or uint8 [M,N/2] for MKQ_I4) and
    optionally ``q`` (packed codes under s_next) and ``acc`` (int32 [M,N]).
    ``config`` / ``k_slices`` call mkq_tuning_linear_int4 (the kernel configuration chosen by the caller).
    ``w_stream``: Wq is in the streaming layout (mkq_linear_int4_stream; ``prefetch_stages`` / ``k_slices``
    call its tuning variant).  ``q_pitch``: codes per row of the code outputs (0 = N; the columns from N on are written
    as zero codes).  ``q_out``: the caller's buffer for the extra codes (implies ``want_q``).
    """
    torch = _torch()
    if a_is_codes is None:
        a_is_codes = a.dtype == torch.uint8
    M = a.shape[0]
    a_dtype = MKQ_I4 if a_is_codes else _dtype_code(a)
    dev = a.device
    code_cols = (int(q_pitch) or N) // 2
    if out is None:
        out = (torch.empty((M, code_cols), dtype=torch.uint8, device=dev) if out_dtype == MKQ_I4
               else torch.empty((M, N), dtype=_torch_dtype(out_dtype), device=dev))
    q = q_out if q_out is not None else (torch.empty((M, code_cols), dtype=torch.uint8, device=dev) if want_q else None)
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    epi = Epilogue(act=int(act), residual=residual.data_ptr() if residual is not None else None,
                   residual_dtype=_dtype_code(residual) if residual is not None else MKQ_F32,
                   s_next=float(s_next), q_out=q.data_ptr() if q is not None else None,
                   acc_out=acc.data_ptr() if acc is not None else None,
                   splitk_scratch=splitk_scratch.data_ptr() if splitk_scratch is not None else None,
                   splitk_scratch_bytes=(splitk_scratch.numel() * splitk_scratch.element_size()
                                         if splitk_scratch is not None else 0), q_pitch=int(q_pitch))
    need = mkq_linear_int4_workspace_bytes(M, N, K, a_dtype)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    if w_stream:
        if not prefetch_stages and not k_slices:
            _check(load().mkq_linear_int4_stream(_ptr(a), a_dtype, float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias),
                                                 M, N, K, _ptr(out), int(out_dtype), C.byref(epi), _ptr(workspace),
                                                 ws_bytes, _stream(stream)), "mkq_linear_int4_stream")
        else:
            _check(load().mkq_tuning_linear_int4_stream(_ptr(a), a_dtype, float(s_x), _ptr(Wq), _ptr(s_w),
                                                        _ptr(bias), M, N, K, _ptr(out), int(out_dtype),
                                                        C.byref(epi), _ptr(workspace), ws_bytes, _stream(stream),
                                                        int(prefetch_stages), int(k_slices)),
                   "mkq_tuning_linear_int4_stream")
    elif config is None and not k_slices:
        _check(load().mkq_linear_int4(_ptr(a), a_dtype, float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias),
                                      M, N, K, _ptr(out), int(out_dtype), C.byref(epi), _ptr(workspace),
                                      ws_bytes, _stream(stream)), "mkq_linear_int4")
    else:
        _check(load().mkq_tuning_linear_int4(_ptr(a), a_dtype, float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias),
                                             M, N, K, _ptr(out), int(out_dtype), C.byref(epi), _ptr(workspace),
                                             ws_bytes, _stream(stream), -1 if config is None else int(config),
                                             int(k_slices)), "mkq_tuning_linear_int4")
    return {"out": out, "q": q, "acc": acc}


def mkq_linear_int4_stream(a, s_x, Wq_stream, s_w, bias, N, K, out_dtype=MKQ_F32, **kw):
    """mkq_linear_int4 on weights in the streaming layout (M <= 128)."""
    return mkq_linear_int4(a, s_x, Wq_stream, s_w, bias, N, K, out_dtype, w_stream=True, **kw)


def mkq_linear_int4_stream_static(a, s_x: float, Wq_stream, s_w, bias, N: int, K: int, out_dtype: int = MKQ_F32, *,
                                  act: int = MKQ_ACT_NONE, residual=None, s_next: float = 0.0, out=None,
                                  q_out=None, acc_out=None, stream=None):
    """mkq_linear_int4_stream on packed codes with the library's own scratch: nothing is allocated by the C
    call (outputs are the caller's: ``out`` and, optionally, ``q_out`` / ``acc_out`` must be passed in)."""
    M = a.shape[0]
    epi = Epilogue(act=int(act), residual=residual.data_ptr() if residual is not None else None,
                   residual_dtype=_dtype_code(residual) if residual is not None else MKQ_F32,
                   s_next=float(s_next), q_out=q_out.data_ptr() if q_out is not None else None,
                   acc_out=acc_out.data_ptr() if acc_out is not None else None,
                   splitk_scratch=None, splitk_scratch_bytes=0)
    _check(load().mkq_linear_int4_stream_static(_ptr(a), float(s_x), _ptr(Wq_stream), _ptr(s_w), _ptr(bias), M, N, K,
                                                _ptr(out), int(out_dtype), C.byref(epi), _stream(stream)),
           "mkq_linear_int4_stream_static")
    return out


def mkq_measure_stream(kind: int, src, dst, nbytes: int, stream=None):
    _check(load().mkq_measure_stream(int(kind), _ptr(src), _ptr(dst), int(nbytes), _stream(stream)), "mkq_measure_stream")


def mkq_measure_mfma_i8(operands, iters: int, sink, stream=None):
    """One launch of the register-only int8 MFMA loop; returns the integer operations it performs."""
    _check(load().mkq_measure_mfma_i8(_ptr(operands), operands.numel() * operands.element_size(), int(iters),
                                      _ptr(sink), _stream(stream)), "mkq_measure_mfma_i8")
    return int(load().mkq_measure_mfma_i8_ops(int(iters)))


def mkq_stream_weight_bytes(N: int, K: int) -> int:
    return int(load().mkq_stream_weight_bytes(N, K))


def mkq_repack_weights_int4_stream(Wq, N: int, K: int, out=None, stream=None):
    """Canonical packed weights -> the streaming layout (uint8 [mkq_stream_weight_bytes(N, K)])."""
    torch = _torch()
    if out is None:
        out = torch.empty(mkq_stream_weight_bytes(N, K), dtype=torch.uint8, device=Wq.device)
    _check(load().mkq_repack_weights_int4_stream(_ptr(Wq), N, K, _ptr(out), _stream(stream)),
           "mkq_repack_weights_int4_stream")
    return out


def mkq_quantize_int8(x, s_x: float, q_out=None, stream=None):
    """x [M,K] float32/float16 -> int8 codes [M,K] (8-bit range of the quantizer)."""
    torch = _torch()
    M, K = x.shape
    if q_out is None:
        q_out = torch.empty((M, K), dtype=torch.int8, device=x.device)
    _check(load().mkq_quantize_int8(_ptr(x), _dtype_code(x), M, K, x.stride(0), float(s_x), _ptr(q_out),
                                    _stream(stream)), "mkq_quantize_int8")
    return q_out


def mkq_pack_weights_int8(W, s_w_in=None, stream=None):
    """W [N,K] float32 -> (int8 codes [N,K], s_w float32 [N])."""
    torch = _torch()
    N, K = W.shape
    Wq = torch.empty((N, K), dtype=torch.int8, device=W.device)
    s_w = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(load().mkq_pack_weights_int8(_ptr(W), N, K, _ptr(s_w_in), _ptr(s_w), _ptr(Wq),
                                        _stream(stream)), "mkq_pack_weights_int8")
    return Wq, s_w


def mkq_linear_int8(a, s_x: float, Wq, s_w, bias, out_dtype: int = MKQ_F32, *, act: int = MKQ_ACT_NONE,
                    residual=None, s_next: float = 0.0, want_acc: bool = False, out=None, stream=None,
                    config: int | None = None, q_pitch: int = 0):
    """The 8-bit linear: ``a`` int8 codes [M,K], ``Wq`` int8 codes [N,K].  ``config``: mkq_tuning_linear_int8.
    ``q_pitch``: codes per row of an int8 code output (0 = N; the padding columns are written as zeros)."""
    torch = _torch()
    M, K = a.shape
    N = Wq.shape[0]
    if out is None:
        cols = int(q_pitch) if (out_dtype == MKQ_I8 and q_pitch) else N
        out = torch.empty((M, cols), dtype=torch.int8 if out_dtype == MKQ_I8 else _torch_dtype(out_dtype),
                          device=a.device)
    acc = torch.empty((M, N), dtype=torch.int32, device=a.device) if want_acc else None
    epi = Epilogue(act=int(act), residual=residual.data_ptr() if residual is not None else None,
                   residual_dtype=_dtype_code(residual) if residual is not None else MKQ_F32,
                   s_next=float(s_next), q_out=None, acc_out=acc.data_ptr() if acc is not None else None,
                   q_pitch=int(q_pitch))
    if config is None:
        _check(load().mkq_linear_int8(_ptr(a), float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias), M, N, K, _ptr(out),
                                      int(out_dtype), C.byref(epi), _stream(stream)), "mkq_linear_int8")
    else:
        _check(load().mkq_tuning_linear_int8(_ptr(a), float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias), M, N, K, _ptr(out),
                                             int(out_dtype), C.byref(epi), _stream(stream), int(config)),
               "mkq_tuning_linear_int8")
    return {"out": out, "acc": acc}


def mkq_quantize_e3m2(x, s_x: float, stream=None):
    """x [M,K] float -> E3M2 containers uint8 [M, 3K/4] (experimental 6-bit float path)."""
    torch = _torch()
    M, K = x.shape
    q = torch.empty((M, K * 3 // 4), dtype=torch.uint8, device=x.device)
    _check(load().mkq_quantize_e3m2(_ptr(x), _dtype_code(x), M, K, x.stride(0), float(s_x), _ptr(q),
                                    _stream(stream)), "mkq_quantize_e3m2")
    return q


def mkq_pack_codes_e3m2(codes, stream=None):
    torch = _torch()
    rows, K = codes.shape
    q = torch.empty((rows, K * 3 // 4), dtype=torch.uint8, device=codes.device)
    _check(load().mkq_pack_codes_e3m2(_ptr(codes), rows, K, _ptr(q), _stream(stream)), "mkq_pack_codes_e3m2")
    return q


def mkq_pack_weights_e3m2(W, s_w_in=None, stream=None):
    torch = _torch()
    N, K = W.shape
    Wq = torch.empty((N, K * 3 // 4), dtype=torch.uint8, device=W.device)
    s_w = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(load().mkq_pack_weights_e3m2(_ptr(W), N, K, _ptr(s_w_in), _ptr(s_w), _ptr(Wq), _stream(stream)),
           "mkq_pack_weights_e3m2")
    return Wq, s_w


def mkq_linear_int4_e3m2(a, s_x: float, Wq, s_w, bias, out_dtype: int = MKQ_F32, *, act: int = MKQ_ACT_NONE,
                         residual=None, s_next: float = 0.0, want_q: bool = False, want_acc: bool = False,
                         out=None, stream=None, config: int | None = None):
    """The 4-bit linear on E3M2 containers: a uint8 [M, 3K/4], Wq uint8 [N, 3K/4].
    ``config`` calls mkq_tuning_linear_int4_e3m2."""
    torch = _torch()
    M, K = a.shape[0], a.shape[1] * 4 // 3
    N = Wq.shape[0]
    dev = a.device
    if out is None:
        out = (torch.empty((M, N // 2), dtype=torch.uint8, device=dev) if out_dtype == MKQ_I4
               else torch.empty((M, N), dtype=_torch_dtype(out_dtype), device=dev))
    q = torch.empty((M, N // 2), dtype=torch.uint8, device=dev) if want_q else None
    acc = torch.empty((M, N), dtype=torch.int32, device=dev) if want_acc else None
    epi = Epilogue(act=int(act), residual=residual.data_ptr() if residual is not None else None,
                   residual_dtype=_dtype_code(residual) if residual is not None else MKQ_F32,
                   s_next=float(s_next), q_out=q.data_ptr() if q is not None else None,
                   acc_out=acc.data_ptr() if acc is not None else None)
    if config is None:
        _check(load().mkq_linear_int4_e3m2(_ptr(a), float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias), M, N, K, _ptr(out),
                                           int(out_dtype), C.byref(epi), _stream(stream)), "mkq_linear_int4_e3m2")
    else:
        _check(load().mkq_tuning_linear_int4_e3m2(_ptr(a), float(s_x), _ptr(Wq), _ptr(s_w), _ptr(bias), M, N, K,
                                                  _ptr(out), int(out_dtype), C.byref(epi), _stream(stream),
                                                  int(config)), "mkq_tuning_linear_int4_e3m2")
    return {"out": out, "q": q, "acc": acc}


def mkq_linear_fp16(a, W, bias, out_dtype: int = MKQ_F16, act: int = MKQ_ACT_NONE, residual=None,
                    out=None, stream=None):
    torch = _torch()
    M, K = a.shape
    N = W.shape[0]
    if out is None:
        out = torch.empty((M, N), dtype=_torch_dtype(out_dtype), device=a.device)
    _check(load().mkq_linear_fp16(_ptr(a), _ptr(W), _ptr(bias), M, N, K, _ptr(out), int(out_dtype),
                                  int(act), _ptr(residual), _stream(stream)), "mkq_linear_fp16")
    return out


def mkq_layernorm(x, gamma, beta, eps: float, s_next: float = 0.0, want_y: bool = True,
                  want_q: bool = False, stream=None):
    torch = _torch()
    M, D = x.shape
    y = torch.empty((M, D), dtype=torch.float16, device=x.device) if want_y else None
    q = torch.empty((M, D // 2), dtype=torch.uint8, device=x.device) if want_q else None
    _check(load().mkq_layernorm(_ptr(x), M, D, _ptr(gamma), _ptr(beta), float(eps), _ptr(y),
                                float(s_next), _ptr(q), _stream(stream)), "mkq_layernorm")
    return y, q


def mkq_attention(qkv, batch: int, seq: int, hidden: int, heads: int, s_next: float = 0.0,
                  want_ctx: bool = True, want_q: bool = False, stream=None):
    torch = _torch()
    M = batch * seq
    ctx = torch.empty((M, hidden), dtype=torch.float16, device=qkv.device) if want_ctx else None
    q = torch.empty((M, hidden // 2), dtype=torch.uint8, device=qkv.device) if want_q else None
    _check(load().mkq_attention(_ptr(qkv), batch, seq, hidden, heads, _ptr(ctx), float(s_next),
                                _ptr(q), _stream(stream)), "mkq_attention")
    return ctx, q


def mkq_layernorm_int8(x, gamma, beta, eps: float, s_next: float, want_y: bool = True, stream=None):
    torch = _torch()
    M, D = x.shape
    y = torch.empty((M, D), dtype=torch.float16, device=x.device) if want_y else None
    q = torch.empty((M, D), dtype=torch.int8, device=x.device)
    _check(load().mkq_layernorm_int8(_ptr(x), M, D, _ptr(gamma), _ptr(beta), float(eps), _ptr(y),
                                     float(s_next), _ptr(q), _stream(stream)), "mkq_layernorm_int8")
    return y, q


def mkq_attention_int8(qkv, batch: int, seq: int, hidden: int, heads: int, s_next: float,
                       want_ctx: bool = True, stream=None):
    torch = _torch()
    M = batch * seq
    ctx = torch.empty((M, hidden), dtype=torch.float16, device=qkv.device) if want_ctx else None
    q = torch.empty((M, hidden), dtype=torch.int8, device=qkv.device)
    _check(load().mkq_attention_int8(_ptr(qkv), batch, seq, hidden, heads, _ptr(ctx), float(s_next),
                                     _ptr(q), _stream(stream)), "mkq_attention_int8")
    return ctx, q


def mkq_attention_varlen(qkv, cu_seqlens, max_seq: int, hidden: int, heads: int, s_next: float = 0.0,
                         want_ctx: bool = True, q_bits: int = 0, stream=None):
    """Attention over a padding-free batch; cu_seqlens int32 device tensor [batch + 1]."""
    torch = _torch()
    total = qkv.shape[0]
    batch = cu_seqlens.numel() - 1
    ctx = torch.empty((total, hidden), dtype=torch.float16, device=qkv.device) if want_ctx else None
    q = None
    if q_bits == 4:
        q = torch.empty((total, hidden // 2), dtype=torch.uint8, device=qkv.device)
    elif q_bits == 8:
        q = torch.empty((total, hidden), dtype=torch.int8, device=qkv.device)
    _check(load().mkq_attention_varlen(_ptr(qkv), _ptr(cu_seqlens), batch, max_seq, hidden, heads, _ptr(ctx),
                                       float(s_next), _ptr(q), int(q_bits) if q_bits else 4, _stream(stream)),
           "mkq_attention_varlen")
    return ctx, q


class BertLayerInt4:
    """Holds the device tensors of one W4A4 encoder layer and its parameter struct."""
    _workspace_fn = "mkq_bert_layer_workspace"
    _run_fn = "mkq_bert_layer_int4"

    def __init__(self, batch, seq, hidden, heads, ffn, packed: dict, sx: dict, ln: dict, ln_eps: float,
                 s_out_next: float = 0.0, next_bits: int = 0, cu_seqlens=None, total_tokens: int = 0):
        self._keep = (packed, ln, cu_seqlens)
        p = BertLayerParams()
        p.next_bits = int(next_bits)
        if cu_seqlens is not None:  # padding-free batch: seq is the upper bound of the lengths
            p.cu_seqlens, p.total_tokens = cu_seqlens.data_ptr(), int(total_tokens)
        p.batch, p.seq, p.hidden, p.heads, p.ffn = batch, seq, hidden, heads, ffn
        for nm in ("qkv", "ao", "up", "down"):
            Wq, s_w, b = packed[nm]
            setattr(p, "Wq_" + nm, Wq.data_ptr())
            setattr(p, "sw_" + nm, s_w.data_ptr())
            setattr(p, "b_" + nm, b.data_ptr())
            setattr(p, "sx_" + nm, float(sx[nm]))
        for nm in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta"):
            setattr(p, nm, ln[nm].data_ptr())
        p.ln_eps = float(ln_eps)
        p.s_out_next = float(s_out_next)
        self.params = p
        self.layout = BertLayerWorkspaceLayout()
        _check(getattr(load(), self._workspace_fn)(C.byref(p), C.byref(self.layout)), self._workspace_fn)
        self.M, self.hidden, self.ffn = (int(total_tokens) if cu_seqlens is not None else batch * seq), hidden, ffn

    def workspace_bytes(self) -> int:
        return int(self.layout.total)

    def __call__(self, h_in, workspace, h_out=None, q_in=None, q_out_next=None, stream=None):
        torch = _torch()
        if h_out is None:
            h_out = torch.empty((self.M, self.hidden), dtype=torch.float16, device=h_in.device)
        _check(getattr(load(), self._run_fn)(C.byref(self.params), _ptr(h_in), _dtype_code(h_in), _ptr(q_in),
                                             _ptr(h_out), _ptr(q_out_next), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)),
               self._run_fn)
        return h_out


class BertLayerInt8(BertLayerInt4):
    """The same layer W8A8: ``packed`` holds int8 weights from mkq_pack_weights_int8, code buffers are int8."""
    _workspace_fn = "mkq_bert_layer_int8_workspace"
    _run_fn = "mkq_bert_layer_int8"


class BertLayerFp16:
    """The 16-bit float baseline layer."""

    def __init__(self, batch, seq, hidden, heads, ffn, weights: dict, ln: dict, ln_eps: float, cu_seqlens=None,
                 total_tokens: int = 0):
        self._keep = (weights, ln, cu_seqlens)
        p = BertLayerParamsFp16()
        if cu_seqlens is not None:
            p.cu_seqlens, p.total_tokens = cu_seqlens.data_ptr(), int(total_tokens)
        p.batch, p.seq, p.hidden, p.heads, p.ffn = batch, seq, hidden, heads, ffn
        for nm in ("qkv", "ao", "up", "down"):
            W, b = weights[nm]
            setattr(p, "W_" + nm, W.data_ptr())
            setattr(p, "b_" + nm, b.data_ptr())
        for nm in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta"):
            setattr(p, nm, ln[nm].data_ptr())
        p.ln_eps = float(ln_eps)
        self.params = p
        self.M, self.hidden = (int(total_tokens) if cu_seqlens is not None else batch * seq), hidden

    def workspace_bytes(self) -> int:
        return int(load().mkq_bert_layer_fp16_workspace_bytes(C.byref(self.params)))

    def __call__(self, h_in, workspace, h_out=None, stream=None):
        torch = _torch()
        if h_out is None:
            h_out = torch.empty((self.M, self.hidden), dtype=torch.float16, device=h_in.device)
        _check(load().mkq_bert_layer_fp16(C.byref(self.params), _ptr(h_in), _ptr(h_out), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(stream)),
               "mkq_bert_layer_fp16")
        return h_out
