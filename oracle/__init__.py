"""CPU oracle for the W4A4 quantized BERT linear layer (test infrastructure only).

The arithmetic lives in ``mkq_oracle.c`` (plain C, built with gcc); this module
only compiles it, loads it with ctypes and marshals numpy arrays.  Nothing here
is imported by the product package: only tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may use it.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mkq_oracle.c")
_LIB = os.path.join(_HERE, "libmkq_oracle.so")

QMIN, QMAX = -8, 7
F32, F16, BF16 = 0, 1, 2
ACT_NONE, ACT_GELU = 0, 1


CFLAGS = ["-O2", "-march=native", "-fopenmp", "-ffp-contract=off"]
# MKQ_ORACLE_SANITIZE=undefined: the same source built with the undefined-behaviour sanitizer (any report aborts
# the process); the CPU test tier runs the oracle's pins once more under it.  (The address sanitizer needs its
# runtime loaded before anything else, which a library loaded into Python cannot arrange: it runs in the
# stand-alone driver sanitize_driver.c instead.)
_SANITIZE = os.environ.get("MKQ_ORACLE_SANITIZE", "")
if _SANITIZE:
    assert _SANITIZE == "undefined", "MKQ_ORACLE_SANITIZE: only 'undefined' can be loaded into Python"
    CFLAGS = ["-O1", "-g", "-fopenmp", "-ffp-contract=off", "-fsanitize=undefined", "-fno-sanitize-recover=all"]
    _LIB = os.path.join(_HERE, "libmkq_oracle_ubsan.so")


def build_sanitizer_driver(out_path: str) -> str:
    """Compile sanitize_driver.c (with the oracle inside it) under the address and undefined-behaviour sanitizers."""
    cmd = ["gcc", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fopenmp",
           "-ffp-contract=off", "-Wall", "-Wextra", "-o", out_path, os.path.join(_HERE, "sanitize_driver.c"), "-lm"]
    subprocess.run(cmd, check=True)
    return out_path


def build_flags() -> str:
    """The compiler and flags the oracle is built with (quoted beside its timing)."""
    return "gcc " + " ".join(CFLAGS)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no HIP, no BLAS).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", *CFLAGS, "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
    return _lib


def num_threads() -> int:
    return int(lib().mkq_ref_num_threads())


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i8(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int8)


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def quantize(x, s, qmin=QMIN, qmax=QMAX):
    """Eq. 1 integer part on a 2-D (or flattened) array -> int8 codes."""
    x = _f32(x)
    shape = x.shape
    x2 = x.reshape(-1, shape[-1]) if x.ndim >= 1 and x.size else x.reshape(0, 1)
    M, K = x2.shape
    out = np.empty((M, K), np.int8)
    rc = lib().mkq_ref_quantize(_p(x2, C.c_float), C.c_int64(M), C.c_int64(K), C.c_int64(K),
                                C.c_float(s), qmin, qmax, _p(out, C.c_int8))
    _check(rc, "quantize")
    return out.reshape(shape)


def dequantize(codes, s):
    codes = _i8(codes)
    out = np.empty(codes.shape, np.float32)
    _check(lib().mkq_ref_dequantize(_p(codes, C.c_int8), C.c_int64(codes.size), C.c_float(s),
                                    _p(out, C.c_float)), "dequantize")
    return out


def absmax_scale(x, per_row=False, qmax=QMAX):
    x = _f32(x)
    M, K = x.shape
    out = np.empty(M if per_row else 1, np.float32)
    _check(lib().mkq_ref_absmax_scale(_p(x, C.c_float), C.c_int64(M), C.c_int64(K), C.c_int64(K),
                                      int(per_row), qmax, _p(out, C.c_float)), "absmax_scale")
    return out if per_row else float(out[0])


def percentile_scale(x, top_ppm=100, qmax=QMAX):
    """(s, T): T = k-th largest |x|, k = max(1, n*top_ppm // 10**6); s = T / qmax."""
    x = _f32(x).ravel()
    s, t = C.c_float(), C.c_float()
    _check(lib().mkq_ref_percentile_scale(_p(x, C.c_float), C.c_int64(x.size), C.c_int64(top_ppm), int(qmax),
                                          C.byref(s), C.byref(t)), "percentile_scale")
    return float(s.value), float(t.value)


def quantize_weights(W, s_w=None, qmin=QMIN, qmax=QMAX):
    """Per-output-channel weight quantization -> (codes [N,K] int8, s_w [N] f32)."""
    W = _f32(W)
    N, K = W.shape
    s_in = _f32(s_w)
    s_out = np.empty(N, np.float32)
    codes = np.empty((N, K), np.int8)
    _check(lib().mkq_ref_quantize_weights(_p(W, C.c_float), C.c_int64(N), C.c_int64(K),
                                          _p(s_in, C.c_float), qmin, qmax, _p(s_out, C.c_float),
                                          _p(codes, C.c_int8)), "quantize_weights")
    return codes, s_out


def pack_nibbles(codes):
    codes = _i8(codes)
    rows, K = codes.shape
    out = np.empty((rows, K // 2), np.uint8)
    _check(lib().mkq_ref_pack_nibbles(_p(codes, C.c_int8), C.c_int64(rows), C.c_int64(K),
                                      _p(out, C.c_uint8)), "pack_nibbles")
    return out


def unpack_nibbles(packed, K):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    rows = packed.size // (K // 2) if K else 0
    out = np.empty((rows, K), np.int8)
    _check(lib().mkq_ref_unpack_nibbles(_p(packed, C.c_uint8), C.c_int64(rows), C.c_int64(K),
                                        _p(out, C.c_int8)), "unpack_nibbles")
    return out


def gemm_codes(a, w):
    a, w = _i8(a), _i8(w)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    acc = np.empty((M, N), np.int32)
    _check(lib().mkq_ref_gemm_codes(_p(a, C.c_int8), _p(w, C.c_int8), C.c_int64(M), C.c_int64(N),
                                    C.c_int64(K), _p(acc, C.c_int32)), "gemm_codes")
    return acc


def epilogue(acc, s_x, s_w, bias=None, residual=None, act=ACT_NONE):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    s_w, bias, residual = _f32(s_w), _f32(bias), _f32(residual)
    y = np.empty((M, N), np.float32)
    _check(lib().mkq_ref_epilogue(_p(acc, C.c_int32), C.c_int64(M), C.c_int64(N), C.c_float(s_x),
                                  _p(s_w, C.c_float), _p(bias, C.c_float), _p(residual, C.c_float),
                                  int(act), _p(y, C.c_float)), "epilogue")
    return y


def round_storage(x, dtype):
    """Round-to-nearest-even narrowing to F16/BF16, returned as float32 values."""
    y = np.array(x, dtype=np.float32, copy=True, order="C")
    _check(lib().mkq_ref_round_storage(_p(y, C.c_float), C.c_int64(y.size), int(dtype)), "round")
    return y


def linear_int4(a_codes, s_x, w_codes, s_w, bias=None, residual=None, act=ACT_NONE,
                out_dtype=F32, s_next=None, qmin=QMIN, qmax=QMAX):
    """Whole quantized linear on codes.  Returns dict(acc, y, q) (q only with s_next)."""
    a, w = _i8(a_codes), _i8(w_codes)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    s_w, bias, residual = _f32(s_w), _f32(bias), _f32(residual)
    acc = np.empty((M, N), np.int32)
    y = np.empty((M, N), np.float32)
    q = np.empty((M, N), np.int8) if s_next is not None else None
    _check(lib().mkq_ref_linear_int4(_p(a, C.c_int8), C.c_float(s_x), _p(w, C.c_int8),
                                     _p(s_w, C.c_float), _p(bias, C.c_float), C.c_int64(M),
                                     C.c_int64(N), C.c_int64(K), _p(residual, C.c_float), int(act),
                                     int(out_dtype), C.c_float(s_next if s_next is not None else 0.0),
                                     int(qmin), int(qmax), _p(acc, C.c_int32), _p(y, C.c_float), _p(q, C.c_int8)),
           "linear_int4")
    return {"acc": acc, "y": y, "q": q}


def linear_float(a, W, bias=None, residual=None, act=ACT_NONE, out_dtype=F32):
    a, W = _f32(a), _f32(W)
    M, K = a.shape
    N = W.shape[0]
    bias, residual = _f32(bias), _f32(residual)
    y = np.empty((M, N), np.float32)
    _check(lib().mkq_ref_linear_float(_p(a, C.c_float), _p(W, C.c_float), _p(bias, C.c_float),
                                      C.c_int64(M), C.c_int64(N), C.c_int64(K),
                                      _p(residual, C.c_float), int(act), int(out_dtype),
                                      _p(y, C.c_float)), "linear_float")
    return y


def layernorm(x, gamma=None, beta=None, eps=1e-12):
    x = _f32(x)
    M, D = x.shape
    gamma, beta = _f32(gamma), _f32(beta)
    y = np.empty((M, D), np.float32)
    _check(lib().mkq_ref_layernorm(_p(x, C.c_float), C.c_int64(M), C.c_int64(D),
                                   _p(gamma, C.c_float), _p(beta, C.c_float), C.c_float(eps),
                                   _p(y, C.c_float)), "layernorm")
    return y


def attention(qkv, B, S, H, heads, p_dtype=F32):
    qkv = _f32(qkv)
    assert qkv.shape == (B * S, 3 * H)
    ctx = np.empty((B * S, H), np.float32)
    _check(lib().mkq_ref_attention(_p(qkv, C.c_float), C.c_int64(B), C.c_int64(S), C.c_int64(H),
                                   C.c_int64(heads), int(p_dtype), _p(ctx, C.c_float)), "attention")
    return ctx


class _LayerParams(C.Structure):
    _fields_ = ([(n, C.c_int64) for n in ("batch", "seq", "hidden", "heads", "ffn")]
                + [(n, C.POINTER(C.c_int8)) for n in ("w_qkv", "w_ao", "w_up", "w_down")]
                + [(n, C.POINTER(C.c_float)) for n in ("sw_qkv", "sw_ao", "sw_up", "sw_down",
                                                        "b_qkv", "b_ao", "b_up", "b_down")]
                + [(n, C.c_float) for n in ("sx_qkv", "sx_ao", "sx_up", "sx_down")]
                + [(n, C.POINTER(C.c_float)) for n in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")]
                + [("ln_eps", C.c_float), ("qmin", C.c_int), ("qmax", C.c_int)])


class _LayerDebug(C.Structure):
    _fields_ = [("c0", C.POINTER(C.c_int8)), ("qkv", C.POINTER(C.c_float)),
                ("ctx", C.POINTER(C.c_float)), ("c1", C.POINTER(C.c_int8)),
                ("u", C.POINTER(C.c_float)), ("h1", C.POINTER(C.c_float)),
                ("c2", C.POINTER(C.c_int8)), ("c3", C.POINTER(C.c_int8)),
                ("d", C.POINTER(C.c_float)), ("g_pre", C.POINTER(C.c_float))]


class _LayerParamsFloat(C.Structure):
    _fields_ = ([(n, C.c_int64) for n in ("batch", "seq", "hidden", "heads", "ffn")]
                + [(n, C.POINTER(C.c_float)) for n in ("w_qkv", "w_ao", "w_up", "w_down",
                                                        "b_qkv", "b_ao", "b_up", "b_down",
                                                        "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")]
                + [("ln_eps", C.c_float)])


def bert_layer_int4(layer: dict, h_in, act_dtype=F16, c0=None, debug=True, qmin=QMIN, qmax=QMAX):
    """One W4A4 post-LN BERT layer.

    ``layer`` holds: batch, seq, hidden, heads, ffn, ln_eps, and for each linear
    name in (qkv, ao, up, down): ``w_<name>`` int8 codes [N,K], ``sw_<name>`` [N],
    ``b_<name>`` [N], ``sx_<name>`` float; plus ln1_gamma/ln1_beta/ln2_gamma/ln2_beta.
    Returns (h_out float32 *before* narrowing, dict of intermediates).
    """
    B, S, H, heads, F = (int(layer[k]) for k in ("batch", "seq", "hidden", "heads", "ffn"))
    M = B * S
    keep = {}
    p = _LayerParams()
    p.batch, p.seq, p.hidden, p.heads, p.ffn = B, S, H, heads, F
    for nm in ("qkv", "ao", "up", "down"):
        keep["w_" + nm] = _i8(layer["w_" + nm])
        keep["sw_" + nm] = _f32(layer["sw_" + nm])
        keep["b_" + nm] = _f32(layer["b_" + nm])
        setattr(p, "w_" + nm, _p(keep["w_" + nm], C.c_int8))
        setattr(p, "sw_" + nm, _p(keep["sw_" + nm], C.c_float))
        setattr(p, "b_" + nm, _p(keep["b_" + nm], C.c_float))
        setattr(p, "sx_" + nm, float(layer["sx_" + nm]))
    for nm in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta"):
        keep[nm] = _f32(layer[nm])
        setattr(p, nm, _p(keep[nm], C.c_float))
    p.ln_eps = float(layer["ln_eps"])
    p.qmin, p.qmax = int(qmin), int(qmax)
    h_in = _f32(h_in).reshape(M, H)
    c0 = _i8(c0)
    h_out = np.empty((M, H), np.float32)
    inter = {}
    dbg = _LayerDebug()
    if debug:
        shapes = {"c0": ((M, H), np.int8), "qkv": ((M, 3 * H), np.float32), "ctx": ((M, H), np.float32),
                  "c1": ((M, H), np.int8), "u": ((M, H), np.float32), "h1": ((M, H), np.float32),
                  "c2": ((M, H), np.int8), "c3": ((M, F), np.int8), "d": ((M, H), np.float32),
                  "g_pre": ((M, F), np.float32)}
        for k, (shp, dt) in shapes.items():
            inter[k] = np.empty(shp, dt)
            setattr(dbg, k, _p(inter[k], C.c_int8 if dt == np.int8 else C.c_float))
    _check(lib().mkq_ref_bert_layer_int4(C.byref(p), _p(h_in, C.c_float), _p(c0, C.c_int8),
                                         int(act_dtype), _p(h_out, C.c_float),
                                         C.byref(dbg) if debug else None), "bert_layer_int4")
    return h_out, inter


def bert_layer_float(layer: dict, h_in, act_dtype=F16):
    """The same layer without quantizers (``w_<name>`` are float arrays [N,K])."""
    B, S, H, heads, F = (int(layer[k]) for k in ("batch", "seq", "hidden", "heads", "ffn"))
    M = B * S
    keep = {}
    p = _LayerParamsFloat()
    p.batch, p.seq, p.hidden, p.heads, p.ffn = B, S, H, heads, F
    for nm in ("w_qkv", "w_ao", "w_up", "w_down", "b_qkv", "b_ao", "b_up", "b_down",
               "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta"):
        keep[nm] = _f32(layer[nm])
        setattr(p, nm, _p(keep[nm], C.c_float))
    p.ln_eps = float(layer["ln_eps"])
    h_in = _f32(h_in).reshape(M, H)
    h_out = np.empty((M, H), np.float32)
    _check(lib().mkq_ref_bert_layer_float(C.byref(p), _p(h_in, C.c_float), int(act_dtype),
                                          _p(h_out, C.c_float)), "bert_layer_float")
    return h_out


def scale_gradients(x, s, qmin=QMIN, qmax=QMAX):
    """(STE-based, MSE-based) scale gradients of section 4.1 for one tensor."""
    x = _f32(x).ravel()
    g1, g2 = C.c_double(), C.c_double()
    _check(lib().mkq_ref_scale_gradients(_p(x, C.c_float), C.c_int64(x.size), C.c_float(s), qmin,
                                         qmax, C.byref(g1), C.byref(g2)), "scale_gradients")
    return g1.value, g2.value
