"""Seeded synthetic inputs for the quantized-linear / BERT-layer workloads.

Shared by the CPU oracle's tests and the GPU path's tests and benchmark.  This
module only draws numbers: it contains none of the method's arithmetic (no
quantizer, no scale calibration, no matmul).  Scales that a workload needs are
either produced by whichever side consumes them or, where the workload calls for
a *learned* step size, given here as a plain constant.

Every generator uses ``numpy.random.default_rng(seed)`` and draws in a fixed
order (activations, weights, bias, then extras), in float32.
"""
from __future__ import annotations

import numpy as np

# Step size standing in for a learned per-tensor activation step on roughly
# unit-variance data: the mean-square-optimal step of a 16-level uniform
# quantizer for a unit Gaussian is about 0.335; outliers then clip.
LEARNED_STEP_UNIT_GAUSSIAN = 0.34

BERT_BASE = dict(hidden=768, heads=12, ffn=3072)
BERT_LARGE = dict(hidden=1024, heads=16, ffn=4096)


def layer_gemm_shapes(hidden: int, ffn: int):
    """(name, K, N) of the four GEMMs of one encoder layer (QKV fused)."""
    return [("qkv", hidden, 3 * hidden), ("ao", hidden, hidden),
            ("up", hidden, ffn), ("down", ffn, hidden)]


def gaussian_linear(M: int, K: int, N: int, seed: int, w_std: float = 0.02, b_std: float = 0.01):
    """Activations ~N(0,1), weights ~N(0,w_std), bias ~N(0,b_std)."""
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K), dtype=np.float32)
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(w_std)
    b = rng.standard_normal(N, dtype=np.float32) * np.float32(b_std)
    return X, W, b


def outlier_activations(rng, M: int, K: int, frac: float, kind: str):
    """~N(0,1) activations with a fraction of outliers.

    kind "x8": the chosen entries are multiplied by 8.
    kind "student": the chosen entries are replaced by 8 * Student-t(nu=2) draws.
    """
    X = rng.standard_normal((M, K), dtype=np.float32)
    mask = rng.random((M, K), dtype=np.float32) < np.float32(frac)
    if kind == "x8":
        X = np.where(mask, X * np.float32(8.0), X)
    elif kind == "student":
        t = rng.standard_t(2.0, size=(M, K)).astype(np.float32) * np.float32(8.0)
        X = np.where(mask, t, X)
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(X, dtype=np.float32)


def outlier_linear(M: int, K: int, N: int, seed: int, frac: float = 0.01, kind: str = "x8",
                   w_std: float = 0.02, b_std: float = 0.01):
    rng = np.random.default_rng(seed)
    X = outlier_activations(rng, M, K, frac, kind)
    W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(w_std)
    b = rng.standard_normal(N, dtype=np.float32) * np.float32(b_std)
    return X, W, b


def uniform_codes_linear(M: int, K: int, N: int, seed: int):
    """Operands drawn directly as signed 4-bit codes, uniform on [-8, 7];
    per-channel scales ~U(0.001, 0.05); one activation step from the same law."""
    rng = np.random.default_rng(seed)
    A = rng.integers(-8, 8, size=(M, K), dtype=np.int8)
    Wc = rng.integers(-8, 8, size=(N, K), dtype=np.int8)
    s_w = rng.uniform(0.001, 0.05, size=N).astype(np.float32)
    s_x = float(np.float32(rng.uniform(0.001, 0.05)))
    return A, Wc, s_w, s_x


def bert_layer_weights(hidden: int, heads: int, ffn: int, seed: int, w_std: float = 0.02,
                       b_std: float = 0.01):
    """Random-init float parameters of one post-LN encoder layer.
    LayerNorm gamma = 1, beta = 0 (fresh initialisation)."""
    rng = np.random.default_rng(seed)
    p = {"hidden": hidden, "heads": heads, "ffn": ffn, "ln_eps": 1e-12}
    for name, K, N in layer_gemm_shapes(hidden, ffn):
        p["W_" + name] = rng.standard_normal((N, K), dtype=np.float32) * np.float32(w_std)
        p["b_" + name] = rng.standard_normal(N, dtype=np.float32) * np.float32(b_std)
    for ln in ("ln1", "ln2"):
        p[ln + "_gamma"] = np.ones(hidden, np.float32)
        p[ln + "_beta"] = np.zeros(hidden, np.float32)
    return p


def hidden_states(batch: int, seq: int, hidden: int, seed: int):
    """Embedding-output stand-in h^0 ~ N(0,1), shape [batch*seq, hidden]."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((batch * seq, hidden), dtype=np.float32)


# The benchmark configurations, by index.
CONFIGS = [
    dict(name="single_linear", M=128, shapes=[("lin", 768, 768)], seed=0),
    dict(name="bert_base_layer_gemms", M=1024, shapes=layer_gemm_shapes(768, 3072), seed=1,
         outlier_frac=0.01, outlier_kind="x8"),
    dict(name="bert_base_encoder", batch=32, seq=128, layers=12, seed=2, **BERT_BASE),
    dict(name="bert_large_layer_gemms", M=8192, shapes=layer_gemm_shapes(1024, 4096), seed=3,
         outlier_frac=0.005, outlier_kind="student"),
    dict(name="large_m_sweep", Ms=[16384, 32768, 65536],
         KN=[(1024, 4096), (4096, 1024), (768, 3072)], seed=4),
]


def ragged_lengths(total: int, batch: int, max_len: int, seed: int):
    """Seeded sequence lengths in [1, max_len] that add up to `total` (a padding-free batch with
    `total` valid tokens, as in the paper's Table 2)."""
    rng = np.random.default_rng(seed)
    lens = np.full(batch, total // batch, np.int64)
    lens[: total - lens.sum()] += 1
    for _ in range(4 * batch):  # move tokens between random pairs, keeping the bounds
        i, j = rng.integers(0, batch, 2)
        d = int(rng.integers(0, 20))
        if lens[i] - d >= 1 and lens[j] + d <= max_len:
            lens[i] -= d
            lens[j] += d
    assert lens.sum() == total and lens.min() >= 1 and lens.max() <= max_len
    return lens


# Table 2 of the paper (section 5.4): batch size and valid tokens of one BERT-base layer, with the
# paper's own latencies in microseconds on an NVIDIA T4 (float32, int8, int4) -- context only.
TABLE2_ROWS = [(16, 440, 1380.0, 213.1, 160.5), (16, 537, 1845.0, 245.7, 179.3), (16, 681, 2690.0, 260.9, 196.5),
               (64, 1691, 6398.0, 567.4, 428.8), (64, 2011, 7185.0, 628.4, 490.1), (64, 2298, 7897.0, 669.9, 533.4)]
