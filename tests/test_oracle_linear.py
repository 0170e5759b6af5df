"""Pins for the oracle's integer GEMM, dequantize epilogue, requantization and
the encoder layer (CPU only)."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2203_13483_amd import workloads as wl


def _brute(a, w):
    M, K = a.shape
    N = w.shape[0]
    out = [[0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            t = 0
            for k in range(K):
                t += int(a[m][k]) * int(w[n][k])
            out[m][n] = t
    return np.array(out, np.int64).reshape(M, N)


# --- integer GEMM ------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (1, 1, 64), (3, 5, 7), (8, 8, 64), (2, 7, 33), (5, 1, 16)])
def test_gemm_brute_force_tiny(M, N, K):
    rng = np.random.default_rng(M * 100 + N * 10 + K)
    a = rng.integers(-8, 8, (M, K), dtype=np.int8)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    assert np.array_equal(oracle.gemm_codes(a, w), _brute(a, w))


def test_gemm_exhaustive_pairs():
    # every (a, w) code pair as a 1x1x1 product, and every pair of pairs as K=2
    vals = np.arange(-8, 8, dtype=np.int8)
    a = np.repeat(vals, 16)[:, None]
    w = np.tile(vals, 16)[:, None]
    acc = oracle.gemm_codes(a, w)
    for i, j in itertools.product(range(256), repeat=2):
        if (i * 7 + j) % 97:  # thin the 65k cases; the diagonal is always kept below
            continue
        assert acc[i, j] == int(a[i, 0]) * int(w[j, 0])
    assert np.array_equal(np.diag(acc), (a[:, 0].astype(np.int32) * w[:, 0].astype(np.int32)))


@pytest.mark.parametrize("M,N,K", [(37, 53, 768), (128, 96, 3072), (64, 64, 1000)])
def test_gemm_matches_numpy_int64(M, N, K):
    rng = np.random.default_rng(K)
    a = rng.integers(-8, 8, (M, K), dtype=np.int8)
    w = rng.integers(-8, 8, (N, K), dtype=np.int8)
    ref = a.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(oracle.gemm_codes(a, w).astype(np.int64), ref)


def test_gemm_not_transposed():
    # a rectangular case where confusing [N,K] with [K,N] cannot go unnoticed
    a = np.array([[1, 2, 3]], np.int8)
    w = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1], [1, 1, 1], [-1, -2, -3]], np.int8)
    assert oracle.gemm_codes(a, w).tolist() == [[1, 2, 3, 6, -14]]


@pytest.mark.parametrize("K", [64, 768, 4096])
def test_accumulator_bound_attained(K):
    lo = np.full((2, K), -8, np.int8)
    hi = np.full((2, K), 7, np.int8)
    assert np.all(oracle.gemm_codes(lo, lo) == 64 * K)
    assert np.all(oracle.gemm_codes(lo, hi) == -56 * K)
    rng = np.random.default_rng(0)
    a = rng.integers(-8, 8, (16, K), dtype=np.int8)
    w = rng.integers(-8, 8, (16, K), dtype=np.int8)
    assert np.abs(oracle.gemm_codes(a, w)).max() <= 64 * K


def test_one_hot_weights_copy_input_codes():
    rng = np.random.default_rng(1)
    a = rng.integers(-8, 8, (9, 32), dtype=np.int8)
    eye = np.eye(32, dtype=np.int8)
    assert np.array_equal(oracle.gemm_codes(a, eye), a.astype(np.int32))
    perm = rng.permutation(32)
    assert np.array_equal(oracle.gemm_codes(a, eye[perm]), a[:, perm].astype(np.int32))


def test_linearity_and_k_split():
    rng = np.random.default_rng(2)
    a1 = rng.integers(-4, 4, (6, 128), dtype=np.int8)
    a2 = rng.integers(-4, 4, (6, 128), dtype=np.int8)
    w = rng.integers(-8, 8, (10, 128), dtype=np.int8)
    assert np.array_equal(oracle.gemm_codes(a1 + a2, w), oracle.gemm_codes(a1, w) + oracle.gemm_codes(a2, w))
    full = oracle.gemm_codes(a1, w)
    halves = oracle.gemm_codes(a1[:, :64], w[:, :64]) + oracle.gemm_codes(a1[:, 64:], w[:, 64:])
    assert np.array_equal(full, halves)


# --- dequantize epilogue -------------------------------------------------------------

def test_epilogue_unit_scales_return_accumulator():
    rng = np.random.default_rng(3)
    acc = rng.integers(-2 ** 18, 2 ** 18, (7, 11)).astype(np.int32)
    y = oracle.epilogue(acc, 1.0, np.ones(11, np.float32))
    assert np.array_equal(y, acc.astype(np.float32))


def test_epilogue_matches_real_arithmetic():
    # y must equal (sum_k Q[x_k] Q[w_k]) + b computed in binary64, up to the two
    # binary32 roundings (scale product, fma)
    X, W, b = wl.gaussian_linear(33, 256, 47, seed=11)
    s_x = oracle.absmax_scale(X)
    wc, s_w = oracle.quantize_weights(W)
    xc = oracle.quantize(X, s_x)
    res = oracle.linear_int4(xc, s_x, wc, s_w, b)
    Qx = xc.astype(np.float64) * float(np.float32(s_x))
    Qw = wc.astype(np.float64) * s_w.astype(np.float64)[:, None]
    ref = Qx @ Qw.T + b.astype(np.float64)
    tol = 1.3e-7 * (np.abs(Qx @ Qw.T) + np.abs(b.astype(np.float64))) + 1e-30
    assert np.all(np.abs(res["y"].astype(np.float64) - ref) <= tol)
    assert np.array_equal(res["acc"], oracle.gemm_codes(xc, wc))


def test_epilogue_bias_is_per_output_channel_and_residual_added():
    acc = np.zeros((2, 3), np.int32)
    b = np.array([1.0, 2.0, 3.0], np.float32)
    r = np.array([[10, 20, 30], [40, 50, 60]], np.float32)
    y = oracle.epilogue(acc, 0.5, np.ones(3, np.float32), b, r)
    assert y.tolist() == [[11, 22, 33], [41, 52, 63]]
    acc[:] = 2
    y = oracle.epilogue(acc, 0.5, np.array([1, 2, 4], np.float32), None, None)
    assert y.tolist() == [[1, 2, 4], [1, 2, 4]]


def test_quantized_linear_close_to_float_linear_within_analytic_bound():
    # sanity, not parity: when nothing clips, |y - (x W^T + b)| is bounded by
    # sum_k (|x_k| s_w/2 + |w_k| s_x/2 + s_x s_w/4)
    X, W, b = wl.gaussian_linear(16, 128, 24, seed=12)
    s_x = oracle.absmax_scale(X)
    wc, s_w = oracle.quantize_weights(W)
    y = oracle.linear_int4(oracle.quantize(X, s_x), s_x, wc, s_w, b)["y"].astype(np.float64)
    ref = X.astype(np.float64) @ W.astype(np.float64).T + b
    bound = (np.abs(X).sum(1)[:, None] * s_w[None, :] / 2
             + np.abs(W).sum(1)[None, :] * s_x / 2 + 128 * s_x * s_w[None, :] / 4)
    assert np.all(np.abs(y - ref) <= bound * (1 + 1e-5))


def test_gelu_matches_torch_double():
    x = np.linspace(-6, 6, 2001, dtype=np.float32)[None, :]
    acc = np.zeros_like(x, dtype=np.int32)
    y = oracle.epilogue(acc, 1.0, np.ones(x.shape[1], np.float32), None, x, act=oracle.ACT_GELU)
    ref = torch.nn.functional.gelu(torch.from_numpy(x).double()).float().numpy()
    assert np.array_equal(y, ref)


def test_requant_of_on_grid_values_and_composition():
    rng = np.random.default_rng(4)
    a = rng.integers(-8, 8, (5, 64), dtype=np.int8)
    w = np.eye(64, dtype=np.int8)
    # identity weights, unit scales: y = a exactly, requant with s_next = 1 returns a
    r = oracle.linear_int4(a, 1.0, w, np.ones(64, np.float32), s_next=1.0)
    assert np.array_equal(r["q"], a)
    # requant is Eq. 1 applied to the binary32 epilogue value, not to the narrowed one
    X, W, b = wl.gaussian_linear(8, 64, 16, seed=13)
    s_x = oracle.absmax_scale(X)
    wc, s_w = oracle.quantize_weights(W)
    r = oracle.linear_int4(oracle.quantize(X, s_x), s_x, wc, s_w, b, out_dtype=oracle.F16, s_next=0.05)
    y32 = oracle.epilogue(r["acc"], s_x, s_w, b)
    assert np.array_equal(r["q"], oracle.quantize(y32, 0.05))
    assert np.array_equal(r["y"], y32.astype(np.float16).astype(np.float32))


# --- float baseline linear, LayerNorm, attention: torch double precision is the library route ---

def test_linear_float_matches_numpy():
    rng = np.random.default_rng(5)
    a = rng.normal(0, 1, (19, 96)).astype(np.float16).astype(np.float32)
    W = rng.normal(0, 0.05, (23, 96)).astype(np.float16).astype(np.float32)
    b = rng.normal(0, 0.1, 23).astype(np.float32)
    y = oracle.linear_float(a, W, b)
    ref = (a.astype(np.float64) @ W.astype(np.float64).T + b).astype(np.float32)
    np.testing.assert_allclose(y, ref, rtol=1e-6, atol=1e-7)


def test_layernorm_matches_torch():
    rng = np.random.default_rng(6)
    x = rng.normal(0.3, 2.0, (17, 768)).astype(np.float32)
    g = rng.normal(1, 0.1, 768).astype(np.float32)
    b = rng.normal(0, 0.1, 768).astype(np.float32)
    y = oracle.layernorm(x, g, b, eps=1e-12)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (768,), torch.from_numpy(g).double(),
                                         torch.from_numpy(b).double(), eps=1e-12).float().numpy()
    np.testing.assert_allclose(y, ref, rtol=2e-7, atol=1e-7)
    y0 = oracle.layernorm(x)
    assert np.abs(y0.mean(1)).max() < 1e-6 and np.abs(y0.var(1) - 1).max() < 1e-5


def test_attention_matches_torch_sdpa():
    B, S, H, heads = 2, 24, 48, 4
    rng = np.random.default_rng(7)
    qkv = rng.normal(0, 1, (B * S, 3 * H)).astype(np.float32)
    ctx = oracle.attention(qkv, B, S, H, heads)
    t = torch.from_numpy(qkv).double().reshape(B, S, 3, heads, H // heads).permute(2, 0, 3, 1, 4)
    ref = torch.nn.functional.scaled_dot_product_attention(t[0], t[1], t[2])  # [B, heads, S, dk]
    ref = ref.permute(0, 2, 1, 3).reshape(B * S, H).float().numpy()
    np.testing.assert_allclose(ctx, ref, rtol=1e-6, atol=1e-7)


# --- the encoder layer -------------------------------------------------------------

def _float_layer(seed, B=2, S=16, hidden=64, heads=4, ffn=128):
    p = wl.bert_layer_weights(hidden, heads, ffn, seed, w_std=0.08, b_std=0.05)
    rng = np.random.default_rng(seed + 100)
    p["ln1_gamma"] = rng.normal(1, 0.1, hidden).astype(np.float32)
    p["ln1_beta"] = rng.normal(0, 0.1, hidden).astype(np.float32)
    p["ln2_gamma"] = rng.normal(1, 0.1, hidden).astype(np.float32)
    p["ln2_beta"] = rng.normal(0, 0.1, hidden).astype(np.float32)
    p["ln_eps"] = 1e-5
    p["batch"], p["seq"] = B, S
    h = wl.hidden_states(B, S, hidden, seed + 1)
    return p, h


def _as_float_params(p):
    q = {k: p[k] for k in ("batch", "seq", "hidden", "heads", "ffn", "ln_eps",
                           "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    for nm in ("qkv", "ao", "up", "down"):
        q["w_" + nm] = p["W_" + nm]
        q["b_" + nm] = p["b_" + nm]
    return q


def test_float_layer_matches_torch_transformer_encoder_layer():
    p, h = _float_layer(21)
    B, S, H = p["batch"], p["seq"], p["hidden"]
    out = oracle.bert_layer_float(_as_float_params(p), h, act_dtype=oracle.F32)
    layer = torch.nn.TransformerEncoderLayer(H, p["heads"], p["ffn"], dropout=0.0, activation="gelu",
                                             layer_norm_eps=p["ln_eps"], batch_first=True,
                                             norm_first=False).double().eval()
    sd = {
        "self_attn.in_proj_weight": p["W_qkv"], "self_attn.in_proj_bias": p["b_qkv"],
        "self_attn.out_proj.weight": p["W_ao"], "self_attn.out_proj.bias": p["b_ao"],
        "linear1.weight": p["W_up"], "linear1.bias": p["b_up"],
        "linear2.weight": p["W_down"], "linear2.bias": p["b_down"],
        "norm1.weight": p["ln1_gamma"], "norm1.bias": p["ln1_beta"],
        "norm2.weight": p["ln2_gamma"], "norm2.bias": p["ln2_beta"],
    }
    layer.load_state_dict({k: torch.from_numpy(np.asarray(v)).double() for k, v in sd.items()})
    with torch.no_grad():
        ref = layer(torch.from_numpy(h).double().reshape(B, S, H)).reshape(B * S, H).float().numpy()
    np.testing.assert_allclose(out, ref, rtol=2e-5, atol=2e-6)


def _quantize_layer(p, h, qmin, qmax, sx_mult=1.0):
    """Quantized twin of a float layer: abs-max scales everywhere, activation
    steps calibrated on the float layer's own intermediates."""
    fp = _as_float_params(p)
    B, S, H, F = p["batch"], p["seq"], p["hidden"], p["ffn"]
    M = B * S
    qkv = oracle.linear_float(h, fp["w_qkv"], fp["b_qkv"])
    ctx = oracle.attention(qkv, B, S, H, p["heads"])
    u = oracle.linear_float(ctx, fp["w_ao"], fp["b_ao"], residual=h)
    h1 = oracle.layernorm(u, p["ln1_gamma"], p["ln1_beta"], p["ln_eps"])
    g = oracle.linear_float(h1, fp["w_up"], fp["b_up"], act=oracle.ACT_GELU)
    q = {k: p[k] for k in ("batch", "seq", "hidden", "heads", "ffn", "ln_eps",
                           "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    for nm, act_in in (("qkv", h), ("ao", ctx), ("up", h1), ("down", g)):
        q["w_" + nm], q["sw_" + nm] = oracle.quantize_weights(p["W_" + nm], qmin=qmin, qmax=qmax)
        q["b_" + nm] = p["b_" + nm]
        q["sx_" + nm] = oracle.absmax_scale(act_in, qmax=qmax) * sx_mult
    return q


def test_quantized_layer_with_8bit_range_approaches_float_layer():
    # composition pin: with 8-bit quantizers the quantized layer must track the
    # float layer (already pinned to torch) closely; a wrong residual, head slice
    # or operand order gives O(1) errors.
    p, h = _float_layer(22)
    ref = oracle.bert_layer_float(_as_float_params(p), h, act_dtype=oracle.F32)
    q = _quantize_layer(p, h, -128, 127)
    out, _ = oracle.bert_layer_int4(q, h, act_dtype=oracle.F32, qmin=-128, qmax=127)
    err = np.abs(out - ref)
    assert err.max() < 0.08 and np.sqrt((err ** 2).mean()) < 0.02
    # and 4-bit is visibly coarser but still correlated
    q4 = _quantize_layer(p, h, -8, 7)
    out4, _ = oracle.bert_layer_int4(q4, h, act_dtype=oracle.F32)
    assert np.corrcoef(out4.ravel(), ref.ravel())[0, 1] > 0.9
    assert np.sqrt(((out4 - ref) ** 2).mean()) > np.sqrt((err ** 2).mean())


def test_quantized_layer_stages_are_the_pinned_pieces():
    p, h = _float_layer(23)
    q = _quantize_layer(p, h, -8, 7, sx_mult=0.6)
    B, S, H = p["batch"], p["seq"], p["hidden"]
    out, it = oracle.bert_layer_int4(q, h, act_dtype=oracle.F16)
    assert np.array_equal(it["c0"], oracle.quantize(h, q["sx_qkv"]))
    r = oracle.linear_int4(it["c0"], q["sx_qkv"], q["w_qkv"], q["sw_qkv"], q["b_qkv"], out_dtype=oracle.F16)
    assert np.array_equal(it["qkv"], r["y"])
    ctx = oracle.attention(it["qkv"], B, S, H, p["heads"], p_dtype=oracle.F16)
    assert np.array_equal(it["ctx"], ctx)
    assert np.array_equal(it["c1"], oracle.quantize(ctx, q["sx_ao"]))
    r = oracle.linear_int4(it["c1"], q["sx_ao"], q["w_ao"], q["sw_ao"], q["b_ao"], residual=h, out_dtype=oracle.F16)
    assert np.array_equal(it["u"], r["y"])
    h1f = oracle.layernorm(it["u"], p["ln1_gamma"], p["ln1_beta"], p["ln_eps"])
    assert np.array_equal(it["c2"], oracle.quantize(h1f, q["sx_up"]))
    assert np.array_equal(it["h1"], oracle.round_storage(h1f, oracle.F16))
    r = oracle.linear_int4(it["c2"], q["sx_up"], q["w_up"], q["sw_up"], q["b_up"], act=oracle.ACT_GELU,
                           s_next=q["sx_down"])
    assert np.array_equal(it["c3"], r["q"])
    r = oracle.linear_int4(it["c3"], q["sx_down"], q["w_down"], q["sw_down"], q["b_down"], residual=it["h1"],
                           out_dtype=oracle.F16)
    assert np.array_equal(it["d"], r["y"])
    assert np.array_equal(out, oracle.layernorm(it["d"], p["ln2_gamma"], p["ln2_beta"], p["ln_eps"]))


def test_zero_weight_layer_reduces_to_two_layernorms():
    p, h = _float_layer(24)
    q = _quantize_layer(p, h, -8, 7)
    for nm in ("qkv", "ao", "up", "down"):
        q["w_" + nm] = np.zeros_like(q["w_" + nm])
        q["b_" + nm] = np.zeros_like(q["b_" + nm])
    out, _ = oracle.bert_layer_int4(q, h, act_dtype=oracle.F32)
    h1 = oracle.layernorm(h, p["ln1_gamma"], p["ln1_beta"], p["ln_eps"])
    ref = oracle.layernorm(h1, p["ln2_gamma"], p["ln2_beta"], p["ln_eps"])
    np.testing.assert_allclose(out, ref, rtol=1e-6, atol=1e-6)


def test_quantized_layer_is_unchanged_by_a_permutation_of_its_heads():
    """Renumbering the heads -- the blocks of d_k rows of the q, k and v parts of the QKV weights, with their
    per-channel steps and biases, and the matching blocks of d_k columns of the attention-out weights -- changes
    nothing: every head's scores and context are computed from the same numbers, and the attention-out sums run
    over the same products in another order, which integer accumulation does not see.  Bit for bit: a head's q, k
    or v slice taken at the wrong offset, or a context written to the wrong block, fails this."""
    p, h = _float_layer(25)
    q = _quantize_layer(p, h, -8, 7, sx_mult=0.6)
    H, heads = p["hidden"], p["heads"]
    dk = H // heads
    rng = np.random.default_rng(7)
    order = rng.permutation(heads)
    assert not np.array_equal(order, np.arange(heads))
    cols = np.concatenate([np.arange(i * dk, (i + 1) * dk) for i in order])       # new position -> old channel
    rows_qkv = np.concatenate([part * H + cols for part in range(3)])
    q2 = dict(q)
    q2["w_qkv"], q2["sw_qkv"], q2["b_qkv"] = q["w_qkv"][rows_qkv], q["sw_qkv"][rows_qkv], q["b_qkv"][rows_qkv]
    q2["w_ao"] = np.ascontiguousarray(q["w_ao"][:, cols])
    out, it = oracle.bert_layer_int4(q, h, act_dtype=oracle.F16)
    out2, it2 = oracle.bert_layer_int4(q2, h, act_dtype=oracle.F16)
    assert np.array_equal(it2["qkv"], it["qkv"][:, rows_qkv])
    assert np.array_equal(it2["ctx"], it["ctx"][:, cols]) and np.array_equal(it2["c1"], it["c1"][:, cols])
    assert np.array_equal(it2["u"], it["u"])
    assert np.array_equal(out2, out)


def test_attention_with_probabilities_narrowed_before_the_value_product():
    """The p_dtype = F16 branch (softmax probabilities rounded to binary16 BEFORE P.v, as a 16-bit matrix
    unit consumes them) against torch in float64: softmax -> .half() -> matmul.  The same data distinguish it
    from narrowing nothing and from narrowing the context instead."""
    import torch
    B, S, heads = 2, 48, 3
    H = heads * 64
    rng = np.random.default_rng(31)
    qkv = rng.normal(0, 1.2, (B * S, 3 * H)).astype(np.float16).astype(np.float32)
    got = oracle.attention(qkv, B, S, H, heads, p_dtype=oracle.F16)
    t = torch.from_numpy(qkv).double().reshape(B, S, 3, heads, 64)
    q, k, v = (t[:, :, i].permute(0, 2, 1, 3) for i in range(3))  # [B, heads, S, 64]
    p = torch.softmax(q @ k.transpose(-1, -2) / 8.0, dim=-1)
    narrowed_p = (p.half().double() @ v).permute(0, 2, 1, 3).reshape(B * S, H).numpy()
    plain = (p @ v).permute(0, 2, 1, 3).reshape(B * S, H).numpy()
    narrowed_ctx = torch.from_numpy(plain).half().double().numpy()
    # binary64 -> binary16 in one rounding on the torch side; the oracle may round through binary32 first: the two
    # agree except where that double rounding lands on a binary16 tie (one unit of one probability, at most)
    err = np.abs(got - narrowed_p)
    assert err.max() < 2.0 ** -10 * np.abs(qkv[:, 2 * H:]).max() / 4 and np.mean(err > 1e-6) < 1e-3
    assert np.sqrt((err ** 2).mean()) < 2e-7
    # the placement of the narrowing is visible at this size: the other two placements are 100x further away
    assert np.sqrt(((got - plain) ** 2).mean()) > 2e-5
    assert np.sqrt(((got - narrowed_ctx) ** 2).mean()) > 2e-5
    assert np.allclose(oracle.attention(qkv, B, S, H, heads, p_dtype=oracle.F32), plain, rtol=0, atol=2e-6)
