"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(automatic tile choice): the whole output where the oracle finishes in seconds,
otherwise sampled token rows (every tile-edge row of the first and last tiles plus random
ones), each compared with the oracle over all channels.  A linear's output rows depend on
one input row each, so the oracle is run on just the sampled rows."""
import numpy as np
import pytest

import oracle
from paper_2203_13483_amd import workloads as wl
from helpers import RTOL, assert_codes_match_with_tie_band, assert_float_close, to_dev, to_np
from layer_checks import LayerBuffers, attention_code_band, check_layer_stagewise, codes_match

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m


def _sample_rows(M, rng, n_random=48, every_block=False):
    edge = [0, 1, 31, 32, 63, 64, 127, 128, 255, 256, 257, 511, 512]
    edge += [M - 1 - e for e in edge]
    rows = {r for r in edge if 0 <= r < M}
    rows.update(int(r) for r in rng.integers(0, M, n_random))
    if every_block:
        # one row, at a random place, in every block of 32 tokens: every tile of every workgroup and every
        # 32-row accumulator block of every wave is looked at
        base = np.arange(0, M, 32)
        rows.update(int(r) for r in np.minimum(base + rng.integers(0, 32, base.size), M - 1))
    return np.array(sorted(rows))


def _pack_rows_on_device(mkq, codes, chunk=8192):
    """int8 codes [R, K] -> packed device tensor, in chunks (the int8 copy is 2x the packed size)."""
    import torch
    R, K = codes.shape
    out = torch.empty((R, K // 2), dtype=torch.uint8, device="cuda")
    for r0 in range(0, R, chunk):
        out[r0:r0 + chunk] = mkq.mkq_pack_codes_int4(to_dev(codes[r0:r0 + chunk]))
    return out


@pytest.mark.parametrize("M", [16384, 32768, 65536])
@pytest.mark.parametrize("K,N", [(1024, 4096), (4096, 1024), (768, 3072)])
def test_large_m_sweep_bf16_sampled_rows(mkq, M, K, N):
    """The large-M sweep, all nine points: uniform codes, per-channel scales U(0.001, 0.05), bf16 out; one
    sampled row in every block of 32 tokens (all channels of it), tile-edge rows and random rows."""
    import torch
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed=4)
    a_d = _pack_rows_on_device(mkq, A)
    w_d = mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1)
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), None, N, K, mkq.MKQ_BF16, out=out)
    torch.cuda.synchronize()
    rows = _sample_rows(M, np.random.default_rng(M + K), every_block=True)
    got = to_np(out[torch.from_numpy(rows).cuda()]).astype(np.float32)
    ref = oracle.linear_int4(A[rows], s_x, Wc, s_w, None, out_dtype=oracle.BF16)
    assert np.array_equal(got, ref["y"])  # identical binary32 values, one RNE narrowing
    # every element was written (the buffer started as NaN)
    assert not torch.isnan(out).any()


def test_bert_large_layer_gemms_fused_requant(mkq):
    """The BERT-large layer GEMMs workload: M = 8192, hidden 1024, FFN 4096, heavy-tailed outliers; int4 in,
    int4 out through the fused re-quantization, GELU on FFN-up.  Sampled token rows."""
    import torch
    cfg = wl.CONFIGS[3]
    M = cfg["M"]
    rng = np.random.default_rng(cfg["seed"])
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    rows = _sample_rows(M, np.random.default_rng(99))
    for name, K, N in cfg["shapes"]:
        X = wl.outlier_activations(rng, M, K, cfg["outlier_frac"], cfg["outlier_kind"])
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
        b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
        gelu = name == "up"
        Wq, s_w = mkq.mkq_pack_weights_int4(to_dev(W))
        wc_ref, sw_ref = oracle.quantize_weights(W)
        assert np.array_equal(to_np(s_w), sw_ref)
        codes_d = mkq.mkq_quantize(to_dev(X), s_x)
        c_ref = oracle.quantize(X[rows], s_x)
        assert np.array_equal(oracle.unpack_nibbles(to_np(codes_d[torch.from_numpy(rows).cuda()]), K), c_ref)
        y32 = oracle.linear_int4(c_ref, s_x, wc_ref, sw_ref, b, act=oracle.ACT_GELU if gelu else oracle.ACT_NONE)["y"]
        s_next = float(np.float32(np.abs(y32).max() / 10))  # clips the largest outputs
        r = mkq.mkq_linear_int4(codes_d, s_x, Wq, s_w, to_dev(b), N, K, mkq.MKQ_I4, s_next=s_next,
                                act=mkq.MKQ_ACT_GELU if gelu else mkq.MKQ_ACT_NONE)
        torch.cuda.synchronize()
        got = oracle.unpack_nibbles(to_np(r["out"][torch.from_numpy(rows).cuda()]), N)
        ref = oracle.linear_int4(c_ref, s_x, wc_ref, sw_ref, b, act=oracle.ACT_GELU if gelu else oracle.ACT_NONE,
                                 s_next=s_next)
        if gelu:
            assert_codes_match_with_tie_band(got, ref["q"], ref["y"], s_next, what=name)
        else:
            assert np.array_equal(got, ref["q"]), name


def test_bert_base_layer_gemms_as_benchmarked(mkq):
    """The BERT-base layer GEMMs workload, exactly the benchmark's step: binary16 activations with 1 % x8
    outliers in, quantize + GEMM + dequantize, binary16 out; the whole output is compared."""
    import torch
    cfg = wl.CONFIGS[1]
    M = cfg["M"]
    rng = np.random.default_rng(cfg["seed"])
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    for name, K, N in cfg["shapes"]:
        X = wl.outlier_activations(rng, M, K, cfg["outlier_frac"], cfg["outlier_kind"]).astype(np.float16)
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
        b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
        Wq, s_w = mkq.mkq_pack_weights_int4(to_dev(W))
        r = mkq.mkq_linear_int4(to_dev(X), s_x, Wq, s_w, to_dev(b), N, K, mkq.MKQ_F16)
        torch.cuda.synchronize()
        wc, sw_ref = oracle.quantize_weights(W)
        codes = oracle.quantize(X.astype(np.float32), s_x)
        assert codes.min() == -8 and codes.max() == 7, "the learned step is meant to clip the outliers"
        ref = oracle.linear_int4(codes, s_x, wc, sw_ref, b, out_dtype=oracle.F16)
        got = to_np(r["out"]).astype(np.float32)
        assert_float_close(got, ref["y"], RTOL[1], name)
        assert np.array_equal(got, ref["y"]), name


def _bert_base_layer(mkq, seed, s_out_next=0.0):
    """Device tensors and oracle parameters of one BERT-base layer with the benchmark's activation steps."""
    H, heads, F = 768, 12, 3072
    p = wl.bert_layer_weights(H, heads, F, seed)
    packed, sx, q = {}, {}, {k: p[k] for k in ("hidden", "heads", "ffn", "ln_eps", "ln1_gamma", "ln1_beta",
                                                 "ln2_gamma", "ln2_beta")}
    steps = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
    for nm in ("qkv", "ao", "up", "down"):
        Wq, s_w = mkq.mkq_pack_weights_int4(to_dev(p["W_" + nm]))
        packed[nm] = (Wq, s_w, to_dev(p["b_" + nm]))
        sx[nm] = steps[nm]
        q["w_" + nm], q["sw_" + nm] = oracle.quantize_weights(p["W_" + nm])
        q["b_" + nm], q["sx_" + nm] = p["b_" + nm], steps[nm]
    ln = {k: to_dev(p[k]) for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    return p, packed, sx, ln, q


def test_encoder_layer_full_batch_sampled_sequences(mkq):
    """The full-encoder workload's shape: batch 32 x seq 128, BERT-base layer.  Sequences do not interact, so the
    oracle follows the layer on two of the 32 sequences: every stage against the GPU's own previous stage."""
    import torch
    B, S, H, heads, F = 32, 128, 768, 12, 3072
    p, packed, sx, ln, q = _bert_base_layer(mkq, 102)
    h = wl.hidden_states(B, S, H, 2).astype(np.float16)
    layer = mkq.BertLayerInt4(B, S, H, heads, F, packed, sx, ln, p["ln_eps"], 0.0)
    ws = torch.zeros(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
    out = to_np(layer(to_dev(h), ws)).astype(np.float32)
    torch.cuda.synchronize()
    buf = LayerBuffers(to_np(ws), layer.layout, B * S, H, F, 4)
    check_layer_stagewise(buf, q, h.astype(np.float32), out, [(0, S), (31 * S, S)], what="full batch")
    # and end to end against the oracle's own layer on those sequences: codes may flip near a rounding
    # boundary upstream, so closeness of the whole is asked on top of the stage-wise identity above
    seqs = [0, 31]
    sel = np.concatenate([np.arange(b * S, (b + 1) * S) for b in seqs])
    q["batch"], q["seq"] = len(seqs), S
    ref_out, _ = oracle.bert_layer_int4(q, h[sel].astype(np.float32), act_dtype=oracle.F16)
    err = out[sel] - ref_out
    assert np.sqrt((err ** 2).mean()) < 0.03 * np.sqrt((ref_out ** 2).mean())
    assert np.isfinite(out).all()
    # LayerNorm with gamma = 1, beta = 0: every output row has zero mean and unit variance
    assert np.abs(out.mean(axis=1)).max() < 2e-2 and np.abs(out.var(axis=1) - 1).max() < 5e-2


def test_attention_bert_large_512_tokens_full_batch(mkq):
    """The BERT-large workload's shape of the attention core: 16 sequences of 512 tokens, 16 heads of 64 (the shape
    bench.py times), context and codes of four of the sequences against the oracle."""
    B, S, heads, dk = 16, 512, 16, 64
    H = heads * dk
    rng = np.random.default_rng(77)
    qkv = rng.normal(0, 1.0, (B * S, 3 * H)).astype(np.float16)
    s_next = 0.05
    ctx, q = mkq.mkq_attention(to_dev(qkv), B, S, H, heads, s_next=s_next, want_q=True)
    got, codes = to_np(ctx).astype(np.float32), oracle.unpack_nibbles(to_np(q), H)
    assert np.isfinite(got).all()
    for b in (0, 5, 10, 15):
        rows = slice(b * S, (b + 1) * S)
        x = qkv[rows].astype(np.float32)
        ref = oracle.attention(x, 1, S, H, heads, p_dtype=oracle.F16)
        assert_float_close(got[rows], ref, RTOL[1], f"sequence {b}")
        codes_match(codes[rows], oracle.quantize(ref, s_next), ref, s_next,
                    attention_code_band(x, S, H, heads, s_next), f"context codes of sequence {b}")


def test_student_layer_full_batch_sampled_sequences(mkq):
    """The 4-layer student's layer (hidden 312, 12 heads of 26, FFN 1200: padded code rows) at 32 x 128 tokens,
    stage by stage on the first and the last sequence."""
    import torch
    B, S, H, heads, F = 32, 128, 312, 12, 1200
    p = wl.bert_layer_weights(H, heads, F, 103)
    steps = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
    packed, q = {}, {k: p[k] for k in ("hidden", "heads", "ffn", "ln_eps", "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    for nm in ("qkv", "ao", "up", "down"):
        Wq, s_w = mkq.mkq_pack_weights_int4_padded(to_dev(p["W_" + nm]))
        packed[nm] = (Wq, s_w, to_dev(p["b_" + nm]))
        q["w_" + nm], q["sw_" + nm] = oracle.quantize_weights(p["W_" + nm])
        q["b_" + nm], q["sx_" + nm] = p["b_" + nm], steps[nm]
    ln = {k: to_dev(p[k]) for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    h = wl.hidden_states(B, S, H, 3).astype(np.float16)
    layer = mkq.BertLayerInt4(B, S, H, heads, F, packed, steps, ln, p["ln_eps"], 0.0)
    ws = torch.full((layer.workspace_bytes(),), 0xA5, dtype=torch.uint8, device="cuda")
    out = to_np(layer(to_dev(h), ws)).astype(np.float32)
    torch.cuda.synchronize()
    buf = LayerBuffers(to_np(ws), layer.layout, B * S, H, F, 4)
    check_layer_stagewise(buf, q, h.astype(np.float32), out, [(0, S), (31 * S, S)], what="student layer")
    assert np.isfinite(out).all()
    assert np.abs(out.mean(axis=1)).max() < 2e-2 and np.abs(out.var(axis=1) - 1).max() < 5e-2


def test_twelve_layer_encoder_chain_teacher_forced(mkq):
    """The full-encoder workload: the 12-layer BERT-base encoder at batch 32 x seq 128 exactly as the benchmark
    chains it (every layer hands its binary16 output and the codes of it, under the next layer's step, to the
    next layer through q_out_next / q_in).  The oracle follows two of the 32 sequences layer by layer, each
    layer fed the GPU's previous output and codes: every stage of every layer is checked, and so is the
    hand-over between layers."""
    import torch
    B, S, H, heads, F, LAYERS = 32, 128, 768, 12, 3072, 12
    M = B * S
    h0 = wl.hidden_states(B, S, H, 2).astype(np.float16)
    s_next = wl.LEARNED_STEP_UNIT_GAUSSIAN
    layers = []
    for l in range(LAYERS):
        p, packed, sx, ln, q = _bert_base_layer(mkq, 100 + l)
        layers.append((mkq.BertLayerInt4(B, S, H, heads, F, packed, sx, ln, p["ln_eps"], s_next), q))
    ws = [torch.zeros(layers[0][0].workspace_bytes(), dtype=torch.uint8, device="cuda") for _ in range(LAYERS)]
    hs = [torch.empty((M, H), dtype=torch.float16, device="cuda") for _ in range(LAYERS)]
    qs = [torch.empty((M, H // 2), dtype=torch.uint8, device="cuda") for _ in range(LAYERS)]
    x, qin = to_dev(h0), None
    for l, (layer, _) in enumerate(layers):  # the whole chain is enqueued before anything is read back
        layer(x, ws[l], h_out=hs[l], q_in=qin, q_out_next=qs[l])
        x, qin = hs[l], qs[l]
    torch.cuda.synchronize()
    seqs = [(3 * S, S), (30 * S, S)]
    h_prev, c_prev, flips = h0.astype(np.float32), None, 0
    for l, (layer, q) in enumerate(layers):
        buf = LayerBuffers(to_np(ws[l]), layer.layout, M, H, F, 4)
        h_out = to_np(hs[l]).astype(np.float32)
        q_next = oracle.unpack_nibbles(to_np(qs[l]), H)
        flips += check_layer_stagewise(buf, q, h_prev, h_out, seqs, c0_in=c_prev, q_next=q_next, s_out_next=s_next,
                                       what=f"layer {l}")
        h_prev, c_prev = h_out, q_next
    # drift of the chain against the oracle's own 12 layers on the two sequences (codes flip here and there
    # along the way): the outputs stay close as a whole
    sel = np.concatenate([np.arange(r0, r0 + n) for (r0, n) in seqs])
    x_ref, c_ref = h0[sel].astype(np.float32), None
    for l, (_, q) in enumerate(layers):
        q = dict(q, batch=len(seqs), seq=S)
        # as on the GPU: the next layer takes the binary16 output and the codes of the binary32 one
        y, _ = oracle.bert_layer_int4(q, x_ref, act_dtype=oracle.F16, c0=c_ref)
        x_ref, c_ref = oracle.round_storage(y, oracle.F16), oracle.quantize(y, s_next)
    err = to_np(hs[-1]).astype(np.float32)[sel] - x_ref
    drift = float(np.sqrt((err ** 2).mean()) / np.sqrt((x_ref ** 2).mean()))
    print(f"12-layer chain: {flips} codes differ from the teacher-forced oracle inside their bands; "
          f"rms drift against the oracle's own chain {drift:.4f}")
    assert drift < 0.15


def test_student_four_layer_chain_teacher_forced(mkq):
    """The 4-layer student (hidden 312, 12 heads of 26, FFN 1200) at 32 x 128 tokens, chained through
    q_out_next / q_in: the code rows that cross from layer to layer have a pitch of 384 codes with zero padding.
    Every stage of every layer against the oracle on two sequences, each layer fed the GPU's previous output."""
    import torch
    from layer_checks import code_row_pitch
    B, S, H, heads, F, LAYERS = 32, 128, 312, 12, 1200, 4
    M, pitch = B * S, code_row_pitch(H)
    steps = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
    s_next = steps["qkv"]
    h0 = wl.hidden_states(B, S, H, 5).astype(np.float16)
    layers = []
    for l in range(LAYERS):
        p = wl.bert_layer_weights(H, heads, F, 200 + l)
        packed, q = {}, {k: p[k] for k in ("hidden", "heads", "ffn", "ln_eps", "ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
        for nm in ("qkv", "ao", "up", "down"):
            Wq, s_w = mkq.mkq_pack_weights_int4_padded(to_dev(p["W_" + nm]))
            packed[nm] = (Wq, s_w, to_dev(p["b_" + nm]))
            q["w_" + nm], q["sw_" + nm] = oracle.quantize_weights(p["W_" + nm])
            q["b_" + nm], q["sx_" + nm] = p["b_" + nm], steps[nm]
        ln = {k: to_dev(p[k]) for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
        layers.append((mkq.BertLayerInt4(B, S, H, heads, F, packed, steps, ln, p["ln_eps"], s_next), q))
    ws = [torch.full((layers[0][0].workspace_bytes(),), 0x3C, dtype=torch.uint8, device="cuda") for _ in range(LAYERS)]
    hs = [torch.empty((M, H), dtype=torch.float16, device="cuda") for _ in range(LAYERS)]
    qs = [torch.full((M, pitch // 2), 0x3C, dtype=torch.uint8, device="cuda") for _ in range(LAYERS)]
    x, qin = to_dev(h0), None
    for l, (layer, _) in enumerate(layers):
        layer(x, ws[l], h_out=hs[l], q_in=qin, q_out_next=qs[l])
        x, qin = hs[l], qs[l]
    torch.cuda.synchronize()
    seqs = [(0, S), (17 * S, S)]
    h_prev, c_prev, flips = h0.astype(np.float32), None, 0
    for l, (layer, q) in enumerate(layers):
        buf = LayerBuffers(to_np(ws[l]), layer.layout, M, H, F, 4)
        h_out = to_np(hs[l]).astype(np.float32)
        rows = oracle.unpack_nibbles(to_np(qs[l]), pitch)
        assert not rows[:, H:].any(), "padding codes handed to the next layer must be zero"
        flips += check_layer_stagewise(buf, q, h_prev, h_out, seqs, c0_in=c_prev, q_next=rows[:, :H], s_out_next=s_next,
                                       what=f"student layer {l}")
        h_prev, c_prev = h_out, rows[:, :H]
    assert np.isfinite(to_np(hs[-1]).astype(np.float32)).all()


@pytest.mark.parametrize("M", [440, 537, 681, 1691, 2011, 2298])
@pytest.mark.parametrize("K,N", [(768, 2304), (3072, 768)])
def test_padding_free_token_counts(mkq, M, K, N):
    """The valid-token counts of the paper's Table 2 (section 5.4): ragged M, binary16 out, 4 and 8 bits."""
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed=M)
    b = np.random.default_rng(M).normal(0, 0.1, N).astype(np.float32)
    r = mkq.mkq_linear_int4(mkq.mkq_pack_codes_int4(to_dev(A)), s_x, mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1),
                            to_dev(s_w), to_dev(b), N, K, mkq.MKQ_F16, want_acc=True)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, b, out_dtype=oracle.F16)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    rng = np.random.default_rng(M + 1)
    A8 = rng.integers(-128, 128, (M, K), dtype=np.int8)
    W8 = rng.integers(-128, 128, (N, K), dtype=np.int8)
    r = mkq.mkq_linear_int8(to_dev(A8), 0.01, to_dev(W8), to_dev(s_w), to_dev(b), mkq.MKQ_F16)
    ref = oracle.linear_int4(A8, 0.01, W8, s_w, b, out_dtype=oracle.F16, qmin=-128, qmax=127)
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])


@pytest.mark.parametrize("M,K,N", [(4096, 3072, 768), (4099, 4096, 1024), (2560, 4096, 1024)])
def test_ffn_down_shapes_split_k_tiles_sampled_rows(mkq, M, K, N):
    """FFN-down of a BERT-base / BERT-large layer at M around 4096: at most one 128 x 128 tile per CU and
    a long k loop, which the automatic choice runs with two wave groups sharing the tile's K; binary16
    residual and output as in the layer."""
    import torch
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed=K + M)
    rng = np.random.default_rng(M)
    b = rng.normal(0, 0.3, N).astype(np.float32)
    res = rng.normal(0, 1, (M, N)).astype(np.float16)
    a_d = _pack_rows_on_device(mkq, A)
    w_d = mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1)
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), to_dev(b), N, K, mkq.MKQ_F16, residual=to_dev(res), out=out)
    torch.cuda.synchronize()
    rows = _sample_rows(M, rng)
    got = to_np(out[torch.from_numpy(rows).cuda()]).astype(np.float32)
    ref = oracle.linear_int4(A[rows], s_x, Wc, s_w, b, residual=res[rows].astype(np.float32), out_dtype=oracle.F16)
    assert np.array_equal(got, ref["y"])


@pytest.mark.parametrize("M,K,N", [(16, 16384, 16384), (64, 16384, 16384), (16, 8192, 28672), (1, 28672, 8192), (16, 32768, 32768)])
def test_few_token_streaming_at_benchmark_sizes(mkq, M, K, N):
    """The few-token points of the benchmark (112-512 MiB of weights, both weight layouts, the K split with the
    scratch area that the benchmark hands over): whole output against the oracle."""
    rng = np.random.default_rng(M + K + N)
    A = rng.integers(-8, 8, (M, K), dtype=np.int8)
    Wc = rng.integers(-8, 8, (N, K), dtype=np.int8)
    s_w = rng.uniform(0.001, 0.05, N).astype(np.float32)
    s_x = 0.01
    ref = oracle.linear_int4(A, s_x, Wc, s_w, None, out_dtype=oracle.F16)
    a_d = mkq.mkq_pack_codes_int4(to_dev(A))
    w_d = _pack_rows_on_device(mkq, Wc).reshape(-1)
    scr = mkq.mkq_splitk_scratch_init()
    r = mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), None, N, K, mkq.MKQ_F16, splitk_scratch=scr, want_acc=True)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    w_s = mkq.mkq_repack_weights_int4_stream(w_d, N, K)
    del w_d
    r = mkq.mkq_linear_int4_stream(a_d, s_x, w_s, to_dev(s_w), None, N, K, mkq.MKQ_F16, splitk_scratch=scr, want_acc=True)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
