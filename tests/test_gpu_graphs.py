"""The library's launches under HIP graph capture: every entry point enqueues kernels only (fill kernels, not
memsets; no allocation, no synchronisation), so a captured graph must reproduce the eager result on every
replay -- also the paths that keep state in device memory between kernels (ticket counters of the K split
across workgroups, the histogram workspace of the percentile calibration, the layer's workspace).  Each graph
is replayed several times with new input data, eager work and synchronisations in between, and every replay is
compared bit for bit with the eager result on the same data (which the other tests hold to the oracle)."""
import numpy as np
import pytest

from paper_2203_13483_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    assert m.load().mkq_init() == m.MKQ_OK  # once-per-device set-up must not happen inside a capture
    return m


def _replays(torch, make_inputs, load_inputs, run, outputs, n=4):
    """Captures run() once, then n times: new inputs, eager result, some unrelated eager work, replay, compare."""
    load_inputs(make_inputs(0))
    run()  # warm-up outside the capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run()
    for i in range(1, n + 1):
        load_inputs(make_inputs(i))
        run()
        torch.cuda.synchronize()
        want = [o.clone() for o in outputs()]
        for o in outputs():
            o.fill_(0x5A if o.dtype == torch.uint8 else 7)
        junk = torch.randn(1 << 16, device="cuda").sum()  # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outputs(), want):
            assert torch.equal(got, ref), f"replay {i}"
        assert bool(torch.isfinite(junk))


def test_encoder_layer_graph_replays(mkq):
    import torch
    B, S, H, heads, F = 4, 96, 256, 4, 512
    p = wl.bert_layer_weights(H, heads, F, 11)
    packed = {nm: mkq.mkq_pack_weights_int4(torch.from_numpy(p["W_" + nm]).cuda()) + (torch.from_numpy(p["b_" + nm]).cuda(),)
              for nm in ("qkv", "ao", "up", "down")}
    ln = {k: torch.from_numpy(p[k]).cuda() for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    sx = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
    layer = mkq.BertLayerInt4(B, S, H, heads, F, packed, sx, ln, 1e-12, 0.4)
    h = torch.empty((B * S, H), dtype=torch.float16, device="cuda")
    out = torch.empty_like(h)
    qn = torch.empty((B * S, H // 2), dtype=torch.uint8, device="cuda")
    ws = torch.empty(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
    _replays(torch, lambda i: torch.from_numpy(wl.hidden_states(B, S, H, 100 + i).astype(np.float16)),
             lambda x: h.copy_(x), lambda: layer(h, ws, h_out=out, q_out_next=qn), lambda: [out, qn])


@pytest.mark.parametrize("M,N,K", [(16, 4096, 8192), (100, 1000, 4096)])
def test_few_token_split_k_graph_replays(mkq, M, N, K):
    """Four calls in one graph share one scratch area: the ticket counters must be back at zero after each."""
    import torch
    scr = mkq.mkq_splitk_scratch_init()
    ws_ = [torch.randint(0, 256, (mkq.mkq_stream_weight_bytes(N, K),), dtype=torch.uint8, device="cuda") for _ in range(4)]
    wc = [torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda") for _ in range(2)]
    sw = torch.rand(N, device="cuda") * 0.049 + 0.001
    a = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    outs = [torch.empty((M, N), dtype=torch.float16, device="cuda") for _ in range(6)]

    def run():
        for w, o in zip(ws_, outs):
            mkq.mkq_linear_int4_stream(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=o, splitk_scratch=scr, k_slices=4)
        for w, o in zip(wc, outs[4:]):  # canonical rows: the ring kernel with its K split, then the library's route
            mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=o, splitk_scratch=scr)

    _replays(torch, lambda i: torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda",
                                            generator=torch.Generator("cuda").manual_seed(i)),
             lambda x: a.copy_(x), run, lambda: outs)
    assert int(scr[:16384].view(torch.int32).abs().sum()) == 0


def test_float_input_linear_and_calibration_graph_replays(mkq):
    import torch
    M, K, N = 300, 768, 520
    W = torch.randn(N, K, device="cuda") * 0.02
    Wq, s_w = mkq.mkq_pack_weights_int4(W)
    b = torch.randn(N, device="cuda") * 0.01
    x = torch.empty((M, K), dtype=torch.float16, device="cuda")
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    wsl = torch.empty(mkq.mkq_linear_int4_workspace_bytes(M, N, K, mkq.MKQ_F16), dtype=torch.uint8, device="cuda")
    s1 = torch.empty(1, dtype=torch.float32, device="cuda")
    g2 = torch.empty(2, dtype=torch.float64, device="cuda")
    wsp = torch.empty(mkq.mkq_percentile_scale_workspace_bytes(), dtype=torch.uint8, device="cuda")

    def run():
        mkq.mkq_linear_int4(x, 0.34, Wq, s_w, b, N, K, mkq.MKQ_F16, out=out, workspace=wsl)
        mkq.mkq_percentile_scale(x, 100, 4, s_out=s1, workspace=wsp)
        mkq.mkq_scale_gradients(x, 0.34, 4, g_out=g2)

    # (the scale-gradient sums are atomic additions in an order that is not fixed: compared separately)
    _replays(torch, lambda i: torch.randn((M, K), device="cuda", generator=torch.Generator("cuda").manual_seed(50 + i)).half(),
             lambda v: x.copy_(v), run, lambda: [out, s1])
    assert bool(torch.isfinite(g2).all())
