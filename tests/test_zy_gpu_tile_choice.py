"""The library's own choice of kernel configuration against every configuration it could have picked, at the
benchmark's shapes: the automatic choice must not be more than 5 % (plus timer noise) slower than the fastest
forced configuration.  A timing test: medians of graph replays, on an otherwise idle GPU (the file's name puts it
behind the parity tests: a noisy machine must not keep them from running)."""
import pytest

pytestmark = pytest.mark.gpu

CONFIGS = [11, 12, 14, 18, 19, 20, 27, 28, 29, 31, 33, 35]
# (M, K, N): BERT-base layer GEMMs at M = 1024 and 4096, BERT-large at M = 8192, the large-M sweep at M = 16384
SHAPES = ([(M, K, N) for M in (1024, 4096) for (K, N) in ((768, 2304), (768, 768), (768, 3072), (3072, 768))]
          + [(8192, 1024, 3072), (8192, 1024, 1024), (8192, 1024, 4096), (8192, 4096, 1024)]
          + [(16384, 1024, 4096), (16384, 4096, 1024), (16384, 768, 3072)])


def _time(fn, rep=10, samples=7):
    import torch
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(rep):
            fn()
    ts = []
    for _ in range(samples):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g.replay()
        e0.record()
        g.replay()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        ts.append(e0.elapsed_time(e1) / (2 * rep))
    return sorted(ts)[len(ts) // 2]


# the layer's own epilogues at the BERT-base shapes: binary16 residual (attention-out, FFN-down), GELU with
# codes out (FFN-up)
EPILOGUES = [(M, K, N, kind) for M in (1024, 4096)
             for (K, N, kind) in ((768, 768, "residual"), (768, 3072, "gelu"), (3072, 768, "residual"))]


@pytest.mark.parametrize("M,K,N,kind", [s + ("plain",) for s in SHAPES] + EPILOGUES)
def test_automatic_choice_is_within_five_percent_of_the_best(M, K, N, kind):
    import torch
    import paper_2203_13483_amd as mkq
    mkq.load()
    a = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
    w = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
    sw = torch.rand(N, device="cuda") * 0.049 + 0.001
    out = torch.empty((M, N), dtype=torch.float16, device="cuda")
    res = torch.randn((M, N), dtype=torch.float16, device="cuda") if kind == "residual" else None
    codes = torch.empty((M, N // 2), dtype=torch.uint8, device="cuda")

    def run(cfg):
        if kind == "gelu":
            return lambda: mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_I4, out=codes, act=mkq.MKQ_ACT_GELU,
                                               s_next=0.3, config=cfg)
        return lambda: mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=out, residual=res, config=cfg)

    times = {}
    for cfg in CONFIGS:
        try:
            run(cfg)()
        except mkq.MkqError as e:
            assert e.status == mkq.MKQ_ERR_UNSUPPORTED
            continue
        times[cfg] = _time(run(cfg))
    best_cfg = min(times, key=times.get)
    # the clock moves between measurements (the sweep above heats the chip): the two that are compared are timed
    # again side by side, at least five and at most ten times, and each keeps its fastest sample
    auto = float("inf")
    for attempt in range(10):
        auto = min(auto, _time(run(None)))
        times[best_cfg] = min(times[best_cfg], _time(run(best_cfg)))
        if attempt >= 4 and auto <= 1.05 * times[best_cfg] + 0.0003:
            break
    print(f"M={M} K={K} N={N} {kind}: automatic {auto * 1e3:.2f} us, best forced {best_cfg}: {times[best_cfg] * 1e3:.2f} us; "
          + " ".join(f"{c}:{t * 1e3:.1f}" for c, t in sorted(times.items())))
    assert auto <= 1.05 * times[best_cfg] + 0.0003, (auto, best_cfg, times[best_cfg])
