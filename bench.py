#!/usr/bin/env python3
"""Benchmark of the W4A4 linear hot path on one MI355X.

One step = one pass of the whole hot path over the BERT-base layer GEMM workload
(M = 8 x 128 tokens; QKV 768->2304, attention-out 768->768, FFN-up 768->3072,
FFN-down 3072->768): for each linear, activation quantize (binary16 in, learned
per-tensor step) -> int4 x int4 GEMM (int32 accumulate) -> dequantize epilogue
with bias -> binary16 out.  Inputs are synthetic and resident in HBM before the
timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0  # MI355X dense int8 matrix peak (published), TOP/s
HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the large-M / small-M side measurements")
    return ap.parse_args()


def event_time(fn, iters, warm=3):
    """Average seconds per call of fn(), HIP events on the current stream."""
    import torch
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters


class LinearCase:
    """Device-resident operands of one quantized linear."""

    def __init__(self, mkq, name, X16, W, b, s_x, out_dtype):
        import torch
        self.mkq, self.name = mkq, name
        self.M, self.K = X16.shape
        self.N = W.shape[0]
        self.X = torch.from_numpy(X16).cuda()
        self.Wq, self.s_w = mkq.mkq_pack_weights_int4(torch.from_numpy(W).cuda())
        self.b = torch.from_numpy(b).cuda()
        self.s_x = float(s_x)
        self.out_dtype = out_dtype
        self.out = torch.empty((self.M, self.N), dtype=torch.float16, device="cuda")
        self.ws = torch.empty(mkq.mkq_linear_int4_workspace_bytes(self.M, self.N, self.K, mkq.MKQ_F16),
                              dtype=torch.uint8, device="cuda")
        self.codes = mkq.mkq_quantize(self.X, self.s_x)
        self.ops = 2.0 * self.M * self.N * self.K
        # algorithmic bytes of the GEMM kernel: packed A + packed W + steps/bias + binary16 out
        self.gemm_bytes = self.M * self.K / 2 + self.N * self.K / 2 + 8 * self.N + 2 * self.M * self.N

    def full(self):  # quantize + GEMM + epilogue, float activations in
        self.mkq.mkq_linear_int4(self.X, self.s_x, self.Wq, self.s_w, self.b, self.N, self.K,
                                 self.out_dtype, out=self.out, workspace=self.ws)

    def gemm_only(self):  # pre-quantized activations in
        self.mkq.mkq_linear_int4(self.codes, self.s_x, self.Wq, self.s_w, self.b, self.N, self.K,
                                 self.out_dtype, out=self.out)


def cpu_baseline(cfg, wl, seconds_target=12.0):
    """The oracle, as it stands, on the same workload (rank 0, host cores)."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(cfg["seed"])
    M = cfg["M"]
    cases = []
    for name, K, N in cfg["shapes"]:
        X = wl.outlier_activations(rng, M, K, cfg["outlier_frac"], cfg["outlier_kind"]).astype(np.float16)
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
        b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
        wc, s_w = oracle.quantize_weights(W)
        cases.append((X.astype(np.float32), wc, s_w, b))
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    ops = sum(2.0 * M * c[1].shape[0] * c[1].shape[1] for c in cases)

    def step():
        for X, wc, s_w, b in cases:
            oracle.linear_int4(oracle.quantize(X, s_x), s_x, wc, s_w, b, out_dtype=oracle.F16)

    step()
    t0 = time.perf_counter()
    n = 0
    while True:
        step()
        n += 1
        el = time.perf_counter() - t0
        if el >= seconds_target or n >= 50:
            break
    return {"value": ops * n / el / 1e12, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n} full steps of the same workload (all 4 linears, M={M}) in {el:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); data-parallel sharding over "
              "tokens is described in DESIGN.md but not built.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2203_13483_amd as mkq
    from paper_2203_13483_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    mkq.load()

    cfg = wl.CONFIGS[1]
    M = cfg["M"]
    rng = np.random.default_rng(cfg["seed"])
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    cases = []
    for name, K, N in cfg["shapes"]:
        X = wl.outlier_activations(rng, M, K, cfg["outlier_frac"], cfg["outlier_kind"]).astype(np.float16)
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
        b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
        cases.append(LinearCase(mkq, name, X, W, b, s_x, mkq.MKQ_F16))
    total_ops = sum(c.ops for c in cases)

    def step():
        for c in cases:
            c.full()

    # --- the timed region: W warm-up steps, then exactly K steps -----------------
    graph = None
    if not args.no_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
    run = graph.replay if graph is not None else step
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = total_ops / (elapsed / args.steps) / 1e12

    # --- roofline of the dominant kernel (the int4 GEMM), HIP events -------------
    iters = max(50, min(args.steps, 500))
    t_gemm = [event_time(c.gemm_only, iters) for c in cases]
    achieved = total_ops / sum(t_gemm) / 1e12
    roofline = {
        "bound": "mfma", "kernel": "gemm_i4_kernel", "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS,
        "unit": "TOP/s", "frac": achieved / INT8_MFMA_PEAK_TOPS, "traffic": None,
        "per_launch_us": {c.name: t * 1e6 for c, t in zip(cases, t_gemm)},
        "note": "ops = 2*M*N*K per launch; duration = HIP events around back-to-back launches of that GEMM only",
    }

    extra = {}
    if not args.no_extra:
        extra = side_measurements(mkq, event_time)

    out = {
        "metric": "int4_linear_TOPS", "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4xint4->int32 (int8 MFMA), f32 epilogue", "data": "synthetic",
        "config": {"workload": "BASELINE configs[1]: BERT-base layer GEMMs int4, M=1024 (8x128 tokens), "
                               "QKV 768->2304, attn-out 768->768, FFN-up 768->3072, FFN-down 3072->768; "
                               "binary16 activations in, quantize + GEMM + dequantize, binary16 out",
                   "launch": "HIP graph replay" if graph is not None else "eager"},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, wl)
    if extra:
        out["extra"] = extra
    print(json.dumps(out))


def side_measurements(mkq, event_time):
    """Large-M (MFMA-bound) and small-M (weight-streaming) points beside the headline."""
    import torch
    res = {"large_m": [], "small_m": []}
    for (M, K, N) in [(16384, 1024, 4096), (16384, 4096, 1024), (16384, 768, 3072), (65536, 1024, 4096)]:
        a = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
        w = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
        sw = torch.rand(N, device="cuda") * 0.049 + 0.001
        out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        t = event_time(lambda: mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_BF16, out=out), 30)
        tops = 2.0 * M * N * K / t / 1e12
        res["large_m"].append({"M": M, "K": K, "N": N, "out": "bf16", "us": t * 1e6, "TOPS": tops,
                               "frac_int8_peak": tops / INT8_MFMA_PEAK_TOPS})
        del a, w, out
    return res


if __name__ == "__main__":
    main()
