#!/usr/bin/env python3
"""Benchmark of the W4A4 linear hot path on one MI355X.

One step = one int4 linear at the largest point of the large-M sweep (M = 65536 tokens,
K = 1024, N = 4096): nibble-packed int4 codes in -> int4 x int4 GEMM (int32 accumulate)
-> dequantize epilogue with per-channel scales -> bfloat16 out.  Inputs are synthetic and
resident in HBM before the timed region.  The other workloads (BERT-base layer GEMMs at
M = 1024 with the activation quantizer, the rest of the large-M sweep, few-token weight
streaming, the 12-layer encoder, ...) are measured beside it under "extra".  Prints ONE JSON line.
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
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the large-M / small-M side measurements")
    ap.add_argument("--only", choices=["headline", "large-m", "small-m", "calibration", "layers"], default=None,
                    help="run only that group of side measurements, eagerly and a few launches each (the form "
                         "that rocprofv3 --kernel-trace / --pmc runs are taken of); prints their JSON")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one 256 MiB device-to-device copy kernel, so that a rocprofv3 --pmc run "
                         "of this command holds a kernel of known HBM traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


def graph_time(fn, rep=20, repeats=7, inner=5):
    """Median seconds per call of fn(): a HIP graph of `rep` back-to-back calls, replayed
    `inner` times per sample, `repeats` samples (clocks settle during the first ones)."""
    import torch
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(rep):
            fn()
    ts = sorted(event_time(g.replay, inner, warm=2) / rep for _ in range(repeats))
    return ts[len(ts) // 2]


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


HEADLINE = (65536, 1024, 4096)  # (M, K, N): the largest point of the large-M sweep (configs[4] of the task's baseline file)
HEADLINE_SEED = 4


def cpu_baseline(A, Wc, s_w, s_x, rows, seconds_target=12.0):
    """The oracle, as it stands, on a row sample of the headline's own inputs (rank 0, host cores)."""
    import oracle
    As = A[:rows]
    ops = 2.0 * rows * Wc.shape[0] * Wc.shape[1]
    oracle.linear_int4(As[:256], s_x, Wc, s_w, None, out_dtype=oracle.BF16)
    t0 = time.perf_counter()
    n = 0
    while True:
        oracle.linear_int4(As, s_x, Wc, s_w, None, out_dtype=oracle.BF16)
        n += 1
        el = time.perf_counter() - t0
        if el >= seconds_target or n >= 50:
            break
    return {"value": ops * n / el / 1e12, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "build": oracle.build_flags(),
            "sample": f"{n} passes over rows 0..{rows - 1} of the headline's activations (all {Wc.shape[0]} channels, "
                      f"K={Wc.shape[1]}, bf16 out) in {el:.1f} s"}


def measured_ceilings(mkq):
    """What this machine delivers: HBM read / write / copy of 1 GiB with plain streaming kernels, and the int8 MFMA
    in a register-only loop on operands of the kind the GEMM multiplies (16 * code, uniform codes)."""
    import torch
    out = {}
    nbytes = 1 << 30
    src = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    for name, kind, moved in (("hbm_read_GBps", 0, nbytes), ("hbm_write_GBps", 1, nbytes), ("hbm_copy_GBps", 2, 2 * nbytes)):
        t = sorted(event_time(lambda: mkq.mkq_measure_stream(kind, src, dst, nbytes), 5, warm=1) for _ in range(3))[1]
        out[name] = moved / t / 1e9
    del src, dst
    nb = int(mkq.load().mkq_measure_mfma_i8_operand_bytes())
    codes = torch.randint(-8, 8, (nb,), dtype=torch.int8, device="cuda")
    ops16 = (codes * 16).contiguous()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    iters = 4096
    n_ops = mkq.mkq_measure_mfma_i8(ops16, iters, sink)
    ts = sorted(event_time(lambda: mkq.mkq_measure_mfma_i8(ops16, iters, sink), 5, warm=2) for _ in range(5))
    out["mfma_i8_TOPS"] = n_ops / ts[2] / 1e12
    # one v_mfma_i32_32x32x32_i8 (65536 operations) occupies a SIMD's matrix pipe for 32 cycles: the rate of a
    # loop that keeps the pipe full is 2048 operations per cycle and SIMD, so its rate tells the sustained clock
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out["sustained_clock_GHz_under_the_mfma_loop"] = n_ops / ts[2] / (cus * 4 * 2048) / 1e9
    out["note"] = ("1 GiB streaming kernels; register-only v_mfma_i32_32x32x32_i8 loop, 8 accumulator tiles per "
                   "wave, 8 waves per CU, operands = 16 * uniform codes (the chip's clock under load depends on "
                   "the data)")
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (--gpus 1); data-parallel sharding over "
              "tokens is described in the design notes but not built.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2203_13483_amd as mkq
    from paper_2203_13483_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    mkq.load()

    if args.pmc_calibration:
        src = torch.ones(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.only and args.only != "headline":
        print(json.dumps(profile_launches(mkq, args.only)))
        return

    # --- headline: the largest point of the large-M sweep: uniform int4 codes in, int4 x int4 GEMM with
    # int32 accumulation, dequantize with per-channel scales, bf16 out ------------------------------------
    M, K, N = HEADLINE
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, HEADLINE_SEED)
    a_d = mkq.mkq_pack_codes_int4(torch.from_numpy(A).cuda())
    w_d = mkq.mkq_pack_codes_int4(torch.from_numpy(Wc).cuda()).reshape(-1)
    sw_d = torch.from_numpy(s_w).cuda()
    out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    ops = 2.0 * M * N * K
    alg_bytes = M * K / 2 + N * K / 2 + 4 * N + 2 * M * N

    def step():
        mkq.mkq_linear_int4(a_d, s_x, w_d, sw_d, None, N, K, mkq.MKQ_BF16, out=out)

    # the ceilings every fraction below is also quoted against (stream read / write / copy, register-only MFMA
    # loop); measured first, so that the chip has left its idle clocks before the warm-up steps
    ceil = None if args.only == "headline" else measured_ceilings(mkq)
    # Untimed settling, before the warm-up steps: from idle the chip runs its first few launches at the top clock,
    # is then pulled far below its sustained clock by the power manager and recovers over some tens of
    # milliseconds (per-launch durations of 257, 257, ..., 350, 415, 410, ..., 330, ..., 290 us were measured).
    # Windows of 20 launches are timed until two in a row agree within 1.5 %, so that the timed steps below see
    # the sustained state whatever --warmup is.
    settle = {"launches": 0, "window_us": []}
    if args.only != "headline":
        prev = None
        agree = 0
        while settle["launches"] < 1000 and agree < 2:
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for _ in range(20):
                step()
            ev1.record()
            torch.cuda.synchronize()
            t_win = ev0.elapsed_time(ev1) / 20 * 1e3
            settle["launches"] += 20
            settle["window_us"].append(round(t_win, 1))
            agree = agree + 1 if (prev is not None and abs(t_win - prev) <= 0.015 * prev) else 0
            prev = t_win
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = ops / (elapsed / args.steps) / 1e12
    # launch duration of the dominant (the only) kernel: HIP events on the launch stream around the timed region
    launch_s = e0.elapsed_time(e1) * 1e-3 / args.steps
    achieved = ops / launch_s / 1e12
    if args.only == "headline":
        print(json.dumps({"only": "headline", "M": M, "K": K, "N": N, "launches": args.steps + args.warmup,
                          "us_per_launch": launch_s * 1e6}))
        return

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "gemm_i4_headline_hbm_traffic.txt")
    if os.path.exists(tpath):
        for line in open(tpath):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])
    roofline = {
        "bound": "mfma", "kernel": "gemm_i4_dma_kernel<256x128 tiles, 3-stage ring, bf16 line epilogue>",
        "achieved": achieved, "peak": INT8_MFMA_PEAK_TOPS, "unit": "TOP/s", "frac": achieved / INT8_MFMA_PEAK_TOPS,
        "traffic": traffic, "algorithmic_bytes_per_launch": alg_bytes, "us_per_launch": launch_s * 1e6,
        "measured_mfma_ceiling_TOPS": ceil["mfma_i8_TOPS"], "frac_of_measured_mfma_ceiling": achieved / ceil["mfma_i8_TOPS"],
        "output_write_us_at_measured_hbm_write_rate": 2.0 * M * N / (ceil["hbm_write_GBps"] * 1e9) * 1e6,
        "note": "achieved = 2*M*N*K per launch / average launch duration (HIP events on the launch stream around "
                "the timed steps, back-to-back launches of the one kernel of a step)",
    }

    extra = {"measured_ceilings": ceil}
    if not args.no_extra:
        extra.update(side_measurements(mkq, event_time, ceil))

    res = {
        "metric": "int4_linear_TOPS", "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int4 (int8 MFMA, int32 accumulate)", "data": "synthetic",
        "config": {"workload": f"BASELINE configs[4], largest point: int4 GEMM M={M}, K={K}, N={N}; signed int4 "
                               "uniform codes in [-8,7] in (nibble-packed, resident in HBM), per-channel fp32 scales "
                               "U(0.001,0.05), bf16 out; one step = one linear (GEMM + dequantize epilogue)",
                   "launch": "eager, back-to-back on one stream",
                   "settling_before_warmup": f"{settle['launches']} untimed launches of the same step, in windows "
                                             "of 20 until two windows in a row agree within 1.5 % (the power "
                                             "manager's transient after idle); us per launch of the windows: "
                                             + " ".join(str(t) for t in settle["window_us"])},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(A, Wc, s_w, s_x, rows=16384)
    if not args.no_extra:
        res["summary"] = summary(extra)
    res["extra"] = extra
    print(json.dumps(res))


def summary(extra):
    """The target-bearing side measurements in short form, ahead of the long `extra` object: fractions of the
    published peaks (int8 matrix 5000 TOP/s, HBM 8000 GB/s) and, second, of the ceilings measured in this run."""
    r3 = lambda v: None if v is None else round(v, 3)
    out = {"large_m_MKN_frac_int8_peak_frac_measured_ceiling_e3m2_route_frac_rotating_buffers_frac": [
               [r["M"], r["K"], r["N"], r3(r["frac_int8_peak"]), r3(r["frac_measured_mfma_ceiling"]),
                r3(r.get("e3m2_route_frac_int8_peak")), r3(r.get("rotating_buffers_frac_int8_peak"))]
               for r in extra.get("large_m", [])],
           "small_m_MKN_layout_us_frac_hbm_peak_frac_measured_read": []}
    for r in extra.get("small_m", []):
        for layout in ("canonical", "stream"):
            if layout + "_us_per_call" in r:
                out["small_m_MKN_layout_us_frac_hbm_peak_frac_measured_read"].append(
                    [r["M"], r["K"], r["N"], layout, round(r[layout + "_us_per_call"], 1), r3(r[layout + "_frac_hbm_peak"]),
                     r3(r[layout + "_frac_measured_read_ceiling"])])
    enc = extra.get("encoder") or {}
    out["bert_base_layer_us_int4_int8_fp16"] = [r3(enc.get("int4_us_per_layer")), r3(enc.get("int8_us_per_layer")),
                                                r3(enc.get("fp16_us_per_layer"))]
    return out


# (M, K, N): the large-M sweep and, last, a long-K square where the k loop outweighs the per-tile costs
LARGE_M_SHAPES = [(M, K, N) for M in (16384, 32768, 65536) for (K, N) in ((1024, 4096), (4096, 1024), (768, 3072))] + [
    (8192, 8192, 8192)]
# few tokens: (K, N, number of distinct weight matrices cycled through, token counts); the pool is at least 1 GiB
SMALL_M_SHAPES = [(4096, 4096, 128, (1, 16, 64, 128, 512)), (8192, 8192, 32, (16, 64)), (16384, 16384, 8, (1, 16, 64)),
                  (8192, 28672, 9, (16,)), (28672, 8192, 9, (16,)), (32768, 32768, 3, (16,))]
CALIBRATION_SHAPE = (16384, 4096)  # one activation tensor of the large-M sweep


def profile_launches(mkq, which, launches=5):
    """A few eager launches of each large-M GEMM (bf16 out) or of the small-M weight-streaming
    linears (cold weights), for profiler runs; returns what was launched."""
    import torch
    done = []
    if which == "large-m":
        for (M, K, N) in LARGE_M_SHAPES:
            a = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
            w = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
            sw = torch.rand(N, device="cuda") * 0.049 + 0.001
            out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
            for _ in range(launches):
                mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_BF16, out=out)
            torch.cuda.synchronize()
            # the experimental 6-bit float route of the same linear
            a6 = mkq.mkq_pack_codes_e3m2(torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda"))
            w6 = mkq.mkq_pack_codes_e3m2(torch.randint(-8, 8, (N, K), dtype=torch.int8, device="cuda"))
            for _ in range(launches):
                mkq.mkq_linear_int4_e3m2(a6, 0.01, w6, sw, None, mkq.MKQ_BF16, out=out)
            torch.cuda.synchronize()
            done.append({"M": M, "K": K, "N": N, "launches": launches, "ops_per_launch": 2.0 * M * N * K,
                         "grid_threads": None})
            del a, w, out, a6, w6
    elif which == "layers":
        # whole encoder layers in 4 bits, eagerly: every kernel of the layer shows with its own duration
        from paper_2203_13483_amd import workloads as wl
        for (name, batch, seq, H, heads, F) in (("bert_base", 32, 128, 768, 12, 3072),
                                                ("bert_large_seq512", 16, 512, 1024, 16, 4096),
                                                ("student_4layer", 32, 128, 312, 12, 1200)):
            p = wl.bert_layer_weights(H, heads, F, 301)
            ln = {k: torch.from_numpy(p[k]).cuda() for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
            pack = mkq.mkq_pack_weights_int4_padded if H % 32 else mkq.mkq_pack_weights_int4
            packed = {nm: pack(torch.from_numpy(p["W_" + nm]).cuda()) + (torch.from_numpy(p["b_" + nm]).cuda(),)
                      for nm in ("qkv", "ao", "up", "down")}
            sx = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
            layer = mkq.BertLayerInt4(batch, seq, H, heads, F, packed, sx, ln, 1e-12)
            h = torch.randn((batch * seq, H), dtype=torch.float16, device="cuda")
            out = torch.empty_like(h)
            ws = torch.empty(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
            for _ in range(launches):
                layer(h, ws, h_out=out)
            torch.cuda.synchronize()
            done.append({"layer": name, "batch": batch, "seq": seq, "hidden": H, "heads": heads, "ffn": F,
                         "launches": launches})
    elif which == "calibration":
        M, K = CALIBRATION_SHAPE
        x = torch.randn((M, K), dtype=torch.float16, device="cuda")
        g = torch.empty(2, dtype=torch.float64, device="cuda")
        s1 = torch.empty(1, dtype=torch.float32, device="cuda")
        wsp = torch.empty(mkq.mkq_percentile_scale_workspace_bytes(), dtype=torch.uint8, device="cuda")
        for _ in range(launches):
            mkq.mkq_scale_gradients(x, 0.34, 4, g_out=g)
            mkq.mkq_percentile_scale(x, 100, 4, s_out=s1, workspace=wsp)
        torch.cuda.synchronize()
        done.append({"M": M, "K": K, "x": "binary16", "launches": launches, "bytes_per_pass": 2 * M * K})
    else:
        scr = mkq.mkq_splitk_scratch_init()
        for (K, N, pool) in ((4096, 4096, 24), (16384, 16384, 8), (8192, 28672, 8), (32768, 32768, 3)):
            ws = [torch.randint(0, 256, (mkq.mkq_stream_weight_bytes(N, K),), dtype=torch.uint8, device="cuda")
                  for _ in range(pool)]
            sw = torch.rand(N, device="cuda") * 0.049 + 0.001
            for M in (1, 16, 64):
                a = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
                out = torch.empty((M, N), dtype=torch.float16, device="cuda")
                for rep in range(3):
                    for w in ws:  # canonical rows, then the streaming layout (the bytes are random either way)
                        mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=out)
                    for w in ws:
                        mkq.mkq_linear_int4_stream(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=out, splitk_scratch=scr)
                torch.cuda.synchronize()
                done.append({"M": M, "K": K, "N": N, "launches_per_layout": 3 * len(ws),
                             "bytes_per_launch": M * K / 2 + N * K / 2 + 8 * N + 2 * M * N})
            del ws
    return {"only": which, "launched": done}


def layer_gemms_m1024(mkq):
    """The BERT-base layer GEMMs workload: the four linears of a BERT-base layer at M = 1024 (8 x 128 tokens), binary16
    activations in -> quantize -> int4 GEMM -> dequantize -> binary16 out, replayed as a HIP graph.  Each GEMM
    is 1.2 - 4.8 GOP: launch- and latency-bound, far from either roofline."""
    import numpy as np
    import torch
    from paper_2203_13483_amd import workloads as wl
    cfg = wl.CONFIGS[1]
    M = cfg["M"]
    rng = np.random.default_rng(cfg["seed"])
    cases = []
    for name, K, N in cfg["shapes"]:
        X = wl.outlier_activations(rng, M, K, cfg["outlier_frac"], cfg["outlier_kind"]).astype(np.float16)
        W = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
        b = rng.standard_normal(N, dtype=np.float32) * np.float32(0.01)
        cases.append(LinearCase(mkq, name, X, W, b, wl.LEARNED_STEP_UNIT_GAUSSIAN, mkq.MKQ_F16))
    total_ops = sum(c.ops for c in cases)

    def step():
        for c in cases:
            c.full()

    t = graph_time(step, rep=1, repeats=7, inner=20)
    per = {c.name: graph_time(c.gemm_only) * 1e6 for c in cases}
    return {"workload": "BERT-base layer GEMMs, M=1024: quantize + GEMM + dequantize x 4, HIP graph", "us_per_step": t * 1e6,
            "TOPS": total_ops / t / 1e12, "gemm_only_us": per,
            "gemm_only_frac_int8_peak": total_ops / (sum(per.values()) * 1e-6) / 1e12 / INT8_MFMA_PEAK_TOPS,
            "latency_bound": True}


def side_measurements(mkq, event_time, ceil):
    """Points beside the headline: large-M (MFMA-bound) GEMMs, small-M weight streaming
    (HBM-bound, cold weights), and the 12-layer encoder in int4 vs the binary16 baseline."""
    import numpy as np
    import torch
    res = {"layer_gemms_m1024": layer_gemms_m1024(mkq), "large_m": [], "small_m": [], "encoder": None}
    for (M, K, N) in LARGE_M_SHAPES:
        a = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
        w = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
        sw = torch.rand(N, device="cuda") * 0.049 + 0.001
        out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        t = graph_time(lambda: mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_BF16, out=out))
        tops = 2.0 * M * N * K / t / 1e12
        row = {"M": M, "K": K, "N": N, "out": "bf16", "us": t * 1e6, "TOPS": tops,
               "frac_int8_peak": tops / INT8_MFMA_PEAK_TOPS,
               "frac_measured_mfma_ceiling": tops / ceil["mfma_i8_TOPS"],
               "output_write_us_at_measured_write_rate": 2.0 * M * N / (ceil["hbm_write_GBps"] * 1e9) * 1e6,
               "protocol": "HIP graph of 20 back-to-back launches, median of 7 samples"}
        # rotating buffers: every launch of the graph reads another activation matrix and writes another output,
        # at least 1 GiB in all (4 x the 256 MB last-level cache), so that nothing a launch touches except the
        # weights was left in a cache by the launch before it
        pairs = max(2, min(8, -(-(1 << 30) // (M * K // 2 + 2 * M * N))))
        rot = [(a, out)] + [(torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda"),
                             torch.empty((M, N), dtype=torch.bfloat16, device="cuda")) for _ in range(pairs - 1)]

        def every_pair():
            for (ai, oi) in rot:
                mkq.mkq_linear_int4(ai, 0.01, w, sw, None, N, K, mkq.MKQ_BF16, out=oi)
        t_rot = graph_time(every_pair, rep=max(1, 20 // pairs), repeats=5) / pairs
        row["rotating_buffers_us"] = t_rot * 1e6
        row["rotating_buffers_frac_int8_peak"] = 2.0 * M * N * K / t_rot / 1e12 / INT8_MFMA_PEAK_TOPS
        row["rotating_buffers"] = f"{pairs} (activations, output) pairs cycled through by the launches of one graph"
        del rot, a, w
        if M != 16384 and (M, K, N) != (8192, 8192, 8192) and (M, K, N) != HEADLINE:
            # the comparison kernels below are timed at M = 16384 and at the headline shape only
            c8 = torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda")
            a6 = mkq.mkq_pack_codes_e3m2(c8)
            del c8
            w6 = mkq.mkq_pack_codes_e3m2(torch.randint(-8, 8, (N, K), dtype=torch.int8, device="cuda"))
            row["e3m2_route_us"] = graph_time(lambda: mkq.mkq_linear_int4_e3m2(a6, 0.01, w6, sw, None, mkq.MKQ_BF16,
                                                                               out=out), repeats=5) * 1e6
            row["e3m2_route_frac_int8_peak"] = 2.0 * M * N * K / (row["e3m2_route_us"] * 1e-6) / 1e12 / INT8_MFMA_PEAK_TOPS
            res["large_m"].append(row)
            del a6, w6, out
            continue
        # context beside it, same shape and protocol: this library's 8-bit linear (int8 codes in,
        # bf16 out) and the vendor library's int8 (int32 out) and bf16 GEMMs as torch calls them
        a8 = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
        w8 = torch.randint(-128, 128, (N, K), dtype=torch.int8, device="cuda")
        row["int8_us"] = graph_time(lambda: mkq.mkq_linear_int8(a8, 0.01, w8, sw, None, mkq.MKQ_BF16, out=out)) * 1e6
        try:
            torch._int_mm(a8, w8.t())
            row["vendor_int8_us"] = graph_time(lambda: torch._int_mm(a8, w8.t())) * 1e6
        except Exception:
            row["vendor_int8_us"] = None
        # the experimental 6-bit float route of the same 4-bit linear (E3M2 containers, exact integers)
        c8 = torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda")
        a6 = mkq.mkq_pack_codes_e3m2(c8)
        del c8
        w6 = mkq.mkq_pack_codes_e3m2(torch.randint(-8, 8, (N, K), dtype=torch.int8, device="cuda"))
        row["e3m2_route_us"] = graph_time(lambda: mkq.mkq_linear_int4_e3m2(a6, 0.01, w6, sw, None, mkq.MKQ_BF16,
                                                                           out=out)) * 1e6
        row["e3m2_route_frac_int8_peak"] = 2.0 * M * N * K / (row["e3m2_route_us"] * 1e-6) / 1e12 / INT8_MFMA_PEAK_TOPS
        del a6, w6
        a16 = torch.randn((M, K), dtype=torch.bfloat16, device="cuda")
        w16 = torch.randn((N, K), dtype=torch.bfloat16, device="cuda")
        torch.mm(a16, w16.t(), out=out)
        row["vendor_bf16_us"] = graph_time(lambda: torch.mm(a16, w16.t(), out=out)) * 1e6
        res["large_m"].append(row)
        del a8, w8, a16, w16, out

    # Few tokens: every call reads a different weight matrix from a pool of at least 1 GiB (4 x the 256 MB
    # last-level cache), so the weights always come from HBM.  Two weight layouts: canonical rows
    # (mkq_linear_int4) and the streaming layout (mkq_linear_int4_stream, with a scratch area for its K split).
    scr = mkq.mkq_splitk_scratch_init()
    for (K, N, pool, Ms) in SMALL_M_SHAPES:
        ws = [torch.randint(0, 256, (mkq.mkq_stream_weight_bytes(N, K),), dtype=torch.uint8, device="cuda")
              for _ in range(pool)]
        sw = torch.rand(N, device="cuda") * 0.049 + 0.001
        for M in Ms:
            a = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            nbytes = M * K / 2 + N * K / 2 + 8 * N + 2 * M * N
            row = {"M": M, "K": K, "N": N, "out": "f16", "weight_MiB": N * K // 2 >> 20, "algorithmic_bytes": nbytes,
                   "protocol": f"HIP graph of {pool} back-to-back calls on one stream, one distinct weight matrix each"}
            for layout in ("canonical", "stream"):
                if layout == "stream" and M > 128:
                    continue

                def sweep():
                    for w in ws:
                        if layout == "canonical":
                            mkq.mkq_linear_int4(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=out)
                        else:
                            mkq.mkq_linear_int4_stream(a, 0.01, w, sw, None, N, K, mkq.MKQ_F16, out=out, splitk_scratch=scr)

                sweep()
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    sweep()
                t = sorted(event_time(g.replay, 5, warm=1) for _ in range(5))[2] / pool
                row[layout + "_us_per_call"] = t * 1e6
                row[layout + "_GBps"] = nbytes / t / 1e9
                row[layout + "_frac_hbm_peak"] = nbytes / t / 1e9 / HBM_PEAK_GBS
                row[layout + "_frac_measured_read_ceiling"] = nbytes / t / 1e9 / ceil["hbm_read_GBps"]
                del g
            # beyond the ridge of the two rooflines (4 M operations per weight byte > 625) the matrix peak binds
            row["frac_int8_peak_best"] = (2.0 * M * N * K / (min(row.get("canonical_us_per_call", 1e30),
                                                                  row.get("stream_us_per_call", 1e30)) * 1e-6)
                                          / 1e12 / INT8_MFMA_PEAK_TOPS)
            res["small_m"].append(row)
            del a, out
        del ws

    # The same protocol for the 8-bit linear (one byte per code): few tokens take the register-streaming kernel too
    res["small_m_int8"] = []
    for (K, N, pool, Ms) in ((4096, 4096, 64, (1, 16, 64)), (8192, 8192, 16, (16,))):
        ws8 = [torch.randint(-128, 128, (N, K), dtype=torch.int8, device="cuda") for _ in range(pool)]
        sw = torch.rand(N, device="cuda") * 0.049 + 0.001
        for M in Ms:
            a8 = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
            out = torch.empty((M, N), dtype=torch.float16, device="cuda")
            nbytes = M * K + N * K + 8 * N + 2 * M * N

            def sweep8():
                for w in ws8:
                    mkq.mkq_linear_int8(a8, 0.01, w, sw, None, mkq.MKQ_F16, out=out)

            sweep8()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                sweep8()
            t = sorted(event_time(g.replay, 5, warm=1) for _ in range(5))[2] / pool
            res["small_m_int8"].append({"M": M, "K": K, "N": N, "weight_MiB": N * K >> 20, "algorithmic_bytes": nbytes,
                                        "us_per_call": t * 1e6, "GBps": nbytes / t / 1e9,
                                        "frac_hbm_peak": nbytes / t / 1e9 / HBM_PEAK_GBS})
            del g, a8, out
        del ws8

    # Scale machinery (streaming reductions, HBM-bound): one read of x per pass
    res["calibration"] = []
    M, K = CALIBRATION_SHAPE
    g = torch.empty(2, dtype=torch.float64, device="cuda")
    s1 = torch.empty(1, dtype=torch.float32, device="cuda")
    wsp = torch.empty(mkq.mkq_percentile_scale_workspace_bytes(), dtype=torch.uint8, device="cuda")
    for dt, nb in ((torch.float16, 2), (torch.float32, 4)):
        x = torch.randn((M, K), dtype=dt, device="cuda")
        t = graph_time(lambda: mkq.mkq_scale_gradients(x, 0.34, 4, g_out=g), rep=5, repeats=5)
        res["calibration"].append({"op": "scale_gradients", "M": M, "K": K, "x_bytes": nb, "us": t * 1e6,
                                   "GBps": nb * M * K / t / 1e9, "frac_hbm_peak": nb * M * K / t / 1e9 / HBM_PEAK_GBS})
        t = graph_time(lambda: mkq.mkq_percentile_scale(x, 100, 4, s_out=s1, workspace=wsp), rep=5, repeats=5)
        res["calibration"].append({"op": "percentile_scale (radix select, 3 counting passes over x)", "M": M, "K": K,
                                   "x_bytes": nb, "us": t * 1e6,
                                   "GBps": nb * M * K / t / 1e9, "frac_hbm_peak": nb * M * K / t / 1e9 / HBM_PEAK_GBS,
                                   "note": "algorithmic bytes = one read of x; the kernel reads it three times "
                                           f"({3 * nb * M * K / t / 1e9:.0f} GB/s of actual traffic)"})
        del x

    # The token counts of the paper's Table 2 (padding-free batches of 16 and 64 sentences): the four
    # GEMMs of one BERT-base layer at exactly M valid tokens, binary16 out, in 4 bits, 8 bits and binary16
    res["table2_token_counts"] = []
    H, F = 768, 3072
    for M in (440, 537, 681, 1691, 2011, 2298):
        row = {"M": M, "int4_us": 0.0, "int8_us": 0.0, "fp16_us": 0.0, "vendor_fp16_us": 0.0}
        for (K, N) in ((H, 3 * H), (H, H), (H, F), (F, H)):
            o16 = torch.empty((M, N), dtype=torch.float16, device="cuda")
            sw = torch.rand(N, device="cuda") * 0.049 + 0.001
            b32 = torch.zeros(N, device="cuda")
            a4 = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
            w4 = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
            row["int4_us"] += graph_time(lambda: mkq.mkq_linear_int4(a4, 0.01, w4, sw, b32, N, K, mkq.MKQ_F16, out=o16),
                                         repeats=5) * 1e6
            a8 = torch.randint(-128, 128, (M, K), dtype=torch.int8, device="cuda")
            w8 = torch.randint(-128, 128, (N, K), dtype=torch.int8, device="cuda")
            row["int8_us"] += graph_time(lambda: mkq.mkq_linear_int8(a8, 0.01, w8, sw, b32, mkq.MKQ_F16, out=o16),
                                         repeats=5) * 1e6
            a16 = torch.randn(M, K, device="cuda", dtype=torch.float16)
            w16 = torch.randn(N, K, device="cuda", dtype=torch.float16) * 0.02
            row["fp16_us"] += graph_time(lambda: mkq.mkq_linear_fp16(a16, w16, b32, mkq.MKQ_F16, out=o16),
                                         repeats=5) * 1e6
            b16 = b32.half()
            torch.nn.functional.linear(a16, w16, b16)
            row["vendor_fp16_us"] += graph_time(lambda: torch.nn.functional.linear(a16, w16, b16), repeats=5) * 1e6
        row["int8_over_int4"] = row["int8_us"] / row["int4_us"]
        row["fp16_over_int4"] = row["fp16_us"] / row["int4_us"]
        row["vendor_fp16_over_int4"] = row["vendor_fp16_us"] / row["int4_us"]
        res["table2_token_counts"].append(row)

    # The BERT-large layer GEMMs workload: the four GEMMs of a BERT-large layer at M = 8192 (batch 16 x seq 512), int4 codes
    # in, fused re-quantization to int4 codes out (GELU on FFN-up)
    res["bert_large_gemms_int4_chain"] = []
    M = 8192
    for (name, K, N, act) in (("qkv", 1024, 3072, mkq.MKQ_ACT_NONE), ("attn_out", 1024, 1024, mkq.MKQ_ACT_NONE),
                              ("ffn_up_gelu", 1024, 4096, mkq.MKQ_ACT_GELU), ("ffn_down", 4096, 1024, mkq.MKQ_ACT_NONE)):
        a4 = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
        w4 = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
        sw = torch.rand(N, device="cuda") * 0.049 + 0.001
        b32 = torch.randn(N, device="cuda") * 0.01
        o4 = torch.empty((M, N // 2), dtype=torch.uint8, device="cuda")
        t = graph_time(lambda: mkq.mkq_linear_int4(a4, 0.01, w4, sw, b32, N, K, mkq.MKQ_I4, act=act, s_next=0.3,
                                                   out=o4), repeats=5)
        res["bert_large_gemms_int4_chain"].append({"linear": name, "M": M, "K": K, "N": N, "us": t * 1e6,
                                                    "TOPS": 2.0 * M * N * K / t / 1e12,
                                                    "frac_int8_peak": 2.0 * M * N * K / t / 1e12 / INT8_MFMA_PEAK_TOPS})
        del a4, w4, o4

    # The four linears of a layer of the paper's 4-layer student (hidden 312, FFN 1200: K is not a
    # multiple of 32, operands are stored padded with zero codes to a multiple of 128), float activations in: quantize + GEMM
    res["tinybert4_linears"] = []
    H, F = 312, 1200
    for M in (440, 2298, 4096):
        row = {"M": M, "int4_us": 0.0, "vendor_fp16_us": 0.0}
        for (K, N) in ((H, 3 * H), (H, H), (H, F), (F, H)):
            x16 = torch.randn(M, K, device="cuda", dtype=torch.float16)
            w32 = torch.randn(N, K, device="cuda") * 0.02
            b32 = torch.zeros(N, device="cuda")
            w4, sw = mkq.mkq_pack_weights_int4_padded(w32)
            Kp = mkq.mkq_padded_k(K)
            a4 = torch.empty((M, Kp // 2), dtype=torch.uint8, device="cuda")
            o16 = torch.empty((M, N), dtype=torch.float16, device="cuda")

            def lin():
                mkq.mkq_quantize_padded(x16, 0.34, q_out=a4)
                mkq.mkq_linear_int4(a4, 0.34, w4, sw, b32, N, Kp, mkq.MKQ_F16, out=o16)

            row["int4_us"] += graph_time(lin, repeats=5) * 1e6
            w16, b16 = w32.half(), b32.half()
            torch.nn.functional.linear(x16, w16, b16)
            row["vendor_fp16_us"] += graph_time(lambda: torch.nn.functional.linear(x16, w16, b16), repeats=5) * 1e6
        row["vendor_fp16_over_int4"] = row["vendor_fp16_us"] / row["int4_us"]
        res["tinybert4_linears"].append(row)

    # One BERT-base layer on padding-free batches with the batch sizes and valid-token counts of the
    # paper's Table 2 (seeded sequence lengths <= 128), in 4 bits, 8 bits and binary16
    try:
        res["table2_layers"] = table2_layers(mkq)
    except Exception as e:
        res["table2_layers"] = {"error": repr(e)}

    # Whole layers beyond BERT-base at 128 tokens: the 4-layer student (head size 26, padded code rows) and a
    # BERT-large layer on 512-token sequences (key-block attention kernel)
    try:
        res["layers_other_shapes"] = layers_other_shapes(mkq)
    except Exception as e:
        res["layers_other_shapes"] = {"error": repr(e)}

    # 12-layer BERT-base encoder, batch 32 x seq 128 (M = 4096), int4 vs binary16 layers
    try:
        res["encoder"] = encoder_latency(mkq, event_time)
    except Exception as e:  # keep the headline line even if this side measurement fails
        res["encoder"] = {"error": repr(e)}
    return res


def table2_layers(mkq):
    import numpy as np
    import torch
    from paper_2203_13483_amd import workloads as wl
    H, heads, F = 768, 12, 3072
    p = wl.bert_layer_weights(H, heads, F, 300)
    ln = {k: torch.from_numpy(p[k]).cuda() for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
    packed4, packed8, w16 = {}, {}, {}
    for nm in ("qkv", "ao", "up", "down"):
        W = torch.from_numpy(p["W_" + nm]).cuda()
        b = torch.from_numpy(p["b_" + nm]).cuda()
        packed4[nm] = mkq.mkq_pack_weights_int4(W) + (b,)
        packed8[nm] = mkq.mkq_pack_weights_int8(W) + (b,)
        w16[nm] = (W.half(), b)
    sx4 = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
    sx8 = {k: v * 7.0 / 127.0 for k, v in sx4.items()}
    rows = []
    for (batch, tokens, t4_f32, t4_i8, t4_i4) in wl.TABLE2_ROWS:
        lens = wl.ragged_lengths(tokens, batch, 128, seed=tokens)
        cu = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
        h = torch.randn((tokens, H), dtype=torch.float16, device="cuda")
        out = torch.empty_like(h)
        layers = {
            "int4": mkq.BertLayerInt4(batch, 128, H, heads, F, packed4, sx4, ln, 1e-12, cu_seqlens=cu, total_tokens=tokens),
            "int8": mkq.BertLayerInt8(batch, 128, H, heads, F, packed8, sx8, ln, 1e-12, cu_seqlens=cu, total_tokens=tokens),
            "fp16": mkq.BertLayerFp16(batch, 128, H, heads, F, w16, ln, 1e-12, cu_seqlens=cu, total_tokens=tokens),
        }
        row = {"batch": batch, "valid_tokens": tokens}
        for name, layer in layers.items():
            ws = torch.empty(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
            row[name + "_us"] = graph_time(lambda: layer(h, ws, h_out=out), rep=10, repeats=5) * 1e6
        row["int8_over_int4"] = row["int8_us"] / row["int4_us"]
        row["fp16_over_int4"] = row["fp16_us"] / row["int4_us"]
        row["paper_T4_us"] = {"float32": t4_f32, "int8": t4_i8, "int4": t4_i4, "int8_over_int4": t4_i8 / t4_i4}
        rows.append(row)
    return rows


def layers_other_shapes(mkq):
    import torch
    from paper_2203_13483_amd import workloads as wl
    rows = []
    for (name, batch, seq, H, heads, F) in (("student_4layer", 32, 128, 312, 12, 1200),
                                            ("bert_large_seq512", 16, 512, 1024, 16, 4096)):
        p = wl.bert_layer_weights(H, heads, F, 301)
        ln = {k: torch.from_numpy(p[k]).cuda() for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
        padded = H % 32 != 0
        packed4, packed8, w16 = {}, {}, {}
        for nm in ("qkv", "ao", "up", "down"):
            W = torch.from_numpy(p["W_" + nm]).cuda()
            b = torch.from_numpy(p["b_" + nm]).cuda()
            packed4[nm] = (mkq.mkq_pack_weights_int4_padded if padded else mkq.mkq_pack_weights_int4)(W) + (b,)
            if not padded:
                packed8[nm] = mkq.mkq_pack_weights_int8(W) + (b,)
                w16[nm] = (W.half(), b)
        sx4 = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
        sx8 = {k: v * 7.0 / 127.0 for k, v in sx4.items()}
        M = batch * seq
        h = torch.randn((M, H), dtype=torch.float16, device="cuda")
        out = torch.empty_like(h)
        layers = {"int4": mkq.BertLayerInt4(batch, seq, H, heads, F, packed4, sx4, ln, 1e-12)}
        if not padded:  # the 8-bit and binary16 layers take hidden % 64 == 0 only
            layers["int8"] = mkq.BertLayerInt8(batch, seq, H, heads, F, packed8, sx8, ln, 1e-12)
            layers["fp16"] = mkq.BertLayerFp16(batch, seq, H, heads, F, w16, ln, 1e-12)
        row = {"layer": name, "batch": batch, "seq": seq, "hidden": H, "heads": heads, "ffn": F}
        for kind, layer in layers.items():
            ws = torch.empty(layer.workspace_bytes(), dtype=torch.uint8, device="cuda")
            row[kind + "_us"] = graph_time(lambda: layer(h, ws, h_out=out), rep=10, repeats=5) * 1e6
        qkv = torch.randn((M, 3 * H), dtype=torch.float16, device="cuda")
        row["attention_core_us"] = graph_time(lambda: mkq.mkq_attention(qkv, batch, seq, H, heads, s_next=0.05,
                                                                        want_ctx=False, want_q=True), rep=10, repeats=5) * 1e6
        # q k^T and p v: 4 * seq * d_k operations per (query, head)
        row["attention_core_TFLOPs"] = 4.0 * batch * heads * seq * seq * (H // heads) / (row["attention_core_us"] * 1e-6) / 1e12
        rows.append(row)
    return rows


def encoder_latency(mkq, event_time, layers=12, batch=32, seq=128):
    import numpy as np
    import torch
    from paper_2203_13483_amd import workloads as wl
    H, heads, F = 768, 12, 3072
    M = batch * seq
    h = torch.from_numpy(wl.hidden_states(batch, seq, H, 2).astype(np.float16)).cuda()
    int4_layers, fp16_layers, int8_layers = [], [], []
    for l in range(layers):
        p = wl.bert_layer_weights(H, heads, F, 100 + l)
        ln = {k: torch.from_numpy(p[k]).cuda() for k in ("ln1_gamma", "ln1_beta", "ln2_gamma", "ln2_beta")}
        packed, w16, packed8 = {}, {}, {}
        for nm in ("qkv", "ao", "up", "down"):
            W = torch.from_numpy(p["W_" + nm]).cuda()
            b = torch.from_numpy(p["b_" + nm]).cuda()
            Wq, s_w = mkq.mkq_pack_weights_int4(W)
            packed[nm] = (Wq, s_w, b)
            w16[nm] = (W.half(), b)
            packed8[nm] = mkq.mkq_pack_weights_int8(W) + (b,)
        # stand-ins for learned steps: ~unit-variance LayerNorm outputs, small context / GELU outputs
        sx = {"qkv": wl.LEARNED_STEP_UNIT_GAUSSIAN, "ao": 0.05, "up": wl.LEARNED_STEP_UNIT_GAUSSIAN, "down": 0.05}
        int4_layers.append(mkq.BertLayerInt4(batch, seq, H, heads, F, packed, sx, ln, 1e-12,
                                             s_out_next=wl.LEARNED_STEP_UNIT_GAUSSIAN))
        fp16_layers.append(mkq.BertLayerFp16(batch, seq, H, heads, F, w16, ln, 1e-12))
        # the same layer W8A8 (8-bit layers of a mixed model): the same clipping points, 127 / 7 finer steps
        sx8 = {k: v * 7.0 / 127.0 for k, v in sx.items()}
        int8_layers.append(mkq.BertLayerInt8(batch, seq, H, heads, F, packed8, sx8, ln, 1e-12,
                                             s_out_next=wl.LEARNED_STEP_UNIT_GAUSSIAN * 7.0 / 127.0))
    ws4 = torch.empty(int4_layers[0].workspace_bytes(), dtype=torch.uint8, device="cuda")
    ws8 = torch.empty(int8_layers[0].workspace_bytes(), dtype=torch.uint8, device="cuda")
    q8bufs = [torch.empty((M, H), dtype=torch.int8, device="cuda") for _ in range(2)]
    ws16 = torch.empty(fp16_layers[0].workspace_bytes(), dtype=torch.uint8, device="cuda")
    bufs = [torch.empty((M, H), dtype=torch.float16, device="cuda") for _ in range(2)]
    qbufs = [torch.empty((M, H // 2), dtype=torch.uint8, device="cuda") for _ in range(2)]

    def run_int4():
        x, q = h, None
        for i, layer in enumerate(int4_layers):
            layer(x, ws4, h_out=bufs[i & 1], q_in=q, q_out_next=qbufs[i & 1])
            x, q = bufs[i & 1], qbufs[i & 1]

    def run_int8():
        x, q = h, None
        for i, layer in enumerate(int8_layers):
            layer(x, ws8, h_out=bufs[i & 1], q_in=q, q_out_next=q8bufs[i & 1])
            x, q = bufs[i & 1], q8bufs[i & 1]

    def run_fp16():
        x = h
        for i, layer in enumerate(fp16_layers):
            layer(x, ws16, h_out=bufs[i & 1])
            x = bufs[i & 1]

    # a mixed model (section 4.2: later layers 4-bit, the rest 8-bit): first half W8A8, second half W4A4;
    # the layer at the seam writes its output codes at the width of the next
    half = layers // 2
    mixed_layers = []
    for l in range(layers):
        src = int8_layers[l] if l < half else int4_layers[l]
        cls = mkq.BertLayerInt8 if l < half else mkq.BertLayerInt4
        nb = 4 if l + 1 >= half else 8
        s_next = wl.LEARNED_STEP_UNIT_GAUSSIAN * (1.0 if nb == 4 else 7.0 / 127.0)
        packed_l, ln_l = src._keep[:2]
        sx_l = {nm: getattr(src.params, "sx_" + nm) for nm in ("qkv", "ao", "up", "down")}
        mixed_layers.append((cls(batch, seq, H, heads, F, packed_l, sx_l, ln_l, 1e-12, s_out_next=s_next, next_bits=nb),
                             nb))

    def run_mixed():
        x, q = h, None
        for i, (layer, nb) in enumerate(mixed_layers):
            qo = q8bufs[i & 1] if nb == 8 else qbufs[i & 1]
            layer(x, ws8, h_out=bufs[i & 1], q_in=q, q_out_next=qo)
            x, q = bufs[i & 1], qo

    out = {"layers": layers, "batch": batch, "seq": seq, "hidden": H, "ffn": F}
    for name, fn in (("int4", run_int4), ("fp16", run_fp16), ("int8", run_int8), ("mixed_6x8bit_6x4bit", run_mixed)):
        fn()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        t = event_time(g.replay, 20)
        out[name + "_us_per_layer"] = t * 1e6 / layers
    out["int4_vs_fp16_speedup"] = out["fp16_us_per_layer"] / out["int4_us_per_layer"]
    out["int4_vs_int8_speedup"] = out["int8_us_per_layer"] / out["int4_us_per_layer"]
    # context for the binary16 baseline's own quality: the layer's four GEMMs alone, this library's
    # binary16 kernel vs the vendor library's (torch.nn.functional.linear = hipBLASLt) vs the int4 path
    try:
        gem = {"ours_fp16_us": 0.0, "vendor_fp16_us": 0.0, "int4_us": 0.0}
        for (K, N) in ((H, 3 * H), (H, H), (H, F), (F, H)):
            a16 = torch.randn(M, K, device="cuda", dtype=torch.float16)
            w16 = torch.randn(N, K, device="cuda", dtype=torch.float16) * 0.02
            b32 = torch.zeros(N, device="cuda")
            o16 = torch.empty((M, N), dtype=torch.float16, device="cuda")
            gem["ours_fp16_us"] += graph_time(lambda: mkq.mkq_linear_fp16(a16, w16, b32, mkq.MKQ_F16, out=o16)) * 1e6
            gem["vendor_fp16_us"] += graph_time(lambda: torch.nn.functional.linear(a16, w16, out=None)) * 1e6
            a4 = torch.randint(0, 256, (M, K // 2), dtype=torch.uint8, device="cuda")
            w4 = torch.randint(0, 256, (N * K // 2,), dtype=torch.uint8, device="cuda")
            sw = torch.rand(N, device="cuda") * 0.049 + 0.001
            gem["int4_us"] += graph_time(lambda: mkq.mkq_linear_int4(a4, 0.01, w4, sw, b32, N, K, mkq.MKQ_F16, out=o16)) * 1e6
        out["layer_gemms_only_us"] = gem
    except Exception as e:
        out["layer_gemms_only_us"] = {"error": repr(e)}
    gemm_ops = 2.0 * M * (H * 3 * H + H * H + 2 * H * F)
    out["int4_layer_gemm_TOPS"] = gemm_ops / (out["int4_us_per_layer"] * 1e-6) / 1e12
    out["paper_context"] = ("paper: int4 layer 8.6-14.9x faster than float32 and 1.26-1.37x faster than int8 "
                            "on NVIDIA T4 (Table 2); different hardware and baseline precision")
    return out


if __name__ == "__main__":
    main()
