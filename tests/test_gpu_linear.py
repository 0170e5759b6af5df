"""GPU parity: the W4A4 linear (int4 GEMM + dequantize epilogue + requantization)
vs the CPU oracle.  Integer results bit-exact, floats within 1e-3 (binary32 out)
or 1e-2 (16-bit out) by the rule |gpu-ref| <= rtol*|ref| + rtol*rms(ref)."""
import numpy as np
import pytest

import oracle
from paper_2203_13483_amd import workloads as wl
from helpers import RTOL, assert_codes_match_with_tie_band, assert_float_close, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mkq():
    import torch
    assert torch.cuda.is_available()
    import paper_2203_13483_amd as m
    m.load()
    return m


def _codes_case(M, N, K, seed):
    A, Wc, s_w, s_x = wl.uniform_codes_linear(M, K, N, seed)
    rng = np.random.default_rng(seed + 1000)
    bias = rng.normal(0, 0.5, N).astype(np.float32)
    return A, Wc, s_w, s_x, bias


def _run(mkq, A, Wc, s_w, s_x, bias, out_dtype, **kw):
    M, K = A.shape
    N = Wc.shape[0]
    a_d = mkq.mkq_pack_codes_int4(to_dev(A))
    w_d = mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1)
    return mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), None if bias is None else to_dev(bias), N, K,
                               out_dtype, **kw)


SHAPES = [(128, 768, 768), (1, 32, 32), (16, 16, 64), (200, 328, 800), (257, 130, 96),
          (64, 2304, 768), (1024, 768, 3072), (300, 300, 2048), (129, 257, 160)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_accumulators_and_f32_output(mkq, M, N, K):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M + N + K)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F32, want_acc=True)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert_float_close(to_np(r["out"]), ref["y"], RTOL[0], "f32 out")
    # every op of the epilogue is a correctly rounded binary32 op on both sides
    assert np.array_equal(to_np(r["out"]), ref["y"])


@pytest.mark.parametrize("K", [64, 768, 4096, 8192])
def test_accumulator_extremes(mkq, K):
    M, N = 48, 80
    lo = np.full((M, K), -8, np.int8)
    hi = np.full((N, K), 7, np.int8)
    ones = np.ones(N, np.float32)
    r = _run(mkq, lo, np.full((N, K), -8, np.int8), ones, 1.0, None, mkq.MKQ_F32, want_acc=True)
    assert np.all(to_np(r["acc"]) == 64 * K)
    assert np.all(to_np(r["out"]) == 64.0 * K)
    r = _run(mkq, lo, hi, ones, 1.0, None, mkq.MKQ_F32, want_acc=True)
    assert np.all(to_np(r["acc"]) == -56 * K)


@pytest.mark.parametrize("out_dtype", [1, 2])
@pytest.mark.parametrize("M,N,K", [(128, 768, 768), (200, 328, 800), (77, 100, 96)])
def test_narrow_outputs(mkq, M, N, K, out_dtype):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=out_dtype + M)
    r = _run(mkq, A, Wc, s_w, s_x, bias, out_dtype)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=out_dtype)
    got = to_np(r["out"]).astype(np.float32)
    assert_float_close(got, ref["y"], RTOL[out_dtype], "narrow out")
    assert np.array_equal(got, ref["y"])  # RNE narrowing of identical binary32 values


@pytest.mark.parametrize("res_dtype", ["f32", "f16"])
def test_residual_and_requant_without_gelu_is_bit_exact(mkq, res_dtype):
    import torch
    M, N, K = 200, 328, 800
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=5)
    rng = np.random.default_rng(6)
    res = rng.normal(0, 1, (M, N)).astype(np.float32)
    if res_dtype == "f16":
        res = res.astype(np.float16).astype(np.float32)
    res_d = to_dev(res, torch.float16 if res_dtype == "f16" else None)
    ref32 = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res)
    s_next = float(np.float32(np.abs(ref32["y"]).max() / 20))
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res, out_dtype=oracle.F16, s_next=s_next)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, residual=res_d, s_next=s_next, want_q=True)
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(ref["q"]))
    assert ref["q"].min() == -8 and ref["q"].max() == 7  # the clamp is exercised
    r4 = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_I4, residual=res_d, s_next=s_next)
    assert np.array_equal(to_np(r4["out"]), oracle.pack_nibbles(ref["q"]))


# code outputs with a row pitch: the next linear's reduction length is padded (312 -> 384, 1200 -> 1280 codes)
@pytest.mark.parametrize("M,N,K,pitch", [(100, 312, 384, 384), (1, 1200, 384, 1280), (300, 1200, 128, 1280),
                                         (40, 312, 1280, 320), (700, 768, 256, 768)])
def test_code_outputs_with_a_row_pitch(mkq, M, N, K, pitch):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M + pitch)
    ref32 = oracle.linear_int4(A, s_x, Wc, s_w, bias)
    s_next = float(np.float32(np.abs(ref32["y"]).max() / 20))
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.F16, s_next=s_next)
    want = np.zeros((M, pitch), np.int8)
    want[:, :N] = ref["q"]
    import torch
    stale = lambda: torch.full((M, pitch // 2), 0x5A, dtype=torch.uint8, device="cuda")  # the padding must be written
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, s_next=s_next, q_out=stale(), q_pitch=pitch)
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(want))
    r4 = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_I4, s_next=s_next, out=stale(), q_pitch=pitch)
    assert np.array_equal(to_np(r4["out"]), oracle.pack_nibbles(want))
    with pytest.raises(mkq.MkqError):
        _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_I4, s_next=s_next, q_pitch=N - 8)


@pytest.mark.parametrize("M,N,K", [(128, 3072, 768), (130, 202, 96)])
def test_gelu_then_requant(mkq, M, N, K):
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=9)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU)
    s_next = float(np.float32(np.abs(ref["y"]).max() / 12))
    refq = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU, s_next=s_next)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F32, act=mkq.MKQ_ACT_GELU, s_next=s_next, want_q=True)
    assert_float_close(to_np(r["out"]), ref["y"], RTOL[0], "gelu out")
    got_codes = oracle.unpack_nibbles(to_np(r["q"]), N)
    assert_codes_match_with_tie_band(got_codes, refq["q"], ref["y"], s_next, what="gelu requant")


def test_config1_single_linear_float_input(mkq):
    # The single-linear workload (configs[0]): X [128,768] ~N(0,1), s_x = max|X|/7, W ~N(0,0.02) per-channel abs-max, seed 0
    X, W, b = wl.gaussian_linear(128, 768, 768, seed=0)
    s_x = oracle.absmax_scale(X)
    wc, s_w_ref = oracle.quantize_weights(W)
    ref = oracle.linear_int4(oracle.quantize(X, s_x), s_x, wc, s_w_ref, b)
    Wq, s_w = mkq.mkq_pack_weights_int4(to_dev(W))
    s_x_gpu = float(to_np(mkq.mkq_absmax_scale(to_dev(X)))[0])
    assert np.float32(s_x_gpu) == np.float32(s_x)
    r = mkq.mkq_linear_int4(to_dev(X), s_x_gpu, Wq, s_w, to_dev(b), 768, 768, mkq.MKQ_F32, want_acc=True)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert_float_close(to_np(r["out"]), ref["y"], RTOL[0], "config 1")
    assert np.abs(ref["acc"]).max() <= 64 * 768


def test_half_precision_float_input_and_empty_batch(mkq):
    import torch
    X, W, b = wl.outlier_linear(96, 256, 64, seed=3)
    Xh = X.astype(np.float16)
    s_x = wl.LEARNED_STEP_UNIT_GAUSSIAN
    wc, s_w = oracle.quantize_weights(W)
    ref = oracle.linear_int4(oracle.quantize(Xh.astype(np.float32), s_x), s_x, wc, s_w, b, out_dtype=oracle.F16)
    Wq, s_wd = mkq.mkq_pack_weights_int4(to_dev(W))
    r = mkq.mkq_linear_int4(to_dev(Xh), s_x, Wq, s_wd, to_dev(b), 64, 256, mkq.MKQ_F16, want_acc=True)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    empty = torch.empty((0, 128), dtype=torch.uint8, device="cuda")
    r = mkq.mkq_linear_int4(empty, s_x, Wq, s_wd, to_dev(b), 64, 256, mkq.MKQ_F32)
    assert r["out"].shape == (0, 64)


def test_deterministic_and_no_out_of_bounds_writes(mkq):
    import torch
    M, N, K = 200, 328, 800
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=21)
    a_d = mkq.mkq_pack_codes_int4(to_dev(A))
    w_d = mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1)
    guard = 4096
    buf = torch.full((M * N + 2 * guard,), 1234.5, dtype=torch.float32, device="cuda")
    out = buf[guard: guard + M * N].view(M, N)
    r1 = mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), to_dev(bias), N, K, mkq.MKQ_F32, out=out)
    first = to_np(r1["out"]).copy()
    assert torch.all(buf[:guard] == 1234.5) and torch.all(buf[guard + M * N:] == 1234.5)
    r2 = mkq.mkq_linear_int4(a_d, s_x, w_d, to_dev(s_w), to_dev(bias), N, K, mkq.MKQ_F32)
    assert np.array_equal(first, to_np(r2["out"]))


ALL_CFGS = [2, 3, 11, 12, 14, 18, 19, 20, 27, 28, 29, 31, 33, 35]
K_GROUPS = {31: 2, 33: 2, 35: 2}  # configurations that split the k loop between wave groups


@pytest.mark.parametrize("cfg", ALL_CFGS)
@pytest.mark.parametrize("M,N,K", [(300, 520, 1024), (257, 130, 96), (512, 256, 2048), (1500, 1100, 384)])
def test_every_tile_configuration(mkq, cfg, M, N, K):
    if cfg >= 10 and K % 128:
        pytest.skip("direct-to-LDS configurations need whole 64-byte k stages")
    if cfg in K_GROUPS and K % (128 * K_GROUPS[cfg]):
        pytest.skip("the k split needs a whole number of stages per wave group")
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=cfg + M)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.BF16, s_next=0.7)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_BF16, want_acc=True, want_q=True, s_next=0.7, config=cfg)
    acc, out, q = to_np(r["acc"]), to_np(r["out"]), to_np(r["q"])
    assert np.array_equal(acc, ref["acc"])
    assert np.array_equal(out.astype(np.float32), ref["y"])
    assert np.array_equal(q, oracle.pack_nibbles(ref["q"]))


@pytest.mark.parametrize("cfg", [c for c in ALL_CFGS if c >= 10])
@pytest.mark.parametrize("K", [128, 640])
def test_single_stage_tiles_and_f16_residual(mkq, cfg, K):
    """K = 128 is one ring stage per tile (the shortest pipeline); with a binary16 residual
    and binary16 output the compile-time residual epilogue runs."""
    import torch
    K *= K_GROUPS.get(cfg, 1)  # one and five stages per wave group
    M, N = 2100, 1160
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=cfg + K)
    res = np.random.default_rng(K).normal(0, 1, (M, N)).astype(np.float16)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res.astype(np.float32), out_dtype=oracle.F16)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, residual=to_dev(res), config=cfg)
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])


@pytest.mark.parametrize("cfg", [c for c in ALL_CFGS if c >= 10])
@pytest.mark.parametrize("out_name", ["bf16", "i4"])
def test_persistent_pipeline_over_many_tiles(mkq, cfg, out_name):
    """More tiles than resident workgroups, ragged edges, the compile-time epilogues:
    the ring pipeline carries on across tiles and epilogue stores stay in flight."""
    M, N, K = 8200, 2312, 128 * max(2, K_GROUPS.get(cfg, 1))
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=cfg)
    if out_name == "bf16":
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.BF16)
    else:
        ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, s_next=0.9)
    if out_name == "bf16":
        r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_BF16, config=cfg)
        assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    else:
        r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_I4, s_next=0.9, config=cfg)
        assert np.array_equal(to_np(r["out"]), oracle.pack_nibbles(ref["q"]))


@pytest.mark.parametrize("M", [1, 16, 33, 64, 100, 128])
@pytest.mark.parametrize("N,K", [(200, 256), (40, 512), (768, 768), (328, 4096), (96, 2304), (72, 8192), (40, 10240)])
def test_few_token_register_path(mkq, M, N, K):
    """Configuration 30: the first few-token kernel (K split over 8 waves, reduced in LDS)."""
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M * 7 + N)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.F16, s_next=0.8)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, want_acc=True, want_q=True, s_next=0.8, config=30)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(ref["q"]))


@pytest.fixture(scope="module")
def scratch(mkq):
    return mkq.mkq_splitk_scratch_init()


# k_slices: 0 = the library's choice, 1 = no split, others forced (clamped to K / 256)
@pytest.mark.parametrize("k_slices", [0, 1, 2, 3, 5, 16])
@pytest.mark.parametrize("M", [1, 16, 33, 64, 65, 100, 128])
@pytest.mark.parametrize("N,K", [(200, 256), (40, 512), (768, 768), (328, 4096), (130, 2304), (72, 8192),
                                 (1100, 1280), (4096, 2048)])
def test_few_token_streaming_path(mkq, scratch, M, N, K, k_slices):
    """M <= 128 takes the weight-streaming kernel: 128-channel workgroups (N not a multiple of 128, of 32,
    of 8), K slices across workgroups with remainders (K / 256 not a multiple of the slice count), the
    last-ticket reduction, and the counters left clear for the next call (every case shares one area)."""
    if K % 256:
        pytest.skip("the streaming kernel needs whole 128-byte row groups")
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M * 7 + N)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.F16, s_next=0.8)
    r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, want_acc=True, want_q=True, s_next=0.8,
             splitk_scratch=scratch, config=50, k_slices=k_slices)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(ref["q"]))
    import torch
    assert int(scratch[:16384].view(torch.int32).abs().sum()) == 0, "ticket counters not cleared"


def test_few_token_default_route_and_no_scratch(mkq, scratch):
    """The library's own route for M <= 128 with and without a scratch area gives identical bits."""
    M, N, K = 48, 1000, 4096
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=5)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.BF16)
    r0 = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_BF16, want_acc=True)
    r1 = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_BF16, want_acc=True, splitk_scratch=scratch)
    for r in (r0, r1):
        assert np.array_equal(to_np(r["acc"]), ref["acc"])
        assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])


def _stream_layout(packed, N, K):
    """The streaming layout written out from its definition in the header: piece l of block g * pitch + q
    is bytes [32 g + 16 (l // 32), + 16) of the canonical row of channel 32 q + r(l % 32); pitch = the number
    of panels made odd."""
    rows = packed.reshape(N, K // 2)
    panels = (N + 31) // 32
    out = np.zeros((K // 64, panels | 1, 64, 16), np.uint8)
    for l in range(64):
        i = l % 32
        r = 16 * (i // 16) + 8 * ((i // 4) % 2) + 4 * ((i // 8) % 2) + i % 4
        for q in range(panels):
            n = 32 * q + r
            if n < N:
                out[:, q, l, :] = rows[n].reshape(K // 64, 2, 16)[:, l // 32, :]
    return out.reshape(-1)


@pytest.mark.parametrize("N,K", [(32, 64), (64, 64), (100, 256), (130, 1280), (768, 768 + 256)])
def test_stream_layout_repack(mkq, N, K):
    rng = np.random.default_rng(N + K)
    packed = rng.integers(0, 256, N * K // 2, dtype=np.uint8)
    got = to_np(mkq.mkq_repack_weights_int4_stream(to_dev(packed), N, K))
    assert got.size == mkq.mkq_stream_weight_bytes(N, K) == (((N + 31) // 32) | 1) * 32 * K // 2
    assert np.array_equal(got, _stream_layout(packed, N, K))


@pytest.mark.parametrize("prefetch,k_slices", [(0, 0), (2, 1), (3, 2), (4, 3), (6, 5), (4, 16)])
@pytest.mark.parametrize("M", [1, 16, 33, 64, 65, 100, 128])
@pytest.mark.parametrize("N,K", [(200, 256), (40, 512), (768, 768), (328, 4096), (130, 2304), (72, 8192),
                                 (1100, 1280), (4096, 2048)])
def test_few_token_linear_on_streaming_layout(mkq, scratch, M, N, K, prefetch, k_slices):
    """mkq_linear_int4_stream: same bits as the oracle's linear on the canonical codes, for every prefetch
    depth, with and without K slices across workgroups, ragged N (partial panels, partial 128-channel tiles)."""
    if K % 256:
        pytest.skip("the streaming kernel needs whole 128-byte row groups")
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M * 5 + N)
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.F16, s_next=0.8)
    a_d = mkq.mkq_pack_codes_int4(to_dev(A))
    w_s = mkq.mkq_repack_weights_int4_stream(mkq.mkq_pack_codes_int4(to_dev(Wc)).reshape(-1), N, K)
    r = mkq.mkq_linear_int4_stream(a_d, s_x, w_s, to_dev(s_w), to_dev(bias), N, K, mkq.MKQ_F16, want_acc=True,
                                   want_q=True, s_next=0.8, splitk_scratch=scratch, prefetch_stages=prefetch,
                                   k_slices=k_slices)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(ref["q"]))


def test_init_and_ceiling_probes(mkq):
    """mkq_init (all once-per-device set-up ahead of the first call) and the probes behind the benchmark's
    measured ceilings: they run, move the bytes they say they move, and report whole MFMA instructions."""
    import torch
    lib = mkq.load()
    assert lib.mkq_init() == mkq.MKQ_OK and lib.mkq_init() == mkq.MKQ_OK
    n = 1 << 20
    src = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
    mkq.mkq_measure_stream(2, src, dst, n)
    assert torch.equal(src, dst)
    mkq.mkq_measure_stream(0, src, dst, n)       # a read leaves both alone
    assert torch.equal(src, dst)
    mkq.mkq_measure_stream(1, None, dst, n - 4096)
    assert torch.equal(src[n - 4096:], dst[n - 4096:]) and not torch.equal(src[:n - 4096], dst[:n - 4096])
    need = lib.mkq_measure_mfma_i8_operand_bytes()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert need == cus * 2 * 256 * 6 * 16
    ops = torch.randint(0, 256, (need,), dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    done = mkq.mkq_measure_mfma_i8(ops, 16, sink)
    torch.cuda.synchronize()
    assert done == cus * 8 * 16 * 8 * 2 * 32 * 32 * 32
    with pytest.raises(mkq.MkqError):
        mkq.mkq_measure_mfma_i8(ops[:need - 16], 16, sink)


# Tile kernels with the k loop split across workgroups (configurations 60: 128 x 128 tiles, 61: 64 x 64 tiles with
# two wave groups, 62: 128 x 64 tiles).  k_slices: 0 = the library's choice, else forced; a split that does not
# divide K's stages is refused before anything is launched.
@pytest.mark.parametrize("k_slices", [0, 1, 2, 4, 8])
@pytest.mark.parametrize("cfg", [60, 61, 62])
@pytest.mark.parametrize("M,N,K", [(65, 200, 1024), (128, 768, 2048), (300, 520, 4096), (512, 1100, 1024),
                                   (100, 130, 8192), (257, 4096, 2048), (700, 300, 3072)])
def test_tiles_with_k_split_across_workgroups(mkq, scratch, cfg, M, N, K, k_slices):
    import torch
    A, Wc, s_w, s_x, bias = _codes_case(M, N, K, seed=M + N + cfg)
    try:
        r = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, want_acc=True, splitk_scratch=scratch, config=cfg,
                 k_slices=k_slices)
    except mkq.MkqError as e:
        assert e.status == mkq.MKQ_ERR_UNSUPPORTED
        stages = K // 128 // (2 if cfg == 61 else 1)
        BM, BN = {60: (128, 128), 61: (64, 64), 62: (128, 64)}[cfg]
        tiles = -(-M // BM) * -(-N // BN)
        too_big = tiles * k_slices * BM * BN * 4 > 16 << 20  # the partial sums exceed the scratch area
        assert k_slices > 0 and (stages % k_slices or stages // k_slices < 2 or too_big), "a split that applies was refused"
        pytest.skip("this split does not divide the k loop or does not fit the scratch area")
    ref = oracle.linear_int4(A, s_x, Wc, s_w, bias, out_dtype=oracle.F16)
    assert np.array_equal(to_np(r["acc"]), ref["acc"])
    assert np.array_equal(to_np(r["out"]).astype(np.float32), ref["y"])
    assert int(scratch[:16384].view(torch.int32).abs().sum()) == 0, "ticket counters not cleared"
    # the compile-time epilogues: plain binary16, binary16 residual, GELU + codes
    r16 = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, splitk_scratch=scratch, config=cfg, k_slices=k_slices)
    assert np.array_equal(to_np(r16["out"]).astype(np.float32), ref["y"])
    if N % 8 == 0:
        res = np.random.default_rng(M).normal(0, 1, (M, N)).astype(np.float16)
        refr = oracle.linear_int4(A, s_x, Wc, s_w, bias, residual=res.astype(np.float32), out_dtype=oracle.F16)
        rr = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_F16, residual=to_dev(res), splitk_scratch=scratch, config=cfg,
                  k_slices=k_slices)
        assert np.array_equal(to_np(rr["out"]).astype(np.float32), refr["y"])
        refg = oracle.linear_int4(A, s_x, Wc, s_w, bias, act=oracle.ACT_GELU, s_next=0.5)
        rg = _run(mkq, A, Wc, s_w, s_x, bias, mkq.MKQ_I4, act=mkq.MKQ_ACT_GELU, s_next=0.5, splitk_scratch=scratch,
                  config=cfg, k_slices=k_slices)
        assert_codes_match_with_tie_band(oracle.unpack_nibbles(to_np(rg["out"]), N), refg["q"], refg["y"], 0.5,
                                         what="gelu codes")
    assert int(scratch[:16384].view(torch.int32).abs().sum()) == 0, "ticket counters not cleared"


# The fused code decision at and next to exact ties.  With unit weight scales, a power-of-two activation step and
# no bias the dequantized value is acc * s_x exactly, so a step s_next = 2 * s_x * m puts every accumulator that is
# an odd multiple of m exactly half way between two codes (round half to even decides), and a step one ulp either
# side of it, or one such as 2/3 or 0.4 times that has no exact binary32 form, leaves the quotient an ulp off the
# tie, where only the correctly rounded division knows the side.  No tie band here: the codes must be the oracle's.
# (the tile configurations are forced so that the direct epilogue of the small tiles and the row epilogue of the
# large ones, which decides eight codes at a time, both run)
@pytest.mark.parametrize("s_x", [1.0, 0.125])
@pytest.mark.parametrize("M,N,K,config", [(256, 128, 64, None), (300, 200, 128, None), (300, 200, 128, 28),
                                          (300, 200, 128, 29), (520, 264, 256, 18)])
def test_fused_code_decision_at_and_next_to_exact_ties(mkq, M, N, K, s_x, config):
    rng = np.random.default_rng(M + K)
    # sparse codes keep the accumulators small enough that most of them fall inside the 4-bit range of a step ~ 2
    A = (rng.integers(-8, 8, (M, K)) * (rng.random((M, K)) < 0.08)).astype(np.int8)
    Wc = (rng.integers(-7, 8, (N, K)) * (rng.random((N, K)) < 0.3)).astype(np.int8)
    ones = np.ones(N, np.float32)
    two = np.float32(2.0 * s_x)
    steps = [two, np.nextafter(two, np.float32(np.inf)), np.nextafter(two, np.float32(0)),
             np.float32(two / 3), np.float32(two * 0.4), np.float32(two * 3), np.float32(two * 0.1)]
    ties = 0
    for s_next in steps:
        ref = oracle.linear_int4(A, s_x, Wc, ones, None, s_next=float(s_next))
        assert np.array_equal(ref["y"], ref["acc"].astype(np.float32) * np.float32(s_x))
        q = ref["y"].astype(np.float64) / np.float64(s_next)
        ties += int(((np.abs(q - np.floor(q) - 0.5) < 1e-6) & (np.abs(q) < 7)).sum())
        r4 = _run(mkq, A, Wc, ones, s_x, None, mkq.MKQ_I4, s_next=float(s_next), config=config)
        assert np.array_equal(to_np(r4["out"]), oracle.pack_nibbles(ref["q"])), f"s_next={s_next!r}"
        r = _run(mkq, A, Wc, ones, s_x, None, mkq.MKQ_F32, s_next=float(s_next), want_q=True, config=config)
        assert np.array_equal(to_np(r["q"]), oracle.pack_nibbles(ref["q"])), f"s_next={s_next!r} (second output)"
    assert ties > 1000  # the case really sits on the boundaries
