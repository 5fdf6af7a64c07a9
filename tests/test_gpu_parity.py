"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.  Integer codes, activation scales and int32 accumulators must be
bit-identical; fp16 outputs must agree within 1e-3 relative (one fp16 ulp is at most
2^-10 = 9.8e-4 relative; below the fp16 normal range one subnormal step 2^-24)."""
import sys

import numpy as np
import pytest

import workload

pytestmark = pytest.mark.gpu


def say(*a):
    print("[case]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2511_11446_amd as ql
    ql.lib()
    assert torch.cuda.is_available()
    ql.set_gemm_variant(-1)
    return ql


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def assert_y_close(y_gpu, y_ref):
    """|y_gpu - y_ref| <= 1e-3 |y_ref| (or one subnormal step near zero); returns the number of differing elements."""
    a = y_gpu.astype(np.float64)
    b = y_ref.astype(np.float64)
    assert np.isfinite(b).all()
    tol = np.maximum(1e-3 * np.abs(b), 2.0 ** -24)
    bad = np.abs(a - b) > tol
    assert not bad.any(), "max rel err %g at %s" % (np.max(np.abs(a - b) / np.maximum(np.abs(b), 1e-30)),
                                                     np.argwhere(bad)[:4].tolist())
    return int((y_gpu.view(np.uint16) != y_ref.view(np.uint16)).sum())


# ------------------------------------------------------------------ DAQ

DAQ_CASES = [
    # M, K, R
    (256, 1152, 256),   # one 256-token image, per tensor
    (64, 1152, 1),      # per token, K/8 = 144 chunks: 2 full lanes-rounds + a ragged third
    (37, 1152, 1),      # rows not a multiple of the 4 rows per workgroup
    (16, 4608, 1),      # 9 chunks per lane
    (6, 8192, 1),       # 16 chunks per lane (largest register-cached row)
    (3, 16384, 1),      # longer than the register cache: re-read path
    (8, 64, 1), (8, 8, 1), (8, 520, 1),
    (5, 100, 1), (7, 1151, 1), (9, 3, 3),   # K % 8 != 0: element-wise kernel
    (512, 1152, 256), (48, 256, 4), (48, 256, 48), (1024, 384, 1024),
]


@pytest.mark.parametrize("M,K,R", DAQ_CASES)
def test_daq_parity(gpu, orc, M, K, R):
    say("daq", M, K, R)
    x = workload.activations(M, K, "daq", R, sigma=float(workload.rng("dsig", M, K).uniform(0.05, 6.0)))
    q_ref, s_ref = orc.daq(x, R, nthreads=8)
    q, s = gpu.daq_quantize(dev(x), R)
    assert np.array_equal(host(q), q_ref)
    assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32))


def test_daq_edge_values(gpu, orc):
    say("daq edge values")
    K = 1152
    x = workload.activations(12, K, "edge")
    x[0] = 0                                    # all-zero row: scale 1, codes 0
    x[1] = np.float16(-0.0)
    x[2] = np.float16(65504.0)                  # largest finite fp16 everywhere
    x[3, :] = np.float16(6e-8)                  # smallest subnormal
    x[4, ::2] = np.float16(6e-8)
    x[4, 1::2] = np.float16(-3e-5)              # subnormal mixture
    x[5, :] = 0
    x[5, 77] = np.float16(-123.5)               # single non-zero element
    x[6] = (np.arange(K) % 255 - 127).astype(np.float16)       # amax 127 -> alpha 1: pure ties-to-even check
    x[7] = ((np.arange(K) % 255 - 127) / 2.0).astype(np.float16)  # half-integers / alpha 0.5
    x[8] = (np.arange(K) % 509 - 254).astype(np.float16) * np.float16(0.5)  # .5 ties with alpha = 1
    for R in (1, 4, 12):
        q_ref, s_ref = orc.daq(x, R)
        q, s = gpu.daq_quantize(dev(x), R)
        assert np.array_equal(host(q), q_ref), R
        assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32)), R
    q, s = gpu.daq_quantize(dev(x), 1)
    assert not host(q)[0].any() and host(s)[0] == 1.0
    assert host(q)[6].tolist() == [int(np.rint(v)) for v in x[6].astype(np.float64)]


def test_daq_power_of_two_invariance_on_gpu(gpu):
    say("daq power-of-two invariance")
    x = workload.activations(32, 1152, "p2gpu", n_outlier=0)
    x = np.where(np.abs(x) < 2.0 ** -6, np.float16(2.0 ** -6), x).astype(np.float16)
    q0, s0 = gpu.daq_quantize(dev(x), 1)
    for j in (-6, 3, 7):
        xs = (x.astype(np.float32) * np.float32(2.0 ** j)).astype(np.float16)
        q, s = gpu.daq_quantize(dev(xs), 1)
        assert np.array_equal(host(q), host(q0))
        assert np.array_equal(host(s), host(s0) * np.float32(2.0 ** j))


# ------------------------------------------------------------------ W8A8 layer

def run_w8(gpu, orc, M, K, N, R, key, use_bias=True, sigma=1.0, check_exact=False):
    x = workload.activations(M, K, key, sigma=sigma)
    lw = workload.layer_weights(key, K, N, 8, "gpu")
    b = lw["bias"] if use_bias else None
    ref = orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], b, nthreads=16)
    out = gpu.qlinear_w8a8(dev(x), R, dev(lw["w"]), dev(lw["s_w"]), None if b is None else dev(b), debug=True)
    assert np.array_equal(host(out["q"]), ref["q"])
    assert np.array_equal(host(out["s_a"]).view(np.uint32), ref["s_a"].view(np.uint32))
    assert np.array_equal(host(out["acc"]), ref["acc"])
    ndiff = assert_y_close(host(out["y"]), ref["y"])
    # without the debug exports the same y must come out
    y2 = gpu.qlinear_w8a8(dev(x), R, dev(lw["w"]), dev(lw["s_w"]), None if b is None else dev(b))
    assert np.array_equal(host(y2).view(np.uint16), host(out["y"]).view(np.uint16))
    if check_exact:
        assert ndiff == 0
    return ndiff


def test_w8a8_c1_single_linear(gpu, orc):
    say("C1 single W8A8 256x1152x1152 per-tensor")
    ndiff = run_w8(gpu, orc, 256, 1152, 1152, 256, "c1", check_exact=True)
    assert ndiff == 0


W8_SHAPES = [
    # M, K, N, R: several tiles plus ragged tails in M and N
    (300, 192, 200, 1), (129, 64, 33, 1), (1, 64, 1, 1), (257, 128, 385, 1), (512, 1152, 1152, 256),
    (96, 4608, 160, 32), (64, 1152, 3456, 1),
]


@pytest.mark.parametrize("M,K,N,R", W8_SHAPES)
def test_w8a8_shapes_default_variant(gpu, orc, M, K, N, R):
    say("w8a8", M, K, N, R)
    run_w8(gpu, orc, M, K, N, R, ("w8", M, K, N), use_bias=(M % 2 == 0), check_exact=True)


def test_w8a8_every_variant(gpu, orc):
    names = gpu.gemm_variants()
    try:
        for v, name in enumerate(names + ["generic"]):
            if v < len(names) and not name.startswith("w8"):
                continue
            gpu.set_gemm_variant(v)
            for (M, K, N, R) in [(300, 256, 200, 1), (520, 1152, 1152, 1), (260, 128, 640, 4)]:
                say("w8a8 variant", v, name, M, K, N, R)
                run_w8(gpu, orc, M, K, N, R, ("w8v", M, K, N), check_exact=True)
    finally:
        gpu.set_gemm_variant(-1)


def test_w8a8_unaligned_k_uses_generic_kernel(gpu, orc):
    for (M, K, N, R) in [(33, 100, 50, 1), (16, 72, 16, 4), (5, 7, 3, 5), (20, 1160, 40, 1)]:
        say("w8a8 generic", M, K, N, R)
        run_w8(gpu, orc, M, K, N, R, ("w8g", M, K, N), check_exact=True)


def test_w8a8_extreme_fill_and_zero_input(gpu, orc):
    say("w8a8 extreme fill")
    M, K, N = 64, 4608, 128
    x = np.full((M, K), 3.0, np.float16)
    x[1::2] = np.float16(-3.0)
    w = np.full((N, K), 127, np.int8)
    w[:, ::3] = -127
    s_w = np.full((N,), 2.0 ** -12, np.float32)
    ref = orc.qlinear_w8a8(x, 1, w, s_w, None, nthreads=8)
    out = gpu.qlinear_w8a8(dev(x), 1, dev(w), dev(s_w), None, debug=True)
    assert np.array_equal(host(out["acc"]), ref["acc"])
    assert np.abs(ref["acc"]).max() == 127 * 127 * (K - 2 * len(range(0, K, 3)))
    assert_y_close(host(out["y"]), ref["y"])
    w[:] = 127
    out = gpu.qlinear_w8a8(dev(x), 1, dev(w), dev(s_w), None, debug=True)
    assert np.abs(host(out["acc"])).max() == 4608 * 127 * 127      # the largest sum the DiT shapes can reach
    say("w8a8 zero input -> bias")
    lw = workload.layer_weights("z", 1152, 256, 8, "z")
    y = gpu.qlinear_w8a8(dev(np.zeros((40, 1152), np.float16)), 1, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]))
    assert np.array_equal(host(y), np.repeat(lw["bias"][None], 40, 0))


def test_w8a8_longest_k_fills_int32(gpu, orc):
    """K at the ABI's limit (the largest multiple of 128 below 133143), every product +-127*127: the accumulator ends
    400 000 below 2^31 and must not wrap; also the longest row the DAQ kernels see (re-read path)."""
    M, K, N = 8, 133120, 32
    say("w8a8 longest K", M, K, N)
    x = np.full((M, K), 5.0, np.float16)
    x[1::2] = np.float16(-5.0)
    w = np.full((N, K), 127, np.int8)
    w[1::2] = -127
    s_w = np.full((N,), 2.0 ** -20, np.float32)
    ref = orc.qlinear_w8a8(x, 1, w, s_w, None, nthreads=8)
    assert np.abs(ref["acc"]).max() == 127 * 127 * K and 127 * 127 * K < 2 ** 31
    out = gpu.qlinear_w8a8(dev(x), 1, dev(w), dev(s_w), None, debug=True)
    assert np.array_equal(host(out["q"]), ref["q"])
    assert np.array_equal(host(out["acc"]), ref["acc"])
    assert assert_y_close(host(out["y"]), ref["y"]) == 0


# ------------------------------------------------------------------ W4A8 layer

def run_w4(gpu, orc, M, K, N, R, key, use_bias=True, check_exact=False):
    x = workload.activations(M, K, key)
    lw = workload.layer_weights(key, K, N, 4, "gpu")
    b = lw["bias"] if use_bias else None
    w4 = gpu.ql_pack_w4_host(lw["w"])
    ref = orc.qlinear_w4a8(x, R, orc.pack_w4(lw["w"]), lw["s_w"], b, nthreads=16)
    out = gpu.qlinear_w4a8(dev(x), R, dev(w4), dev(lw["s_w"]), None if b is None else dev(b), debug=True)
    assert np.array_equal(host(out["q"]), ref["q"])
    assert np.array_equal(host(out["s_a"]).view(np.uint32), ref["s_a"].view(np.uint32))
    assert np.array_equal(host(out["P"]), ref["P"])
    ndiff = assert_y_close(host(out["y"]), ref["y"])
    y2 = gpu.qlinear_w4a8(dev(x), R, dev(w4), dev(lw["s_w"]), None if b is None else dev(b))
    assert np.array_equal(host(y2).view(np.uint16), host(out["y"]).view(np.uint16))
    if check_exact:
        assert ndiff == 0
    return ndiff


W4_SHAPES = [(300, 256, 200, 1), (129, 128, 33, 1), (64, 1152, 1152, 1), (260, 1152, 384, 4), (40, 4608, 160, 1),
             (1, 128, 1, 1)]


@pytest.mark.parametrize("M,K,N,R", W4_SHAPES)
def test_w4a8_shapes_default_variant(gpu, orc, M, K, N, R):
    say("w4a8", M, K, N, R)
    run_w4(gpu, orc, M, K, N, R, ("w4", M, K, N), use_bias=(M % 2 == 0), check_exact=True)


def test_w4a8_every_variant(gpu, orc):
    names = gpu.gemm_variants()
    try:
        for v, name in enumerate(names + ["generic"]):
            if v < len(names) and not name.startswith("w4"):
                continue
            gpu.set_gemm_variant(v)
            for (M, K, N, R) in [(300, 256, 200, 1), (264, 1152, 320, 1)]:
                say("w4a8 variant", v, name, M, K, N, R)
                run_w4(gpu, orc, M, K, N, R, ("w4v", M, K, N), check_exact=True)
    finally:
        gpu.set_gemm_variant(-1)


def test_w4a8_nibble_extremes(gpu, orc):
    say("w4a8 nibble extremes")
    M, K, N = 32, 256, 64
    x = workload.activations(M, K, "nib")
    codes = np.full((N, K), -8, np.int8)
    codes[1::2] = 7
    codes[:, 5::7] = -1
    s = workload.w4_scales(N, K, "nib")
    ref = orc.qlinear_w4a8(x, 1, orc.pack_w4(codes), s, None)
    out = gpu.qlinear_w4a8(dev(x), 1, dev(gpu.ql_pack_w4_host(codes)), dev(s), None, debug=True)
    assert np.array_equal(host(out["P"]), ref["P"])
    assert assert_y_close(host(out["y"]), ref["y"]) == 0


# ------------------------------------------------------------------ GEMM stage alone, determinism

def test_qgemm_on_given_codes_and_determinism(gpu, orc):
    say("qgemm on given codes")
    import torch
    M, K, N, R = 384, 1152, 640, 1
    g = workload.rng("qg")
    q = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    s_a = g.uniform(1e-3, 1e-1, M // R).astype(np.float32)
    lw = workload.layer_weights("qg", K, N, 8, 0)
    acc_ref = orc.gemm_i8(q, lw["w"], nthreads=8)
    y_ref = orc.epilogue_w8(acc_ref, s_a, R, lw["s_w"], lw["bias"])
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    args = (dev(q), dev(s_a), R, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]))
    y = gpu.qgemm_w8a8(*args, acc=acc)
    assert np.array_equal(host(acc), acc_ref)
    assert assert_y_close(host(y), y_ref) == 0
    for _ in range(3):   # integer results cannot depend on timing: any difference is a race
        acc2 = torch.empty_like(acc)
        y2 = gpu.qgemm_w8a8(*args, acc=acc2)
        assert torch.equal(acc2, acc) and torch.equal(y2.view(torch.int16), y.view(torch.int16))
    l4 = workload.layer_weights("qg", K, N, 4, 0)
    P_ref = orc.gemm_w4g128(q, orc.pack_w4(l4["w"]), nthreads=8)
    y4_ref = orc.epilogue_w4(P_ref, s_a, R, l4["s_w"], l4["bias"])
    P = torch.empty((M, K // 128, N), dtype=torch.int32, device="cuda")
    y4 = gpu.qgemm_w4a8(dev(q), dev(s_a), R, dev(gpu.ql_pack_w4_host(l4["w"])), dev(l4["s_w"]), dev(l4["bias"]), acc=P)
    assert np.array_equal(host(P), P_ref)
    assert assert_y_close(host(y4), y4_ref) == 0


# ------------------------------------------------------------------ DiT block shapes (configs of the benchmark)

def test_c2_block_m2048_full_compare(gpu, orc):
    """One DiT-XL/2 block at 8 images x 256 tokens, per-token DAQ, every output element compared."""
    M, R = 2048, 1
    y_fc1 = None
    for name, K, N in workload.BLOCK_LAYERS:
        say("C2", name, M, K, N)
        if name == "fc2":
            x = workload.gelu_tanh_f16(y_fc1)     # fc2 sees GELU of the oracle's fc1 output
        else:
            x = workload.activations(M, K, "c2", name)
        lw = workload.layer_weights(name, K, N, 8, "c2")
        ref = orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], lw["bias"], nthreads=16)
        if name == "fc1":
            y_fc1 = ref["y"]
        out = gpu.qlinear_w8a8(dev(x), R, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]), debug=True)
        assert np.array_equal(host(out["q"]), ref["q"])
        assert np.array_equal(host(out["s_a"]).view(np.uint32), ref["s_a"].view(np.uint32))
        assert np.array_equal(host(out["acc"]), ref["acc"])
        assert assert_y_close(host(out["y"]), ref["y"]) == 0


def _sampled_layer_check(gpu, orc, name, K, N, bits, M, R, rows, key, sigma):
    """Full-size launch on the GPU; the oracle recomputes a sample of rows (whole scale blocks)."""
    import torch
    x = workload.activations(M, K, key, name, sigma=sigma)
    lw = workload.layer_weights(name, K, N, bits, key)
    xd = dev(x)
    if bits == 8:
        out = gpu.qlinear_w8a8(xd, R, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]), debug=True)
        ref = orc.qlinear_w8a8(x[rows], R if R == 1 else len(rows), lw["w"], lw["s_w"], lw["bias"], nthreads=16)
        accname = "acc"
    else:
        out = gpu.qlinear_w4a8(xd, R, dev(gpu.ql_pack_w4_host(lw["w"])), dev(lw["s_w"]), dev(lw["bias"]), debug=True)
        ref = orc.qlinear_w4a8(x[rows], R if R == 1 else len(rows), orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"],
                               nthreads=16)
        accname = "P"
    idx = torch.from_numpy(rows).cuda()
    assert np.array_equal(host(out["q"][idx]), ref["q"])
    assert np.array_equal(host(out[accname][idx]), ref[accname])
    sidx = idx if R == 1 else idx[:1] // R
    assert np.array_equal(host(out["s_a"][sidx]).view(np.uint32), ref["s_a"].view(np.uint32))
    assert assert_y_close(host(out["y"][idx]), ref["y"]) == 0
    # properties that hold at any size: codes bounded, every scale block reaches +-127
    qa = out["q"].view(M // R, -1).abs().amax(dim=1)
    assert int(qa.max()) == 127 and int(qa.min()) == 127
    del out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("name,K,N,bits", [("qkv", 1152, 3456, 8), ("proj", 1152, 1152, 8),
                                           ("fc1", 1152, 4608, 4), ("fc2", 4608, 1152, 4)])
def test_c3_mixed_m8192_sampled(gpu, orc, name, K, N, bits):
    M = 8192
    rows = np.sort(workload.rng("c3rows", name).choice(M, size=96, replace=False))
    rows[0], rows[-1] = 0, M - 1
    say("C3", name, bits, "rows", len(rows))
    _sampled_layer_check(gpu, orc, name, K, N, bits, M, 1, rows, "c3", 1.0)


@pytest.mark.parametrize("name,K,N", [("qkv", 1152, 3456), ("fc2", 4608, 1152)])
def test_c4_m16384_drift_sampled(gpu, orc, name, K, N):
    M = 16384
    sig = workload.sigma_schedule(50)
    for step in (0, 49):
        rows = np.sort(workload.rng("c4rows", name, step).choice(M, size=64, replace=False))
        rows[0], rows[-1] = 0, M - 1
        say("C4", name, "step", step, "sigma", float(sig[step]))
        _sampled_layer_check(gpu, orc, name, K, N, 8, M, 1, rows, ("c4", step), float(sig[step]))


def test_c4_per_sample_scales_m16384(gpu, orc):
    """The paper's own granularity: one scale per image (1024 tokens) per timestep."""
    M, R = 16384, 1024
    rows = np.arange(5 * R, 6 * R)          # one whole image
    say("C4 per-sample proj, image 5")
    _sampled_layer_check(gpu, orc, "proj", 1152, 1152, 8, M, R, rows, "c4ps", 2.0)


def test_daq_seeded_random_shapes(gpu, orc):
    """Forty seeded shapes, scale granularities and quantizer settings drawn at random: the absmax and the percentile
    entry points against the oracle, bit for bit."""
    g = workload.rng("daq-random-shapes")
    for case in range(40):
        K = int(g.choice([8, 24, 64, 100, 136, 520, 1152, 1160, 2048, 4608, 9000]))
        R = int(g.choice([1, 1, 1, 2, 5, 16, 64]))
        M = R * int(g.integers(1, 12 if K > 2000 else 40))
        robust = bool(g.integers(0, 2))
        p_ppm = int(g.choice([1000000, 999000, 990000, 900000, 500000]))
        a_bits = int(g.integers(2, 9))
        sigma = float(g.uniform(1e-4, 50.0))
        say("daq random", case, M, K, R, robust, p_ppm, a_bits)
        x = workload.activations(M, K, "daq-rand", case, sigma=sigma)
        if case % 7 == 0:
            x[:: max(1, M // 3)] = 0          # some all-zero rows
        if robust:
            q_ref, s_ref = orc.daq_robust(x, R, p_ppm=p_ppm, a_bits=a_bits, nthreads=8)
            q, s = gpu.daq_quantize_robust(dev(x), R, p_ppm=p_ppm, a_bits=a_bits)
        else:
            q_ref, s_ref = orc.daq(x, R, nthreads=8)
            q, s = gpu.daq_quantize(dev(x), R)
        assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32)), case
        assert np.array_equal(host(q), q_ref), case


# ------------------------------------------------------------------ percentile-clipped DAQ (eq. (4) as printed)

ROBUST_CASES = [
    # M, K, R, p_ppm, a_bits
    (64, 1152, 1, 999000, 8),      # the paper's p = 99.9: second largest of 1152
    (16, 4608, 1, 999000, 8),      # fifth largest of 4608
    (37, 1152, 1, 990000, 6),
    (8, 8192, 1, 900000, 4),       # largest register-cached row
    (3, 16384, 1, 999000, 8),      # re-read path
    (5, 100, 1, 950000, 5), (7, 1151, 1, 999000, 8), (9, 3, 3, 500000, 8),   # K % 8 != 0
    (8, 64, 1, 1000000, 8), (8, 8, 1, 1, 2),
    (256, 1152, 256, 999000, 8),   # one image per scale: histogram selection
    (512, 1152, 256, 990000, 4), (48, 256, 4, 750000, 7), (48, 256, 48, 999000, 8),
    (1024, 384, 1024, 999900, 8), (40, 100, 8, 900000, 8),
]


@pytest.mark.parametrize("M,K,R,p_ppm,a_bits", ROBUST_CASES)
def test_daq_robust_parity(gpu, orc, M, K, R, p_ppm, a_bits):
    say("daq robust", M, K, R, p_ppm, a_bits)
    x = workload.activations(M, K, "daq-robust", R, p_ppm, sigma=float(workload.rng("rsig", M, K).uniform(0.05, 6.0)))
    q_ref, s_ref = orc.daq_robust(x, R, p_ppm=p_ppm, a_bits=a_bits, nthreads=8)
    q, s = gpu.daq_quantize_robust(dev(x), R, p_ppm=p_ppm, a_bits=a_bits)
    assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(host(q), q_ref)


def test_daq_robust_ties_zero_blocks_and_absmax_special_case(gpu, orc):
    say("daq robust ties / zero blocks")
    g = workload.rng("robust-ties")
    x = (g.integers(-5, 6, size=(24, 1152)) * 0.5).astype(np.float16)    # few distinct magnitudes: heavy ties
    x[3] = 0
    x[5, 7:] = 0                                                          # more than p of the row is zero -> tau = 0
    for R in (1, 8):
        for p_ppm, a_bits in ((999000, 8), (600000, 3), (1000000, 8)):
            q_ref, s_ref = orc.daq_robust(x, R, p_ppm=p_ppm, a_bits=a_bits)
            q, s = gpu.daq_quantize_robust(dev(x), R, p_ppm=p_ppm, a_bits=a_bits)
            assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32)), (R, p_ppm)
            assert np.array_equal(host(q), q_ref), (R, p_ppm)
    # magnitudes in the fp16 subnormal range
    x3 = (workload.activations(16, 1152, "robust-subnormal").astype(np.float32) * np.float32(2.0 ** -18)).astype(np.float16)
    assert (np.abs(x3.astype(np.float32)) < 2.0 ** -14).mean() > 0.5
    for R in (1, 16):
        q_ref, s_ref = orc.daq_robust(x3, R, p_ppm=990000, a_bits=8)
        q, s = gpu.daq_quantize_robust(dev(x3), R, p_ppm=990000, a_bits=8)
        assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32)) and np.array_equal(host(q), q_ref)
    # p = 100 %, 8 bits: the absmax entry point's result
    x2 = workload.activations(64, 1152, "robust-absmax")
    q0, s0 = gpu.daq_quantize(dev(x2), 1)
    q1, s1 = gpu.daq_quantize_robust(dev(x2), 1, p_ppm=1000000, a_bits=8)
    assert np.array_equal(host(q0), host(q1)) and np.array_equal(host(s0), host(s1))


def test_daq_robust_full_size_rows_sampled(gpu, orc):
    """M = 16384 per token at the paper's p; the oracle checks a seeded sample of the rows (rows are independent)."""
    M, K = 16384, 1152
    say("daq robust full size", M, K)
    x = workload.activations(M, K, "robust-full", sigma=2.0)
    q, s = gpu.daq_quantize_robust(dev(x), 1, p_ppm=999000, a_bits=8)
    rows = np.sort(workload.rng("robust-rows").choice(M, size=512, replace=False))
    q_ref, s_ref = orc.daq_robust(x[rows], 1, p_ppm=999000, a_bits=8, nthreads=8)
    assert np.array_equal(host(q)[rows], q_ref)
    assert np.array_equal(host(s)[rows].view(np.uint32), s_ref.view(np.uint32))


def test_plan_runner_robust_time_bins(gpu, orc):
    """Algorithm 2 Phase B: the same plan run with the activation width of each time bin."""
    import ctypes
    import torch
    M, R = 256, 64
    shapes = [("a", 256, 384, 8), ("b", 384, 256, 4)]
    layers, xs = [], []
    for name, K, N, bits in shapes:
        lw = workload.layer_weights(name, K, N, bits, "plan-robust")
        w = dev(lw["w"]) if bits == 8 else dev(gpu.ql_pack_w4_host(lw["w"]))
        layers.append(dict(K=K, N=N, bits=bits, w=w, w_scale=dev(lw["s_w"]), bias=dev(lw["bias"]), host=lw))
        xs.append(workload.activations(M, K, "plan-robust", name))
    plan = gpu.Plan([{k: v for k, v in l.items() if k != "host"} for l in layers], M_max=M)
    ys = [torch.zeros((M, l["N"]), dtype=torch.float16, device="cuda") for l in layers]
    xd = [dev(x) for x in xs]
    ws = gpu.workspace(plan.workspace_bytes(M, R))
    xp = (ctypes.c_void_p * 2)(*[t.data_ptr() for t in xd])
    yp = (ctypes.c_void_p * 2)(*[t.data_ptr() for t in ys])
    sptr = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    policy = {0: 8, 1: 6, 2: 4}          # activation bits per bin (early, mid, late)
    for step in (0, 4, 8):
        a_bits = policy[gpu.time_bin(step, 9)]
        say("plan robust step", step, "a_bits", a_bits)
        plan.run_ptrs_robust(xp, yp, M, R, 999000, a_bits, ws, sptr)
        torch.cuda.synchronize()
        for l, x, y in zip(layers, xs, ys):
            lw = l["host"]
            q, s = orc.daq_robust(x, R, p_ppm=999000, a_bits=a_bits)
            if l["bits"] == 8:
                ref = orc.epilogue_w8(orc.gemm_i8(q, lw["w"]), s, R, lw["s_w"], lw["bias"])
            else:
                ref = orc.epilogue_w4(orc.gemm_w4g128(q, orc.pack_w4(lw["w"])), s, R, lw["s_w"], lw["bias"])
            assert assert_y_close(host(y), ref) == 0
    plan.close()


def test_prepack_w4_from_pair_order_on_the_device(gpu, orc):
    """Weights that arrive two per byte in pair order (low nibble = even k): the device re-layout gives the bytes the
    oracle's own packer writes for the same codes, and a layer run on them matches the oracle."""
    import torch
    M, K, N, R = 300, 1152, 200, 1
    say("prepack w4", M, K, N)
    lw = workload.layer_weights("prepack", K, N, 4, 0)
    w = lw["w"]
    pairs = ((w[:, 0::2] & 0xF) | ((w[:, 1::2] & 0xF) << 4)).astype(np.uint8)
    packed = gpu.prepack_w4(dev(pairs))
    assert np.array_equal(host(packed), orc.pack_w4(w))
    x = workload.activations(M, K, "prepack")
    ref = orc.qlinear_w4a8(x, R, orc.pack_w4(w), lw["s_w"], lw["bias"], nthreads=8, want_debug=False)["y"]
    y = gpu.qlinear_w4a8(dev(x), R, packed, dev(lw["s_w"]), dev(lw["bias"]))
    assert assert_y_close(host(y), ref) == 0
    # a ragged block count (N*K/8 not a multiple of 256) and the smallest row
    w2 = workload.rng("prepack2").integers(-8, 8, size=(3, 8), dtype=np.int8)
    p2 = ((w2[:, 0::2] & 0xF) | ((w2[:, 1::2] & 0xF) << 4)).astype(np.uint8)
    assert np.array_equal(host(gpu.prepack_w4(dev(p2))), orc.pack_w4(w2))


# ------------------------------------------------------------------ 4-bit weights with other group sizes

W4G_CASES = [
    # M, K, N, R, group
    (192, 1152, 192, 1, 288),     # the paper's most used group size: 2.25 K steps per group
    (160, 1152, 200, 1, 192),     # ragged M and N
    (128, 1152, 128, 1, 64),
    (96, 1152, 64, 1, 32),        # one group per 32-wide K slice
    (256, 4608, 256, 64, 288),
    (64, 1152, 96, 1, 1152),      # one group for the whole row
    (64, 1152, 96, 1, 384),
    (48, 576, 80, 1, 288),        # K % 128 != 0: generic kernel
    (40, 96, 24, 1, 96),
    # more than 256 rows: the pipelined kernel, whose restart pattern is unrolled for the group set of Algorithm 1
    (384, 1152, 320, 1, 32),
    (384, 1152, 320, 1, 64),
    (300, 2304, 200, 1, 192),     # period of 3 K steps, 6 periods
    (520, 1152, 136, 4, 288),     # period of 9 K steps = the whole row
    (300, 4608, 200, 1, 288),     # 4 periods
    (300, 4608, 200, 1, 64),      # 72 groups: the table of up to 144 groups, one workgroup per CU
    (300, 4608, 136, 1, 32),      # 144 groups
    (300, 1152, 200, 1, 384),     # a group size outside the set: the uniform-branch form
]


@pytest.mark.parametrize("M,K,N,R,group", W4G_CASES)
def test_w4a8_group_sizes(gpu, orc, M, K, N, R, group):
    say("w4 group", M, K, N, R, group)
    x = workload.activations(M, K, "w4g", group)
    lw = workload.layer_weights("w4g", K, N, 4, group)
    sw = workload.w4_scales_group(N, K, group, "w4g")
    q_ref, s_ref = orc.daq(x, R)
    P_ref = orc.gemm_w4g(q_ref, orc.pack_w4(lw["w"]), group, nthreads=8)
    y_ref = orc.epilogue_w4(P_ref, s_ref, R, sw, lw["bias"])
    out = gpu.qlinear_w4a8(dev(x), R, dev(gpu.ql_pack_w4_host(lw["w"])), dev(sw), dev(lw["bias"]), debug=True, group=group)
    assert np.array_equal(host(out["q"]), q_ref)
    assert np.array_equal(host(out["P"]), P_ref)
    assert assert_y_close(host(out["y"]), y_ref) == 0
    # the same without the debug exports (the path a plan takes)
    y = gpu.qlinear_w4a8(dev(x), R, dev(gpu.ql_pack_w4_host(lw["w"])), dev(sw), dev(lw["bias"]), group=group)
    assert assert_y_close(host(y), y_ref) == 0


def test_w4a8_group128_through_the_group_entry_point_and_both_any_group_variants(gpu, orc):
    M, K, N = 256, 1152, 256
    x = workload.activations(M, K, "w4g128")
    lw = workload.layer_weights("w4g128", K, N, 4)
    ref = orc.qlinear_w4a8(x, 1, orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"], want_debug=False)["y"]
    w4 = dev(gpu.ql_pack_w4_host(lw["w"]))
    names = gpu.gemm_variants()
    sw288 = workload.w4_scales_group(N, K, 288, "v")
    q_ref, s_ref = orc.daq(x, 1)
    ref288 = orc.epilogue_w4(orc.gemm_w4g(q_ref, orc.pack_w4(lw["w"]), 288), s_ref, 1, sw288, lw["bias"])
    try:
        for v, nm in enumerate(names):
            if not nm.startswith("w4 any-group"):
                continue
            say("variant", nm)
            gpu.set_gemm_variant(v)
            y = gpu.qlinear_w4a8(dev(x), 1, w4, dev(lw["s_w"]), dev(lw["bias"]))            # group 128 on the generic-group kernel
            assert assert_y_close(host(y), ref) == 0
            y = gpu.qlinear_w4a8(dev(x), 1, w4, dev(sw288), dev(lw["bias"]), group=288)
            assert assert_y_close(host(y), ref288) == 0
    finally:
        gpu.set_gemm_variant(-1)


def test_plan_with_mixed_group_sizes(gpu, orc):
    import torch
    M, R = 256, 1
    shapes = [("a", 1152, 192, 4, 288), ("b", 1152, 128, 4, 128), ("c", 1152, 160, 8, 0), ("d", 1152, 96, 4, 64)]
    layers, xs, refs = [], [], []
    for name, K, N, bits, group in shapes:
        lw = workload.layer_weights(name, K, N, bits, "plan-groups")
        x = workload.activations(M, K, "plan-groups", name)
        if bits == 8:
            refs.append(orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], lw["bias"], want_debug=False)["y"])
            layers.append(dict(K=K, N=N, bits=8, w=dev(lw["w"]), w_scale=dev(lw["s_w"]), bias=dev(lw["bias"])))
        else:
            sw = workload.w4_scales_group(N, K, group, name)
            q, s = orc.daq(x, R)
            refs.append(orc.epilogue_w4(orc.gemm_w4g(q, orc.pack_w4(lw["w"]), group), s, R, sw, lw["bias"]))
            layers.append(dict(K=K, N=N, bits=4, group=group, w=dev(gpu.ql_pack_w4_host(lw["w"])), w_scale=dev(sw),
                               bias=dev(lw["bias"])))
        xs.append(dev(x))
    plan = gpu.Plan(layers, M_max=M)
    ys = [torch.zeros((M, l["N"]), dtype=torch.float16, device="cuda") for l in layers]
    ws = gpu.workspace(plan.workspace_bytes(M, R))
    plan.run(xs, ys, M, R, ws)
    torch.cuda.synchronize()
    for y, ref in zip(ys, refs):
        assert assert_y_close(host(y), ref) == 0
    plan.close()


# ------------------------------------------------------------------ block glue folded into the epilogue

def _glue_reference(orc, x, R, lw, bits, group, act, residual, gate, gate_rows):
    q, s = orc.daq(x, R, nthreads=8)
    if bits == 8:
        u = orc.dequant_w8(orc.gemm_i8(q, lw["w"], nthreads=8), s, R, lw["s_w"], lw["bias"])
    else:
        u = orc.dequant_w4(orc.gemm_w4g(q, orc.pack_w4(lw["w"]), group, nthreads=8), s, R, lw["s_w"], lw["bias"])
    return orc.block_glue(u, act=act, residual=residual, gate=gate, gate_rows=gate_rows)


GLUE_CASES = [
    # M, K, N, R, bits, group, act, residual, gate_rows (0 = no gate)
    (512, 1152, 384, 1, 8, 0, 1, False, 0),       # fc1-like: GELU only, full tiles
    (512, 1152, 384, 1, 8, 0, 0, True, 256),      # proj-like: gated residual
    (512, 1152, 384, 1, 8, 0, 1, True, 256),      # everything at once
    (300, 1152, 200, 1, 8, 0, 1, True, 100),      # ragged M and N: element-wise epilogue
    (256, 1152, 256, 1, 8, 0, 0, True, 0),        # plain residual
    (256, 1152, 256, 1, 8, 0, 0, False, 64),      # gate alone
    (64, 200, 48, 1, 8, 0, 1, True, 32),          # generic kernel (K % 64 != 0)
    (256, 1152, 256, 1, 4, 128, 1, True, 256),    # 4-bit weights
    (256, 1152, 192, 1, 4, 288, 0, True, 128),    # 4-bit, group 288
    (4096, 1152, 1152, 1, 8, 0, 0, True, 1024),   # a shape of the persistent walk: with glue it runs on 256x192 tiles, eight wavefronts
    (4096, 1152, 3456, 1, 8, 0, 1, False, 0),     # the same for a wide layer, GELU only
    (256, 4608, 384, 256, 8, 0, 0, True, 256),    # K = 4608, per-sample scales
    (384, 4608, 256, 1, 4, 64, 1, True, 128),     # 4-bit, 72 groups along K: the pipelined kernel with the large scale table, with glue
    (384, 1152, 256, 1, 4, 128, 1, True, 128),    # 4-bit group 128 above 256 rows: the pipelined kernel's glue build
]


@pytest.mark.parametrize("M,K,N,R,bits,group,act,use_res,gate_rows", GLUE_CASES)
def test_fused_epilogue(gpu, orc, M, K, N, R, bits, group, act, use_res, gate_rows):
    say("glue", M, K, N, R, bits, group, act, use_res, gate_rows)
    x = workload.activations(M, K, "glue", N, bits)
    lw = workload.layer_weights("glue", K, N, bits, "glue")
    if bits == 4 and group != 128:
        lw = dict(lw, s_w=workload.w4_scales_group(N, K, group, "glue"))
    g = workload.rng("glue-rg", M, N)
    residual = (g.standard_normal((M, N), dtype=np.float32) * 2).astype(np.float16) if use_res else None
    gate = (g.standard_normal((M // gate_rows, N), dtype=np.float32)).astype(np.float16) if gate_rows else None
    ref = _glue_reference(orc, x, R, lw, bits, group, act, residual, gate, max(gate_rows, 1))
    w = dev(lw["w"]) if bits == 8 else dev(gpu.ql_pack_w4_host(lw["w"]))
    y = gpu.qlinear_fused(dev(x), R, w, dev(lw["s_w"]), dev(lw["bias"]), bits=bits, group=group or 128, act=act,
                          residual=None if residual is None else dev(residual), gate=None if gate is None else dev(gate),
                          gate_rows=max(gate_rows, 1))
    if act == 0:
        assert assert_y_close(host(y), ref) == 0          # no transcendental involved: identical
        return
    # fp32 GELU on the GPU against the oracle's fp64 one: h = fp16(gelu(u)) may differ by one fp16 ulp in rare elements.
    # Through the gated addition that is an ABSOLUTE error of |g| ulp(h), which a small |y| (cancellation against the
    # residual) does not shrink: the bound below is 1e-3 relative on y plus one ulp of h carried through the gate.
    yg = host(y).astype(np.float64)
    h_ref = _glue_reference(orc, x, R, lw, bits, group, act, None, None, 1).astype(np.float64)
    gabs = np.abs(np.repeat(gate.astype(np.float64), gate_rows, 0)) if gate is not None else 1.0
    tol = 1e-3 * np.abs(ref.astype(np.float64)) + gabs * np.abs(h_ref) * 2.0 ** -10 + 2.0 ** -24
    assert (np.abs(yg - ref.astype(np.float64)) <= tol).all()
    ndiff = int((host(y).view(np.uint16) != ref.view(np.uint16)).sum())
    assert ndiff <= max(4, y.numel() // 500)              # and such elements are rare


ROWMAX_CASES = [
    # M, K, N, bits, group, act, residual+gate
    (512, 1152, 384, 8, 0, 1, False),       # fc1-like: GELU, staged epilogue (the row maxima pass through the LDS strip)
    (512, 1152, 384, 8, 0, 0, True),        # gated residual: the maximum is taken after the addition
    (300, 1152, 200, 8, 0, 1, False),       # ragged: element-wise epilogue, one atomic per element
    (384, 1152, 320, 4, 128, 1, False),     # the pipelined 4-bit kernel
    (384, 1152, 320, 4, 288, 0, False),     # no glue at all, only the side output
    (4096, 1152, 1152, 8, 0, 1, False),     # 256x192 tiles on eight wavefronts
    (64, 200, 48, 8, 0, 1, True),           # generic kernel
    (384, 1152, 256, 16, 0, 1, False),      # a layer left in FP16
]


@pytest.mark.parametrize("M,K,N,bits,group,act,use_rg", ROWMAX_CASES)
def test_row_absmax_side_output_and_daq_from_it(gpu, orc, M, K, N, bits, group, act, use_rg):
    """The epilogue's side output (largest |y| of every row as a binary16 bit pattern) against the oracle's definition
    applied to the y the same call wrote, and the DAQ that starts from it against the oracle's DAQ of that y: scales and
    codes bit for bit, at one row, a few rows and more than 256 rows per scale."""
    import torch
    say("rowmax", M, K, N, bits, group, act, use_rg)
    x = workload.activations(M, K, "rowmax", N, bits)
    g = workload.rng("rowmax-rg", M, N)
    residual = dev((g.standard_normal((M, N), dtype=np.float32) * 2).astype(np.float16)) if use_rg else None
    gate = dev(g.standard_normal((M // 32, N), dtype=np.float32).astype(np.float16)) if use_rg else None
    rowmax = torch.full((M,), 0x7fffffff, dtype=torch.int32, device="cuda")       # the call clears it
    if bits == 16:
        w = workload.f16_weights(N, K, "rowmax")
        y = gpu.qlinear_f16(dev(x), dev(w), dev(workload.bias(N, "rowmax")), act=act, residual=residual, gate=gate, gate_rows=32,
                            row_absmax=rowmax)
    else:
        lw = workload.layer_weights("rowmax", K, N, bits, "rowmax")
        if bits == 4 and group != 128:
            lw = dict(lw, s_w=workload.w4_scales_group(N, K, group, "rowmax"))
        w = dev(lw["w"]) if bits == 8 else dev(gpu.ql_pack_w4_host(lw["w"]))
        y = gpu.qlinear_fused(dev(x), 1, w, dev(lw["s_w"]), dev(lw["bias"]), bits=bits, group=group or 128, act=act,
                              residual=residual, gate=gate, gate_rows=32, row_absmax=rowmax)
    yh = host(y)
    assert np.isfinite(yh.astype(np.float32)).all()
    assert np.array_equal(host(rowmax).astype(np.uint32), orc.row_absmax_bits(yh))
    for R in (1, 4, M) if M % 4 == 0 else (1, M):
        q_ref, s_ref = orc.daq(yh, R)
        q, s = gpu.daq_quantize_rowmax(y, R, rowmax)
        assert np.array_equal(host(s).view(np.uint32), s_ref.view(np.uint32)), R
        assert np.array_equal(host(q), q_ref), R


def test_fused_epilogue_with_nothing_to_fuse_is_the_plain_layer_and_misaligned_glue_still_works(gpu, orc):
    import torch
    M, K, N = 256, 1152, 256
    x = workload.activations(M, K, "glue0")
    lw = workload.layer_weights("glue0", K, N, 8, "glue0")
    plain = gpu.qlinear_w8a8(dev(x), 1, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]))
    fused = gpu.qlinear_fused(dev(x), 1, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]))
    assert torch.equal(plain, fused)
    # a residual that starts 2 bytes off a 16-byte boundary: the 16-byte piece path must step aside
    res = (workload.rng("glue-mis").standard_normal((M, N), dtype=np.float32)).astype(np.float16)
    buf = torch.zeros(M * N + 8, dtype=torch.float16, device="cuda")
    view = buf[1:1 + M * N].view(M, N)
    view.copy_(dev(res))
    assert view.data_ptr() % 16 == 2
    y = gpu.qlinear_fused(dev(x), 1, dev(lw["w"]), dev(lw["s_w"]), dev(lw["bias"]), residual=view)
    q, s = orc.daq(x, 1)
    ref = orc.block_glue(orc.dequant_w8(orc.gemm_i8(q, lw["w"]), s, 1, lw["s_w"], lw["bias"]), residual=res)
    assert assert_y_close(host(y), ref) == 0


# ------------------------------------------------------------------ layers the plan leaves in FP16

def _f16_tolerance(x, w, ref):
    """fp32 accumulation of K exact products in any order: |error| <= K 2^-24 sum|x w| (loose standard bound), plus the
    rounding to fp16 (the oracle's own fp16 result may sit one ulp away when the two sums straddle a rounding point)."""
    K = x.shape[1]
    mag = np.abs(x.astype(np.float64)) @ np.abs(w.astype(np.float64)).T
    return K * 2.0 ** -24 * mag + 2.0 ** -10 * np.abs(ref.astype(np.float64)) + 2.0 ** -24


F16_CASES = [(512, 1152, 384), (300, 1152, 200), (64, 1152, 128), (33, 100, 17), (4096, 1152, 1152), (256, 4608, 256)]


@pytest.mark.parametrize("M,K,N", F16_CASES)
def test_fp16_layer(gpu, orc, M, K, N):
    say("f16 layer", M, K, N)
    g = workload.rng("f16-gpu", M, K, N)
    x = workload.activations(M, K, "f16-gpu", N)
    w = (g.standard_normal((N, K), dtype=np.float32) * 0.05).astype(np.float16)
    b = workload.bias(N, "f16-gpu")
    ref = orc.linear_f16(x, w, b, nthreads=8)
    y = host(gpu.qlinear_f16(dev(x), dev(w), dev(b)))
    err = np.abs(y.astype(np.float64) - ref.astype(np.float64))
    assert (err <= _f16_tolerance(x, w, ref)).all()
    assert (y.view(np.uint16) != ref.view(np.uint16)).mean() < 0.02      # and almost all outputs are identical
    y2 = host(gpu.qlinear_f16(dev(x), dev(w), None))
    ref2 = orc.linear_f16(x, w, None, nthreads=8)
    assert (np.abs(y2.astype(np.float64) - ref2.astype(np.float64)) <= _f16_tolerance(x, w, ref2)).all()


def test_fp16_layer_with_glue_on_a_shape_that_picks_a_persistent_tile(gpu, orc):
    M, K, N = 4096, 1152, 1152
    g = workload.rng("f16-glue")
    x = workload.activations(M, K, "f16-glue")
    w = (g.standard_normal((N, K), dtype=np.float32) * 0.05).astype(np.float16)
    res = g.standard_normal((M, N), dtype=np.float32).astype(np.float16)
    gate = g.standard_normal((M // 256, N), dtype=np.float32).astype(np.float16)
    rows = np.sort(g.choice(M, size=256, replace=False))
    y = host(gpu.qlinear_f16(dev(x), dev(w), None, residual=dev(res), gate=dev(gate), gate_rows=256))[rows]
    h = orc.linear_f16(x[rows], w, None, nthreads=8)
    ref = (gate[rows // 256].astype(np.float32) * h.astype(np.float32) + res[rows].astype(np.float32)).astype(np.float16)
    # h may sit one fp16 ulp from the oracle's (fp32 against fp64 sums); the gate carries that into y
    tol = _f16_tolerance(x[rows], w, h) * np.abs(gate[rows // 256].astype(np.float64)) + 2.0 ** -10 * np.abs(ref.astype(np.float64)) + 2.0 ** -24
    assert (np.abs(y.astype(np.float64) - ref.astype(np.float64)) <= tol).all()
    assert (y.view(np.uint16) != ref.view(np.uint16)).mean() < 0.02


def test_plan_with_fp16_int8_and_int4_layers(gpu, orc):
    """A plan of the kind Step 2 ends with: FP16, W8 and W4 (two group sizes) layers side by side."""
    import torch
    M, R = 512, 1
    g = workload.rng("plan-f16")
    layers, xs, refs, tols = [], [], [], []
    for name, K, N, bits, group in [("a", 1152, 256, 16, 0), ("b", 1152, 384, 8, 0), ("c", 1152, 192, 4, 288), ("d", 256, 128, 16, 0)]:
        x = workload.activations(M, K, "plan-f16", name)
        xs.append(dev(x))
        if bits == 16:
            w = (g.standard_normal((N, K), dtype=np.float32) * 0.05).astype(np.float16)
            b = workload.bias(N, "plan-f16", name)
            ref = orc.linear_f16(x, w, b, nthreads=8)
            refs.append(ref)
            tols.append(_f16_tolerance(x, w, ref))
            layers.append(dict(K=K, N=N, bits=16, w=dev(w), w_scale=None, bias=dev(b)))
            continue
        lw = workload.layer_weights(name, K, N, bits, "plan-f16")
        q, s = orc.daq(x, R)
        if bits == 8:
            refs.append(orc.epilogue_w8(orc.gemm_i8(q, lw["w"]), s, R, lw["s_w"], lw["bias"]))
            layers.append(dict(K=K, N=N, bits=8, w=dev(lw["w"]), w_scale=dev(lw["s_w"]), bias=dev(lw["bias"])))
        else:
            sw = workload.w4_scales_group(N, K, group, name)
            refs.append(orc.epilogue_w4(orc.gemm_w4g(q, orc.pack_w4(lw["w"]), group), s, R, sw, lw["bias"]))
            layers.append(dict(K=K, N=N, bits=4, group=group, w=dev(gpu.ql_pack_w4_host(lw["w"])), w_scale=dev(sw), bias=dev(lw["bias"])))
        tols.append(None)
    plan = gpu.Plan(layers, M_max=M)
    ys = [torch.zeros((M, l["N"]), dtype=torch.float16, device="cuda") for l in layers]
    ws = gpu.workspace(plan.workspace_bytes(M, R))
    plan.run(xs, ys, M, R, ws)
    torch.cuda.synchronize()
    for y, ref, tol in zip(ys, refs, tols):
        if tol is None:
            assert assert_y_close(host(y), ref) == 0
        else:
            assert (np.abs(host(y).astype(np.float64) - ref.astype(np.float64)) <= tol).all()
    plan.close()


# ------------------------------------------------------------------ the final-plan features at full size (sampled rows)

def test_full_size_group288_fp16_and_fused_layers_sampled(gpu, orc):
    """M = 16384, the launch configuration the c6 workload times: a W4 layer with groups of 288, an FP16 layer and a
    fused W8 layer; the oracle recomputes a seeded sample of rows."""
    import torch
    M, K, N = 16384, 1152, 3456
    g = workload.rng("full-final")
    rows = np.sort(g.choice(M, size=64, replace=False))
    rows[0], rows[-1] = 0, M - 1
    idx = torch.from_numpy(rows).cuda()
    x = workload.activations(M, K, "full-final", sigma=1.0)
    xd = dev(x)
    q_ref, s_ref = orc.daq(x[rows], 1, nthreads=8)
    # W4, groups of 288
    say("full size w4 g288")
    lw = workload.layer_weights("qkv", K, N, 4, "full-final")
    sw = workload.w4_scales_group(N, K, 288, "full-final")
    y = gpu.qlinear_w4a8(xd, 1, dev(gpu.ql_pack_w4_host(lw["w"])), dev(sw), dev(lw["bias"]), group=288)
    ref = orc.epilogue_w4(orc.gemm_w4g(q_ref, orc.pack_w4(lw["w"]), 288, nthreads=8), s_ref, 1, sw, lw["bias"])
    assert assert_y_close(host(y[idx]), ref) == 0
    # FP16 layer
    say("full size fp16")
    w16 = workload.f16_weights(N, K, "full-final")
    b16 = workload.bias(N, "full-final")
    y = gpu.qlinear_f16(xd, dev(w16), dev(b16))
    ref = orc.linear_f16(x[rows], w16, b16, nthreads=8)
    assert (np.abs(host(y[idx]).astype(np.float64) - ref.astype(np.float64)) <= _f16_tolerance(x[rows], w16, ref)).all()
    # fused W8 layer: gated residual (no transcendental: identical)
    say("full size fused w8")
    lw8 = workload.layer_weights("qkv", K, N, 8, "full-final")
    res = g.standard_normal((M, N), dtype=np.float32).astype(np.float16)
    gate = g.standard_normal((M // 256, N), dtype=np.float32).astype(np.float16)
    y = gpu.qlinear_fused(xd, 1, dev(lw8["w"]), dev(lw8["s_w"]), dev(lw8["bias"]), residual=dev(res), gate=dev(gate), gate_rows=256)
    u = orc.dequant_w8(orc.gemm_i8(q_ref, lw8["w"], nthreads=8), s_ref, 1, lw8["s_w"], lw8["bias"])
    # the oracle on the gathered rows, each with its own gate row
    ref = orc.block_glue(u, residual=res[rows], gate=gate[rows // 256], gate_rows=1)
    assert assert_y_close(host(y[idx]), ref) == 0
    del y
    torch.cuda.empty_cache()


# ------------------------------------------------------------------ seeded random layer shapes

def test_layers_seeded_random_shapes(gpu, orc):
    """Thirty seeded layers of random shape, weight width, group size, scale granularity and glue, against the oracle."""
    g = workload.rng("layer-random-shapes")
    for case in range(30):
        bits = int(g.choice([8, 8, 4, 4, 16]))
        K = int(g.choice([64, 128, 192, 576, 1152, 2304]) if bits != 8 else g.choice([24, 64, 200, 576, 1152, 2304]))
        if bits == 4:
            group = int(g.choice([gs for gs in (32, 64, 96, 128, 192, 288, 576) if K % gs == 0]))
        else:
            group = 128
        R = int(g.choice([1, 1, 4]))
        M = R * int(g.integers(1, 100))
        N = int(g.integers(1, 400))
        act = int(g.integers(0, 2))
        use_res, use_gate = bool(g.integers(0, 2)), bool(g.integers(0, 2))
        gate_rows = int(g.choice([d for d in (1, 2, 4, M) if M % d == 0]))
        say("layer random", case, bits, M, K, N, R, group, act, use_res, use_gate, gate_rows)
        x = workload.activations(M, K, "layer-rand", case)
        res = g.standard_normal((M, N), dtype=np.float32).astype(np.float16) if use_res else None
        gate = g.standard_normal((M // gate_rows, N), dtype=np.float32).astype(np.float16) if use_gate else None
        kw = dict(act=act, residual=None if res is None else dev(res), gate=None if gate is None else dev(gate), gate_rows=gate_rows)
        if bits == 16:
            w = (g.standard_normal((N, K), dtype=np.float32) * 0.05).astype(np.float16)
            b = workload.bias(N, "layer-rand", case)
            h = orc.linear_f16(x, w, b, nthreads=8)
            y = host(gpu.qlinear_f16(dev(x), dev(w), dev(b), **kw)).astype(np.float64)
            lo = orc.block_glue(h.astype(np.float32), act=act, residual=res, gate=gate, gate_rows=gate_rows).astype(np.float64)
            gabs = np.abs(np.repeat(gate.astype(np.float64), gate_rows, 0)) if gate is not None else 1.0
            # fp32 against fp64 sums (and fp32 GELU): the value before the glue may move by the accumulation bound plus an ulp
            tol = (_f16_tolerance(x, w, h) + 2.0 ** -9 * np.abs(h.astype(np.float64))) * gabs * (1.2 if act else 1.0) \
                + 2.0 ** -10 * np.abs(lo) + 2.0 ** -24
            assert (np.abs(y - lo) <= tol).all(), case
            continue
        lw = workload.layer_weights("layer-rand", K, N, bits, case)
        if bits == 4:
            lw = dict(lw, s_w=workload.w4_scales_group(N, K, group, "layer-rand", case))
        q, sc = orc.daq(x, R, nthreads=8)
        if bits == 8:
            u = orc.dequant_w8(orc.gemm_i8(q, lw["w"], nthreads=8), sc, R, lw["s_w"], lw["bias"])
            w = dev(lw["w"])
        else:
            u = orc.dequant_w4(orc.gemm_w4g(q, orc.pack_w4(lw["w"]), group, nthreads=8), sc, R, lw["s_w"], lw["bias"])
            w = dev(gpu.ql_pack_w4_host(lw["w"]))
        ref = orc.block_glue(u, act=act, residual=res, gate=gate, gate_rows=gate_rows)
        y = host(gpu.qlinear_fused(dev(x), R, w, dev(lw["s_w"]), dev(lw["bias"]), bits=bits, group=group, **kw))
        if act == 0:
            assert assert_y_close(y, ref) == 0, case
        else:
            h_ref = orc.block_glue(u, act=1).astype(np.float64)
            gabs = np.abs(np.repeat(gate.astype(np.float64), gate_rows, 0)) if gate is not None else 1.0
            tol = 1e-3 * np.abs(ref.astype(np.float64)) + gabs * np.abs(h_ref) * 2.0 ** -10 + 2.0 ** -24
            assert (np.abs(y.astype(np.float64) - ref.astype(np.float64)) <= tol).all(), case


# ------------------------------------------------------------------ LayerNorm + modulation in the DAQ prologue

def _ln_tolerance(x, sh, sc, rows_per_mod, ref):
    """One fp16 step of the result, plus what fp32 evaluation can lose where n (1 + scale) and shift nearly cancel:
    2^-18 of their magnitudes (a handful of fp32 roundings; 128 times below one fp16 step of those magnitudes)."""
    xd = x.astype(np.float64)
    mu = xd.mean(axis=1, keepdims=True)
    n = (xd - mu) / np.sqrt(((xd - mu) ** 2).mean(axis=1, keepdims=True) + 1e-6)
    g = 1.0 if sc is None else 1.0 + np.repeat(sc.astype(np.float64), rows_per_mod, 0)
    b = 0.0 if sh is None else np.repeat(sh.astype(np.float64), rows_per_mod, 0)
    return 2.0 ** -10 * np.abs(ref.astype(np.float64)) + 2.0 ** -18 * (np.abs(n * g) + np.abs(b)) + 2.0 ** -24


LN_CASES = [(64, 1152, 1, 16), (300, 1152, 1, 100), (37, 64, 1, 1), (48, 4608, 1, 48), (1024, 1152, 256, 256), (96, 384, 96, 32)]


@pytest.mark.parametrize("M,K,R,rows_per_mod", LN_CASES)
def test_layernorm_modulate_daq(gpu, orc, M, K, R, rows_per_mod):
    """h (normalised, modulated rows) within one fp16 step of the float64 oracle; the codes and scales are the oracle's
    DAQ of the kernel's own h, bit for bit (the integer decision is taken on the same fp16 values on both sides)."""
    say("ln+daq", M, K, R, rows_per_mod)
    g = workload.rng("ln", M, K)
    x = (workload.activations(M, K, "ln", sigma=2.0).astype(np.float32) + np.float32(1.5)).astype(np.float16)   # non-zero mean
    sc = (g.standard_normal((M // rows_per_mod, K)) * 0.3).astype(np.float16)
    sh = (g.standard_normal((M // rows_per_mod, K)) * 0.5).astype(np.float16)
    for use_mod in (True, False):
        out = gpu.daq_quantize_ln(dev(x), R, dev(sh) if use_mod else None, dev(sc) if use_mod else None, rows_per_mod, 1e-6, want_h=True)
        h = host(out["h"])
        ref = orc.layernorm_modulate(x, sh if use_mod else None, sc if use_mod else None, rows_per_mod, 1e-6)
        a, b = h.astype(np.float64), ref.astype(np.float64)
        assert (np.abs(a - b) <= _ln_tolerance(x, sh if use_mod else None, sc if use_mod else None, rows_per_mod, ref)).all()
        assert (h.view(np.uint16) != ref.view(np.uint16)).mean() < 0.01
        q_ref, s_ref = orc.daq(h, R, nthreads=8)
        assert np.array_equal(host(out["q"]), q_ref)
        assert np.array_equal(host(out["scales"]).view(np.uint32), s_ref.view(np.uint32))
    if R == 1:
        # without the h export the same codes come out
        out2 = gpu.daq_quantize_ln(dev(x), R, None, None, 1, 1e-6, want_h=False)
        assert np.array_equal(host(out2["q"]), host(out["q"]))


def test_layernorm_modulate_daq_full_size(gpu, orc):
    M, K = 16384, 1152
    say("ln+daq full size", M, K)
    x = workload.activations(M, K, "ln-full", sigma=3.0)
    g = workload.rng("ln-full")
    sc = (g.standard_normal((M // 256, K)) * 0.3).astype(np.float16)
    sh = (g.standard_normal((M // 256, K)) * 0.5).astype(np.float16)
    out = gpu.daq_quantize_ln(dev(x), 1, dev(sh), dev(sc), 256, 1e-6, want_h=True)
    h = host(out["h"])
    ref = orc.layernorm_modulate(x, sh, sc, 256, 1e-6)
    assert (np.abs(h.astype(np.float64) - ref.astype(np.float64)) <= _ln_tolerance(x, sh, sc, 256, ref)).all()
    assert (h.view(np.uint16) != ref.view(np.uint16)).mean() < 0.01
    q_ref, s_ref = orc.daq(h, 1, nthreads=16)
    assert np.array_equal(host(out["q"]), q_ref)
    assert np.array_equal(host(out["scales"]).view(np.uint32), s_ref.view(np.uint32))


# ------------------------------------------------------------------ rest of the plan space

@pytest.mark.parametrize("M,K,R,cg", [(512, 1152, 256, 128), (64, 4608, 16, 8), (37, 64, 37, 16), (96, 384, 1, 32), (1024, 1152, 1024, 288)])
def test_daq_channel_groups(gpu, orc, M, K, R, cg):
    say("daq channel groups", M, K, R, cg)
    x = workload.activations(M, K, "daqcg", R, cg, sigma=1.3)
    q_ref, a_ref = orc.daq_cg(x, R, cg, nthreads=8)
    q, a = gpu.daq_quantize_cg(dev(x), R, cg)
    assert np.array_equal(host(a).view(np.uint32), a_ref.view(np.uint32))
    assert np.array_equal(host(q), q_ref)


GROUPED_CASES = [
    # M, K, N, R, group, code range, storage, act_group
    (384, 1152, 256, 1, 64, (-4, 3), 8, 0),        # W3 held as int8
    (300, 1152, 200, 1, 128, (-32, 31), 8, 0),     # W6, ragged tile edges
    (256, 1152, 384, 64, 288, (-127, 127), 8, 0),  # W8 with group scales, per-sample row scales
    (256, 1152, 128, 1, 32, (-15, 15), 8, 0),      # 4-bit codes minus their zero points
    (512, 1152, 256, 256, 128, (-8, 7), 4, 128),   # packed 4-bit, one activation scale per image and channel group
    (512, 1152, 256, 128, 128, (-32, 31), 8, 128), # W6 with channel-group activation scales
    (256, 4608, 128, 128, 128, (-4, 3), 8, 128),   # long K: 36 groups
    (40, 96, 24, 4, 32, (-4, 3), 8, 32),           # neither K nor R fit the pipelined kernel: generic kernel
    (128, 4608, 64, 128, 64, (-8, 7), 4, 64),      # 72 groups: more than the kernel's scale table holds
]


@pytest.mark.parametrize("M,K,N,R,group,rng_,storage,act_group", GROUPED_CASES)
def test_grouped_layer(gpu, orc, M, K, N, R, group, rng_, storage, act_group):
    say("grouped", M, K, N, R, group, rng_, storage, act_group)
    g = workload.rng("grouped", M, K, N, group, storage, act_group)
    x = workload.activations(M, K, "grouped", group, storage, sigma=0.8)
    codes = g.integers(rng_[0], rng_[1] + 1, (N, K), dtype=np.int8)
    s_w = workload.w4_scales_group(N, K, group, "grouped")
    bias = workload.bias(N, "grouped")
    if act_group:
        q_ref, a_ref = orc.daq_cg(x, R, act_group, nthreads=8)
    else:
        q_ref, a_ref = orc.daq(x, R, nthreads=8)
    P_ref = orc.gemm_i8g(q_ref, codes, group, nthreads=16)
    y_ref = orc.epilogue_cg(P_ref, a_ref, R, s_w, bias) if act_group else orc.epilogue_w4(P_ref, a_ref, R, s_w, bias)
    wd = dev(gpu.ql_pack_w4_host(codes)) if storage == 4 else dev(codes)
    out = gpu.qlinear_grouped(dev(x), R, wd, dev(s_w), group, dev(bias), act_group=act_group, storage=storage, debug=True)
    assert np.array_equal(host(out["q"]), q_ref)
    assert np.array_equal(host(out["s_a"]).view(np.uint32), a_ref.view(np.uint32))
    assert np.array_equal(host(out["P"]), P_ref)
    assert assert_y_close(host(out["y"]), y_ref) == 0
    y2 = gpu.qlinear_grouped(dev(x), R, wd, dev(s_w), group, dev(bias), act_group=act_group, storage=storage)
    assert np.array_equal(host(y2).view(np.uint16), host(out["y"]).view(np.uint16))


def test_gptq_asymmetric_codes_through_the_grouped_layer(gpu, orc):
    """Step 2 end to end on synthetic data: GPTQ with per-group scale and zero point (host), zero points folded into the
    codes, dense 3-bit storage and back, then the grouped layer against the oracle on the same codes."""
    say("gptq asym -> grouped layer")
    M, K, N, group = 256, 256, 64, 64
    g = workload.rng("gptq-e2e")
    W = (g.standard_normal((N, K)) * 0.05 + 0.01).astype(np.float32)
    X = workload.activations(512, K, "gptq-e2e-x").astype(np.float64)
    codes, scales, zeros = gpu.gptq_quantize_host(W, X.T @ X, 3, group, symmetric=False, scale_fp16=True)
    diff = gpu.zero_point_fold_host(codes, zeros, group)
    assert diff.min() >= -7 and diff.max() <= 7
    stored = gpu.pack_bits_host(codes, 3)
    assert np.array_equal(gpu.unpack_bits_host(stored, 3, K), codes)
    x = workload.activations(M, K, "gptq-e2e-a")
    s_w = scales.astype(np.float16)
    q_ref, a_ref = orc.daq(x, 1)
    y_ref = orc.epilogue_w4(orc.gemm_i8g(q_ref, diff, group), a_ref, 1, s_w, None)
    y = gpu.qlinear_grouped(dev(x), 1, dev(diff), dev(s_w), group, None)
    assert assert_y_close(host(y), y_ref) == 0
    # and the quantized layer does approximate the float layer it came from
    yf = x.astype(np.float64) @ W.astype(np.float64).T
    rel = np.linalg.norm(host(y).astype(np.float64) - yf) / np.linalg.norm(yf)
    assert rel < 0.6, rel      # 3-bit weights: a gross-scale sanity bound, not parity


# ------------------------------------------------------------------ plan runner

def test_plan_runner_small_mixed_plan(gpu, orc):
    import torch
    M, R = 320, 1
    shapes = [("a", 256, 384, 8), ("b", 384, 256, 4), ("c", 256, 200, 4), ("d", 128, 128, 8), ("e", 1152, 96, 8)]
    layers, xs, refs = [], [], []
    for name, K, N, bits in shapes:
        lw = workload.layer_weights(name, K, N, bits, "plan")
        x = workload.activations(M, K, "plan", name)
        if bits == 8:
            refs.append(orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], lw["bias"], want_debug=False)["y"])
            w = dev(lw["w"])
        else:
            refs.append(orc.qlinear_w4a8(x, R, orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"], want_debug=False)["y"])
            w = dev(gpu.ql_pack_w4_host(lw["w"]))
        layers.append(dict(K=K, N=N, bits=bits, w=w, w_scale=dev(lw["s_w"]), bias=dev(lw["bias"])))
        xs.append(dev(x))
    say("plan create/run", len(layers), "layers")
    plan = gpu.Plan(layers, M_max=512)
    ys = [torch.zeros((M, l["N"]), dtype=torch.float16, device="cuda") for l in layers]
    ws = gpu.workspace(max(plan.workspace_bytes(M, R), plan.workspace_bytes(M, 64)))
    for rep in range(2):
        plan.run(xs, ys, M, R, ws)
        torch.cuda.synchronize()
        for y, ref in zip(ys, refs):
            assert assert_y_close(host(y), ref) == 0
    # per-sample scales through the same plan
    plan.run(xs, ys, M, 64, ws)
    x0 = workload.activations(M, 256, "plan", "a")
    lw0 = workload.layer_weights("a", 256, 384, 8, "plan")
    ref0 = orc.qlinear_w8a8(x0, 64, lw0["w"], lw0["s_w"], lw0["bias"], want_debug=False)["y"]
    assert assert_y_close(host(ys[0]), ref0) == 0
    plan.close()


def test_plan_run_ex_one_block_with_glue_and_percentile_daq(gpu, orc):
    """One DiT block through the plan walk: qkv plain, proj and fc2 with gated residual, fc1 with GELU; then the same
    block with the percentile DAQ at 6 activation bits."""
    import torch
    M, R, tokens = 512, 1, 256
    g = workload.rng("plan-ex")
    specs = [("qkv", 1152, 384, 8, 128), ("proj", 1152, 384, 4, 288), ("fc1", 1152, 512, 8, 128), ("fc2", 512, 384, 16, 0)]
    res = g.standard_normal((M, 384), dtype=np.float32).astype(np.float16)
    gate = g.standard_normal((M // tokens, 384), dtype=np.float32).astype(np.float16)
    fus = [None, dict(residual=dev(res), gate=dev(gate), gate_rows=tokens), dict(act=gpu.ACT_GELU_TANH),
           dict(residual=dev(res), gate=dev(gate), gate_rows=tokens)]
    layers, xs, hosts = [], [], []
    for name, K, N, bits, group in specs:
        x = workload.activations(M, K, "plan-ex", name)
        xs.append(x)
        if bits == 16:
            w = workload.f16_weights(N, K, "plan-ex")
            b = workload.bias(N, "plan-ex", name)
            hosts.append(dict(w=w, bias=b))
            layers.append(dict(K=K, N=N, bits=16, w=dev(w), w_scale=None, bias=dev(b)))
            continue
        lw = workload.layer_weights(name, K, N, bits, "plan-ex")
        if bits == 4:
            lw = dict(lw, s_w=workload.w4_scales_group(N, K, group, "plan-ex"))
        hosts.append(lw)
        layers.append(dict(K=K, N=N, bits=bits, group=group, w=dev(lw["w"]) if bits == 8 else dev(gpu.ql_pack_w4_host(lw["w"])),
                           w_scale=dev(lw["s_w"]), bias=dev(lw["bias"])))
    plan = gpu.Plan(layers, M_max=M)
    ys = [torch.zeros((M, l["N"]), dtype=torch.float16, device="cuda") for l in layers]
    ws = gpu.workspace(plan.workspace_bytes(M, R))
    xd = [dev(x) for x in xs]
    for p_ppm, a_bits in ((None, 8), (990000, 6)):
        say("plan_run_ex", p_ppm, a_bits)
        plan.run_ex(xd, ys, M, R, ws, fusions=fus, p_ppm=p_ppm, a_bits=a_bits)
        torch.cuda.synchronize()
        for i, (name, K, N, bits, group) in enumerate(specs):
            f = fus[i] or {}
            r = res if "residual" in f else None
            gt = gate if "gate" in f else None
            if bits == 16:
                h = orc.linear_f16(xs[i], hosts[i]["w"], hosts[i]["bias"], nthreads=8)
                ref = orc.block_glue(h.astype(np.float32), residual=r, gate=gt, gate_rows=tokens)
                tol = _f16_tolerance(xs[i], hosts[i]["w"], h) * np.abs(np.repeat(gate.astype(np.float64), tokens, 0)) \
                    + 2.0 ** -10 * np.abs(ref.astype(np.float64)) + 2.0 ** -24
                assert (np.abs(host(ys[i]).astype(np.float64) - ref.astype(np.float64)) <= tol).all()
                continue
            q, s = orc.daq(xs[i], R) if p_ppm is None else orc.daq_robust(xs[i], R, p_ppm=p_ppm, a_bits=a_bits)
            if bits == 8:
                u = orc.dequant_w8(orc.gemm_i8(q, hosts[i]["w"], nthreads=8), s, R, hosts[i]["s_w"], hosts[i]["bias"])
            else:
                u = orc.dequant_w4(orc.gemm_w4g(q, orc.pack_w4(hosts[i]["w"]), group, nthreads=8), s, R, hosts[i]["s_w"], hosts[i]["bias"])
            ref = orc.block_glue(u, act=f.get("act", 0), residual=r, gate=gt, gate_rows=tokens)
            if f.get("act", 0) == 0:
                assert assert_y_close(host(ys[i]), ref) == 0
            else:
                assert_y_close(host(ys[i]), ref)       # GELU alone: within the fp16 tolerance
    plan.close()


def test_c5_plan_stack_m16384_sampled(gpu, orc):
    """The 112-layer stack under the seeded bit plan at full size; the oracle checks sampled rows of sampled layers."""
    import torch
    M, R = 16384, 1
    plan_desc = workload.bit_plan()
    sig = float(workload.sigma_schedule(25)[3])
    x_by_type = {name: workload.activations(M, K, "c5", name, sigma=sig) for name, K, N in workload.BLOCK_LAYERS}
    xd = {k: dev(v) for k, v in x_by_type.items()}
    yd = {name: torch.empty((M, N), dtype=torch.float16, device="cuda") for name, K, N in workload.BLOCK_LAYERS}
    layers, host_w = [], {}
    for i, p in enumerate(plan_desc):
        lw = workload.layer_weights(p["name"], p["K"], p["N"], p["bits"], "c5", p["block"])
        w = dev(lw["w"]) if p["bits"] == 8 else dev(gpu.ql_pack_w4_host(lw["w"]))
        layers.append(dict(K=p["K"], N=p["N"], bits=p["bits"], w=w, w_scale=dev(lw["s_w"]), bias=dev(lw["bias"])))
        host_w[i] = lw
    plan = gpu.Plan(layers, M_max=M)
    ws = gpu.workspace(plan.workspace_bytes(M, R))
    check = [0, 1, 2, 3, 14, 15, 57, 110, 111]   # includes W4 and W8 layers of every type
    rows = np.sort(workload.rng("c5rows").choice(M, size=48, replace=False))
    rows[0], rows[-1] = 0, M - 1
    idx = torch.from_numpy(rows).cuda()
    # give every checked layer its own output buffer so the run can be compared afterwards
    x_in = [xd[p["name"]] for p in plan_desc]
    y_out = [yd[p["name"]] for p in plan_desc]
    for i in check:
        y_out[i] = torch.empty((M, plan_desc[i]["N"]), dtype=torch.float16, device="cuda")
    say("C5 plan run", len(layers), "layers", sum(p["bits"] == 4 for p in plan_desc), "at W4")
    plan.run(x_in, y_out, M, R, ws)
    torch.cuda.synchronize()
    for i in check:
        p, lw = plan_desc[i], host_w[i]
        say("C5 check layer", i, p["name"], p["bits"])
        xs = x_by_type[p["name"]][rows]
        if p["bits"] == 8:
            ref = orc.qlinear_w8a8(xs, 1, lw["w"], lw["s_w"], lw["bias"], nthreads=16, want_debug=False)["y"]
        else:
            ref = orc.qlinear_w4a8(xs, 1, orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"], nthreads=16,
                                   want_debug=False)["y"]
        assert assert_y_close(host(y_out[i][idx]), ref) == 0
    plan.close()
