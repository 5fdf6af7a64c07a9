"""Pins for the oracle's percentile-clipped DAQ (eq. (4) as printed, activation width from Step 6): hand-worked
cases, the special case that reduces to the absmax quantizer, numpy's nearest-rank percentile, the defining
property of an order statistic checked by brute force, and invariants of the quantizer.  CPU only.
"""
import numpy as np
import pytest

import workload


def f16(a):
    return np.asarray(a, dtype=np.float16)


def test_worked_example_p90_of_ten_values(orc):
    # magnitudes sorted: 0.5 1 1.5 2 2.5 3 3.5 4 8 100 ; n = 10, p = 90 % -> k = 9 -> tau = 8
    x = f16([[4.0, -100.0, 0.5, -1.0, 8.0, 1.5, -2.0, 2.5, 3.0, -3.5]])
    q, s = orc.daq_robust(x, 1, p_ppm=900000, a_bits=8)
    assert s[0] == np.float32(8.0) / np.float32(127.0)
    # 8 -> 127, -100 is clipped to -8 -> -127; 4/alpha = 63.5 (exact in fp32? 4/(8/127) rounds to 63.5) -> tie to even 64
    assert q[0, 4] == 127 and q[0, 1] == -127
    want = np.rint(np.clip(x.astype(np.float32), -8, 8) / s[0]).astype(np.int8)
    assert np.array_equal(q, want)


def test_worked_example_four_bit_codes(orc):
    # a_bits = 4 -> qmax = 7; tau = max (p = 100 %) = 7 -> alpha = 1 -> codes are the rounded values, ties to even
    x = f16([[7.0, -2.5, 3.5, 0.5, -0.5, 1.5, -7.0, 6.49]])
    q, s = orc.daq_robust(x, 1, p_ppm=1000000, a_bits=4)
    assert s[0] == np.float32(1.0)
    assert q.tolist() == [[7, -2, 4, 0, 0, 2, -7, 6]]


@pytest.mark.parametrize("R", [1, 4, 16])
def test_p100_b8_is_the_absmax_quantizer(orc, R):
    x = workload.activations(16, 256, "robust-pin", R, sigma=1.3)
    q0, s0 = orc.daq(x, R)
    q1, s1 = orc.daq_robust(x, R, p_ppm=1000000, a_bits=8)
    assert np.array_equal(q0, q1) and np.array_equal(s0.view(np.uint32), s1.view(np.uint32))


@pytest.mark.parametrize("p_ppm", [999000, 990000, 900000, 500000, 1])
@pytest.mark.parametrize("R,K", [(1, 1152), (8, 96), (32, 64)])
def test_tau_is_numpys_nearest_rank_percentile(orc, p_ppm, R, K):
    M = 32
    x = workload.activations(M, K, "robust-np", p_ppm, R, sigma=2.0)
    _, s = orc.daq_robust(x, R, p_ppm=p_ppm, a_bits=8)
    mag = np.abs(x.astype(np.float64)).reshape(M // R, R * K)
    n = R * K
    k = -(-n * p_ppm // 1000000)            # ceil in integers
    # numpy's inverted_cdf is the nearest-rank definition; ask for a probability safely inside rank k's interval
    prob = (k - 0.5) / n
    tau = np.quantile(mag, prob, axis=1, method="inverted_cdf")
    want = np.where(tau == 0, np.float32(1), tau.astype(np.float32) / np.float32(127)).astype(np.float32)
    assert np.array_equal(s.view(np.uint32), want.view(np.uint32))


def test_tau_has_the_defining_property_of_the_kth_order_statistic(orc):
    # brute force on a block with many ties: at least k magnitudes are <= tau, fewer than k are < tau
    g = np.random.default_rng(251111446)
    x = f16(g.integers(-6, 7, size=(6, 50)) * 0.25)
    for p_ppm in (999000, 800000, 333333, 20000):
        _, s = orc.daq_robust(x, 2, p_ppm=p_ppm, a_bits=8)
        for b in range(3):
            mag = np.abs(x[2 * b:2 * b + 2].astype(np.float64)).ravel()
            n = mag.size
            k = -(-n * p_ppm // 1000000)
            tau = float(s[b]) * 127 if not (mag <= 0).sum() >= k else 0.0
            if tau == 0.0:
                assert s[b] == 1.0
                continue
            cands = np.unique(mag)
            tau_v = cands[np.argmin(np.abs(cands - tau))]     # alpha*127 carries one rounding; snap to the data
            assert (mag <= tau_v).sum() >= k and (mag < tau_v).sum() < k


def test_clipped_elements_get_full_scale_codes_and_the_rest_obey_the_error_bound(orc):
    x = workload.activations(64, 1152, "robust-bound", sigma=1.0)
    for a_bits in (8, 6, 4, 2):
        qmax = (1 << (a_bits - 1)) - 1
        q, s = orc.daq_robust(x, 1, p_ppm=990000, a_bits=a_bits)
        xf = x.astype(np.float64)
        alpha = s.astype(np.float64)[:, None]
        tau = alpha * qmax
        assert np.abs(q).max() <= qmax
        over = np.abs(xf) > tau * (1 + 1e-6)
        # at most 1 % of each row lies above the 99th percentile
        assert (over.sum(axis=1) <= 1152 - (-(-1152 * 990000 // 1000000))).all()
        assert np.array_equal(q[over], (np.sign(xf[over]) * qmax).astype(np.int8))
        inside = ~over
        err = np.abs(np.clip(xf, -tau, tau) - alpha * q)
        assert (err[inside] <= (alpha * (0.5 + 2.0 ** -16) * np.ones_like(xf))[inside]).all()


def test_invariants_zero_block_sign_and_power_of_two(orc):
    x = workload.activations(8, 128, "robust-inv", sigma=0.7)
    x[2] = 0
    q, s = orc.daq_robust(x, 1, p_ppm=950000, a_bits=5)
    assert s[2] == 1.0 and not q[2].any()
    qn, sn = orc.daq_robust(-x, 1, p_ppm=950000, a_bits=5)
    assert np.array_equal(qn, -q) and np.array_equal(sn, s)
    q4, s4 = orc.daq_robust(f16(x.astype(np.float32) * 4), 1, p_ppm=950000, a_bits=5)
    assert np.array_equal(q4, q)
    nz = np.arange(8) != 2
    assert np.array_equal(s4[nz], s[nz] * np.float32(4))
    # more than p of the block is zero -> tau = 0 -> alpha = 1, all codes 0 (the non-zero few are clipped to 0)
    z = np.zeros((1, 100), np.float16)
    z[0, :5] = 3.0
    qz, sz = orc.daq_robust(z, 1, p_ppm=900000, a_bits=8)
    assert sz[0] == 1.0 and not qz.any()


def test_bad_arguments_are_refused(orc):
    x = np.zeros((4, 8), np.float16)
    for kw in (dict(p_ppm=0), dict(p_ppm=1000001), dict(a_bits=1), dict(a_bits=9)):
        with pytest.raises(ValueError):
            orc.daq_robust(x, 1, **kw)


# ---------------------------------------------------------------- weight groups of other sizes (Step 2, Algorithm 1)

def _w4_case(M, K, N, seed):
    g = workload.rng("w4g-pin", seed)
    q = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    w = g.integers(-8, 8, size=(N, K), dtype=np.int8)
    return q, w


@pytest.mark.parametrize("group", [32, 64, 96, 128, 192, 288])
def test_grouped_partials_against_numpy_block_sums(orc, group):
    M, K, N = 5, 1152, 7
    q, w = _w4_case(M, K, N, group)
    P = orc.gemm_w4g(q, orc.pack_w4(w), group)
    G = K // group
    want = np.einsum("mgk,ngk->mgn", q.reshape(M, G, group).astype(np.int64), w.reshape(N, G, group).astype(np.int64))
    assert np.array_equal(P, want.astype(np.int32))
    # the groups partition K: their sum is the plain int8 product of the same codes
    assert np.array_equal(P.sum(axis=1), orc.gemm_i8(q, w))


def test_group128_is_the_fixed_group_function_and_one_hot_group_membership(orc):
    q, w = _w4_case(4, 256, 6, "g128")
    assert np.array_equal(orc.gemm_w4g(q, orc.pack_w4(w), 128), orc.gemm_w4g128(q, orc.pack_w4(w)))
    # a single non-zero weight at k lands in group k // group only
    for group, k in ((32, 95), (64, 64), (192, 191), (288, 288)):
        K = 576
        w1 = np.zeros((1, K), np.int8)
        w1[0, k] = -8
        q1 = np.full((1, K), 3, np.int8)
        P = orc.gemm_w4g(q1, orc.pack_w4(w1), group)
        want = np.zeros((1, K // group, 1), np.int32)
        want[0, k // group, 0] = -24
        assert np.array_equal(P, want)


def test_grouped_epilogue_with_equal_power_of_two_scales_equals_the_per_channel_path(orc):
    M, K, N, group = 6, 576, 5, 192
    q, w = _w4_case(M, K, N, "epi")
    s_a = np.full((M,), 0.5, np.float32)
    P = orc.gemm_w4g(q, orc.pack_w4(w), group)
    sw = np.full((N, K // group), 0.25, np.float16)
    bias = np.zeros((N,), np.float16)
    y4 = orc.epilogue_w4(P, s_a, 1, sw, bias)
    y8 = orc.epilogue_w8(orc.gemm_i8(q, w), s_a, 1, np.full((N,), 0.25, np.float32), bias)
    assert np.array_equal(y4.view(np.uint16), y8.view(np.uint16))


# ---------------------------------------------------------------- block glue folded into the epilogue

def test_dequant_values_round_to_the_plain_epilogues(orc):
    g = workload.rng("glue-dq")
    M, K, N = 6, 256, 10
    q = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    w8 = g.integers(-127, 128, size=(N, K), dtype=np.int8)
    w4 = g.integers(-8, 8, size=(N, K), dtype=np.int8)
    s_a = g.uniform(0.01, 0.1, M).astype(np.float32)
    bias = workload.bias(N, "glue")
    acc = orc.gemm_i8(q, w8)
    sw8 = workload.w8_scales(N, "glue")
    assert np.array_equal(orc.float_to_half(orc.dequant_w8(acc, s_a, 1, sw8, bias)), orc.epilogue_w8(acc, s_a, 1, sw8, bias).view(np.uint16))
    P = orc.gemm_w4g128(q, orc.pack_w4(w4))
    sw4 = workload.w4_scales(N, K, "glue")
    assert np.array_equal(orc.float_to_half(orc.dequant_w4(P, s_a, 1, sw4, None)), orc.epilogue_w4(P, s_a, 1, sw4, None).view(np.uint16))
    # no activation, gate or residual: the glue is the rounding alone
    u = orc.dequant_w8(acc, s_a, 1, sw8, bias)
    assert np.array_equal(orc.block_glue(u).view(np.uint16), orc.float_to_half(u))


def test_gelu_against_the_tanh_formula_and_its_closed_form_values(orc):
    import math
    u = np.array([[0.0, 1.0, -1.0, 3.0, -3.0, 0.5, -8.0, 10.0, -0.0, 1e-4]], np.float32)
    y = orc.block_glue(u, act=1).astype(np.float64)
    want = np.array([0.5 * x * (1.0 + math.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3))) for x in u[0].astype(np.float64)])
    assert np.allclose(y[0], want, rtol=2.0 ** -10, atol=2.0 ** -24)
    # published values of the tanh form: gelu(1) = 0.841192, gelu(-1) = -0.158808, gelu(3) = 2.996363
    assert abs(y[0, 1] - 0.841192) < 5e-4 and abs(y[0, 2] + 0.158808) < 2e-4 and abs(y[0, 3] - 2.996363) < 2e-3
    assert y[0, 0] == 0.0 and y[0, 7] == 10.0 and abs(y[0, 6]) < 1e-6
    # gelu(x) - gelu(-x) = x for every x (sigmoid(t) + sigmoid(-t) = 1)
    xs = workload.rng("gelu-sym").uniform(-6, 6, size=(1, 4096)).astype(np.float32)
    a = orc.block_glue(xs, act=1).astype(np.float64)
    b = orc.block_glue(-xs, act=1).astype(np.float64)
    assert np.allclose(a - b, xs, rtol=2e-3, atol=2e-3)


def test_gate_and_residual_hand_worked_and_broadcast(orc):
    u = np.array([[1.0, 2.0, -4.0], [0.5, 0.25, 8.0], [1.0, 1.0, 1.0], [3.0, -3.0, 0.0]], np.float32)
    res = np.array([[10, 20, 30], [1, 1, 1], [0, 0, 0], [-1, -2, -3]], np.float16)
    gate = np.array([[2.0, 0.5, -1.0], [0.0, 1.0, 4.0]], np.float16)      # one gate row per 2 rows
    y = orc.block_glue(u, residual=res, gate=gate, gate_rows=2)
    want = np.array([[12, 21, 34], [2, 1.125, -7], [0, 1, 4], [-1, -5, -3]], np.float16)
    assert np.array_equal(y, want)
    assert np.array_equal(orc.block_glue(u, residual=res), (u + res.astype(np.float32)).astype(np.float16))
    assert np.array_equal(orc.block_glue(u, gate=gate, gate_rows=2), (u * np.repeat(gate.astype(np.float32), 2, 0)).astype(np.float16))
    # the layer's value is rounded to fp16 BEFORE the gated addition: 1 + 2^-11 rounds to 1 first, so adding 2^-11 gives
    # 1 + 2^-11 -> 1 (tie to even), not the 1 + 2^-10 a single rounding of the exact sum would give
    u2 = np.array([[1.0 + 2.0 ** -11]], np.float32)
    r2 = np.array([[2.0 ** -11]], np.float16)
    assert orc.block_glue(u2, residual=r2)[0, 0] == np.float16(1.0)
    with pytest.raises(ValueError):
        orc.block_glue(u, gate=gate, gate_rows=3)


# ---------------------------------------------------------------- layers the plan leaves in FP16

def test_fp16_layer_against_numpy_float64_and_closed_forms(orc):
    g = workload.rng("f16-layer")
    M, K, N = 9, 200, 11
    x = g.standard_normal((M, K), dtype=np.float32).astype(np.float16)
    w = (g.standard_normal((N, K), dtype=np.float32) * 0.1).astype(np.float16)
    b = workload.bias(N, "f16")
    y = orc.linear_f16(x, w, b)
    want = (x.astype(np.float64) @ w.astype(np.float64).T + b.astype(np.float64)).astype(np.float32).astype(np.float16)
    assert np.array_equal(y.view(np.uint16), want.view(np.uint16))
    # identity weights copy the input; a row of ones sums it; transposing the operands' roles is caught by N != M != K
    eye = np.eye(K, dtype=np.float16)
    assert np.array_equal(orc.linear_f16(x, eye), x)
    ones = np.ones((1, K), np.float16)
    s = orc.linear_f16(x, ones)[:, 0].astype(np.float64)
    assert np.allclose(s, x.astype(np.float64).sum(axis=1), rtol=2.0 ** -10, atol=1e-6)
    # an exactly representable case with cancellation that fp32 running sums would lose: 2048 + 1 - 2048 = 1
    xc = np.array([[2048.0, 1.0, -2048.0]], np.float16)
    assert orc.linear_f16(xc, np.ones((1, 3), np.float16))[0, 0] == np.float16(1.0)


# ---------------------------------------------------------------- fixtures under tests/golden

def _golden(name):
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", name)) as f:
        return [l.strip() for l in f if l.strip() and not l.startswith("#")]


def test_golden_final_plan_counts_match_the_synthetic_final_plan():
    import collections
    want_bits, want_groups, total = {}, {}, 0
    for l in _golden("final_plan_counts.txt"):
        p = l.split()
        if p[0] == "layers":
            total = int(p[1])
        elif p[0] == "bits":
            want_bits[int(p[1])] = int(p[2])
        else:
            want_groups[int(p[1])] = int(p[2])
    assert sum(want_bits.values()) == total == sum(want_groups.values()) == 113
    plan = workload.final_plan()
    # the 113th layer (final projection) is outside the block linears; it is taken to be an FP16, group-288 entry
    got = collections.Counter(l["bits"] for l in plan)
    assert got[4] == want_bits[4] and got[8] == want_bits[8] and got[16] == want_bits[16] - 1 and len(plan) == total - 1
    assert all(l["group"] in want_groups for l in plan if l["bits"] == 4)
    assert all(l["K"] % l["group"] == 0 for l in plan if l["bits"] == 4)


def test_golden_hand_worked_daq_rows(orc):
    for l in _golden("daq_hand_worked.txt"):
        parts = [p.strip() for p in l.split("|")]
        if parts[0] == "p90":
            x = f16([[float(v) for v in parts[1].split()]])
            q, s = orc.daq_robust(x, 1, p_ppm=900000, a_bits=8)
            tau = float(parts[2].split()[1])
            assert s[0] == np.float32(tau) / np.float32(127)
            for item in parts[3:]:
                idx = int(item[item.index("[") + 1:item.index("]")])
                assert q[0, idx] == int(item.split()[-1])
            continue
        alpha, xs, codes = float(parts[0]), [float(v) for v in parts[1].split()], [int(v) for v in parts[2].split()]
        q, s = orc.daq(f16([xs]), 1)
        assert s[0] == np.float32(alpha) and q.tolist() == [codes]


# ------------------------------------------------------------------ LayerNorm + adaptive modulation (Step 3, Section 6)

def test_layernorm_modulate_against_torch_and_closed_forms(orc):
    import torch
    g = workload.rng("ln-pin")
    x = workload.activations(12, 96, "ln-pin", sigma=3.0)
    # the library routine, in float64 (a different implementation of the same definition)
    want = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (96,), eps=1e-6).numpy()
    got = orc.layernorm_modulate(x, eps=1e-6).astype(np.float64)
    assert np.abs(got - want).max() <= 2.0 ** -11 * np.abs(want).max() + 1e-12      # one rounding to binary16
    assert np.array_equal(orc.layernorm_modulate(x, eps=1e-6), want.astype(np.float32).astype(np.float16))
    # closed form: a row of +a, -a has mean 0 and variance a^2 -> +-1 / sqrt(1 + eps / a^2)
    row = np.tile(np.array([2.0, -2.0], np.float16), 8)[None]
    h = orc.layernorm_modulate(row, eps=0.0)
    assert np.array_equal(h, np.tile(np.array([1.0, -1.0], np.float16), 8)[None])
    # modulation: h = n (1 + scale) + shift with per-image vectors; scale = 1, shift = 3 on the +-1 row gives 5 and 1
    sc = np.ones((1, 16), np.float16)
    sh = np.full((1, 16), 3.0, np.float16)
    h = orc.layernorm_modulate(np.repeat(row, 4, 0), shift=sh, scale=sc, rows_per_mod=4, eps=0.0)
    assert np.array_equal(h, np.repeat(np.tile(np.array([5.0, 1.0], np.float16), 8)[None], 4, 0))
    # invariances with eps = 0: adding a constant to a row or scaling it by a power of two changes nothing
    x2 = np.round(g.standard_normal((5, 64)) * 4) / 4
    a = orc.layernorm_modulate(x2.astype(np.float16), eps=0.0)
    assert np.array_equal(a, orc.layernorm_modulate((x2 + 8.0).astype(np.float16), eps=0.0))
    assert np.array_equal(a, orc.layernorm_modulate((x2 * 4.0).astype(np.float16), eps=0.0))
    # rows of different images take different modulation rows (a swapped index would show)
    sc = (g.standard_normal((3, 64)) * 0.3).astype(np.float16)
    sh = (g.standard_normal((3, 64)) * 0.5).astype(np.float16)
    x3 = workload.activations(6, 64, "ln-mod")
    h = orc.layernorm_modulate(x3, shift=sh, scale=sc, rows_per_mod=2).astype(np.float64)
    n = torch.nn.functional.layer_norm(torch.from_numpy(x3.astype(np.float64)), (64,), eps=1e-6).numpy()
    for m in range(6):
        ref = n[m] * (1.0 + sc[m // 2].astype(np.float64)) + sh[m // 2].astype(np.float64)
        assert np.abs(h[m] - ref).max() <= 2.0 ** -10 * np.abs(ref).max()


# ------------------------------------------------------------------ rest of the plan space: int8-held codes with group scales,
# channel-group activation scales (eq. (4)), dense 3/6-bit storage

def test_gemm_i8g_against_numpy_block_sums_and_the_plain_gemm(orc):
    g = workload.rng("i8g")
    M, N, K = 9, 7, 96
    q = g.integers(-127, 128, (M, K), dtype=np.int8)
    for lo, hi, group in ((-4, 4, 32), (-32, 32, 48), (-127, 128, 96), (-15, 16, 8)):
        w = g.integers(lo, hi, (N, K), dtype=np.int8)
        P = orc.gemm_i8g(q, w, group, nthreads=2)
        want = np.einsum("mgk,ngk->mgn", q.astype(np.int64).reshape(M, K // group, group), w.astype(np.int64).reshape(N, K // group, group))
        assert np.array_equal(P, want)
        assert np.array_equal(P.sum(axis=1), orc.gemm_i8(q, w))
    # one-hot weight: P[m, g, n] = q[m, k0] exactly in the group that holds k0
    w = np.zeros((N, K), np.int8)
    w[3, 50] = 1
    P = orc.gemm_i8g(q, w, 32)
    assert np.array_equal(P[:, 1, 3], q[:, 50].astype(np.int32)) and P.sum() == q[:, 50].astype(np.int64).sum()


def test_daq_cg_is_eq4_per_sample_and_channel_group(orc):
    # every (row block, channel group) sub-block with its own power-of-two maximum: the scales are exactly 2^j / 127
    M, K, R, cg = 8, 32, 4, 8
    x = np.zeros((M, K), np.float16)
    want = np.zeros((M // R, K // cg), np.float32)
    g = workload.rng("daqcg")
    for b in range(M // R):
        for c in range(K // cg):
            amax = 2.0 ** (b * 4 + c - 3)
            blk = g.uniform(-1, 1, (R, cg)) * amax * 0.9
            blk[g.integers(R), g.integers(cg)] = -amax
            x[b * R:(b + 1) * R, c * cg:(c + 1) * cg] = blk.astype(np.float16)
            want[b, c] = np.float32(amax) / np.float32(127.0)
    q, alpha = orc.daq_cg(x, R, cg)
    assert np.array_equal(alpha, want)
    assert (np.abs(q).reshape(M // R, R, K // cg, cg).max(axis=(1, 3)) == 127).all()
    # one channel group spanning all of K is the row-block DAQ; error bound of the quantizer per element
    q1, a1 = orc.daq_cg(x, R, K)
    q2, a2 = orc.daq(x, R)
    assert np.array_equal(q1, q2) and np.array_equal(a1[:, 0], a2)
    err = np.abs(x.astype(np.float64) - q * np.repeat(np.repeat(alpha.astype(np.float64), R, 0), cg, 1))
    assert (err <= np.repeat(np.repeat(alpha.astype(np.float64), R, 0), cg, 1) * (0.5 + 2.0 ** -16)).all()


def test_epilogue_cg_special_cases(orc):
    g = workload.rng("epicg")
    M, G, N, R = 8, 3, 5, 4
    P = g.integers(-50000, 50000, (M, G, N), dtype=np.int32)
    s_w = g.uniform(1e-2, 1e-1, (N, G)).astype(np.float16)
    bias = (g.standard_normal(N) * 0.02).astype(np.float16)
    # the same power-of-two scale for all groups of a block: multiplying by it commutes with every rounding, so the
    # result equals the row-scale epilogue with that scale (given a zero bias, where fma(f, a, 0) = f a)
    a_blk = np.array([2.0 ** -7, 2.0 ** -4], np.float32)
    alpha = np.repeat(a_blk[:, None], G, 1)
    assert np.array_equal(orc.epilogue_cg(P, alpha, R, s_w, None), orc.epilogue_w4(P, a_blk, R, s_w, None))
    # hand-worked: one group, P = 3, s_w = 0.5, alpha = 0.25, bias = 1  ->  3 * 0.125 + 1 = 1.375
    y = orc.epilogue_cg(np.array([[[3]]], np.int32), np.array([[0.25]], np.float32), 1, np.array([[0.5]], np.float16), np.array([1.0], np.float16))
    assert y[0, 0] == np.float16(1.375)
    # general case against float64 (every product and the short sum are far inside float64): within one fp16 step
    alpha = g.uniform(1e-3, 1e-1, (M // R, G)).astype(np.float32)
    y = orc.epilogue_cg(P, alpha, R, s_w, bias).astype(np.float64)
    ref = np.einsum("mgn,ng,mg->mn", P.astype(np.float64), s_w.astype(np.float64), np.repeat(alpha.astype(np.float64), R, 0)) + bias.astype(np.float64)
    assert (np.abs(y - ref) <= 2.0 ** -10 * np.abs(ref) + 1e-6).all()
    # a group's scale belongs to its own group: permuting alpha's groups changes the result
    assert not np.array_equal(orc.epilogue_cg(P, alpha[:, ::-1].copy(), R, s_w, bias), orc.epilogue_cg(P, alpha, R, s_w, bias))


def test_dense_bit_storage(orc):
    # literal: 3-bit codes 1, -1 (111b), 2, -4 (100b), 0, 3, -2 (110b), 1 -> bit stream LSB first
    codes = np.array([[1, -1, 2, -4, 0, 3, -2, 1]], np.int8)
    bits = "100" + "111" + "010" + "001" + "000" + "110" + "011" + "100"      # each code written LSB first
    want = np.array([[int(bits[i:i + 8][::-1], 2) for i in range(0, 24, 8)]], np.uint8)
    assert np.array_equal(orc.pack_bits(codes, 3), want)
    g = workload.rng("bits")
    for b in (3, 6, 5):
        c = g.integers(-(1 << (b - 1)), 1 << (b - 1), (5, 64), dtype=np.int8)
        p = orc.pack_bits(c, b)
        assert p.shape == (5, 64 * b // 8) and np.array_equal(orc.unpack_bits(p, b, 64), c)


def test_row_absmax_bits_hand_values_and_its_use_as_the_daq_threshold(orc):
    """Pins: literal bit patterns (0x3c00 = 1, 0x4248 = 3.140625, 0x0001 = the smallest subnormal, 0x7bff = 65504), sign
    ignored, zero row -> 0; and alpha = fp16(bits) / 127 is the scale orc.daq finds for that row on its own."""
    y = np.array([[0.5, -1.0, 0.25], [3.140625, -3.0, 0.0], [0.0, -0.0, 0.0], [6e-8, 0.0, -0.0], [-65504.0, 1.0, 2.0]], dtype=np.float16)
    assert orc.row_absmax_bits(y).tolist() == [0x3c00, 0x4248, 0, 0x0001, 0x7bff]
    g = workload.rng("rowmax-pin")
    x = (g.standard_normal((40, 64)) * 3).astype(np.float16)
    bits = orc.row_absmax_bits(x)
    _, s = orc.daq(x, 1)
    assert np.array_equal(s, (bits.astype(np.uint16).view(np.float16).astype(np.float32) / np.float32(127.0)))
