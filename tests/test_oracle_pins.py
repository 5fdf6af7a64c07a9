"""Pins for the CPU oracle: each test ties one part of it to something other than
itself: hand-worked cases, invariants of eq. (4), exact rational arithmetic
within the quantizer's error bound, brute force, closed forms, and library
routines for the special cases that reduce to them.  CPU only.
"""
from fractions import Fraction

import numpy as np
import pytest

import workload


def f16(a):
    return np.asarray(a, dtype=np.float16)


# ---------------------------------------------------------------- binary16 <-> binary32

def test_half_to_float_exhaustive_against_numpy(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = orc.half_to_float(bits)
    want = bits.view(np.float16).astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got.view(np.uint32)[~nan], want.view(np.uint32)[~nan])


def test_float_to_half_roundtrip_and_ties(orc):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = bits.view(np.float16).astype(np.float32)
    finite = np.isfinite(vals)
    # exact values come back unchanged
    assert np.array_equal(orc.float_to_half(vals[finite]), bits[finite])
    # the midpoint between neighbours a < b (both finite, same sign) goes to the even one
    pos = np.arange(0, 0x7bff, dtype=np.uint32).astype(np.uint16)
    a = pos.view(np.float16).astype(np.float64)
    b = (pos + np.uint16(1)).view(np.float16).astype(np.float64)
    mid = ((a + b) / 2).astype(np.float32)  # exact: needs 12 significant bits
    got = orc.float_to_half(mid)
    want = np.where(pos % 2 == 0, pos, pos + 1).astype(np.uint16)
    assert np.array_equal(got, want)
    # just above / below the midpoint
    up = np.nextafter(mid, np.float32(np.inf))
    dn = np.nextafter(mid, np.float32(-np.inf))
    assert np.array_equal(orc.float_to_half(up), (pos + 1).astype(np.uint16))
    assert np.array_equal(orc.float_to_half(dn), pos)
    # negative side mirrors
    assert np.array_equal(orc.float_to_half(-mid), want | np.uint16(0x8000))


def test_float_to_half_overflow_and_random_against_numpy(orc):
    edge = np.array([65504.0, 65519.996, 65520.0, 65536.0, 1e30, -65520.0, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                     2.0 ** -24, 2.0 ** -14, 0.0, -0.0, np.inf, -np.inf], dtype=np.float32)
    with np.errstate(over="ignore"):
        assert np.array_equal(orc.float_to_half(edge), edge.astype(np.float16).view(np.uint16))
        g = workload.rng("f2h")
        u = g.integers(0, 2 ** 32, size=400000, dtype=np.uint64).astype(np.uint32)
        f = u.view(np.float32)
        f = f[~np.isnan(f)]
        assert np.array_equal(orc.float_to_half(f), f.astype(np.float16).view(np.uint16))
        # concentrate on the binary16 range too
        f2 = (g.standard_normal(400000) * 10.0 ** g.uniform(-8, 5, 400000)).astype(np.float32)
        assert np.array_equal(orc.float_to_half(f2), f2.astype(np.float16).view(np.uint16))


# ---------------------------------------------------------------- eq. (4): the quantizer

def test_daq_hand_worked_rows(orc):
    # amax = 127 -> alpha = 1 exactly, so the codes are round-half-even of the inputs:
    # 1.5 -> 2, 2.5 -> 2, -0.5 -> -0, 3.5 -> 4, -2.5 -> -2
    q, s = orc.daq(f16([[1.5, 2.5, -0.5, 127.0, 3.5, -2.5, 126.5, 0.49]]), 1)
    assert s[0] == 1.0
    assert q.tolist() == [[2, 2, 0, 127, 4, -2, 126, 0]]
    # amax = 254 -> alpha = 2 exactly: codes = rne(x / 2); 1 -> 0.5 -> 0, 3 -> 1.5 -> 2, 5 -> 2.5 -> 2
    q, s = orc.daq(f16([[254.0, 1.0, 3.0, 5.0, -7.0, -254.0]]), 1)
    assert s[0] == 2.0
    assert q.tolist() == [[127, 0, 2, 2, -4, -127]]
    # amax = 63.5 -> alpha = 0.5 exactly: codes = rne(2x)
    q, s = orc.daq(f16([[63.5, 0.25, 0.75, -1.25, 10.0]]), 1)
    assert s[0] == 0.5
    assert q.tolist() == [[127, 0, 2, -2, 20]]


def test_daq_zero_block(orc):
    # all-zero block: scale 1, every code 0 (no 0/0)
    x = np.zeros((4, 24), np.float16)
    x[2:] = f16(3.0)
    q, s = orc.daq(x, 2)
    assert s[0] == 1.0 and not q[:2].any()
    assert q[2:].tolist() == [[127] * 24] * 2
    # negative zeros count as zero
    q, s = orc.daq(f16([[-0.0, 0.0]]), 1)
    assert s[0] == 1.0 and q.tolist() == [[0, 0]]


@pytest.mark.parametrize("R", [1, 4, 16])
def test_daq_power_of_two_scaling_and_sign(orc, R):
    # values kept in [2^-6, 2^6] so that x * 2^j stays a normal binary16 number for |j| <= 8
    g = workload.rng("p2", R)
    x = (g.standard_normal((16, 40)).astype(np.float32)).astype(np.float16)
    x = np.where(np.abs(x) < 2.0 ** -6, f16(2.0 ** -6), x)
    q0, s0 = orc.daq(x, R)
    for j in (-8, -3, 1, 5, 8):
        xs = (x.astype(np.float32) * np.float32(2.0 ** j)).astype(np.float16)
        assert np.array_equal(xs.astype(np.float32), x.astype(np.float32) * np.float32(2.0 ** j))
        q, s = orc.daq(xs, R)
        assert np.array_equal(q, q0)
        assert np.array_equal(s.view(np.uint32), (s0 * np.float32(2.0 ** j)).view(np.uint32))
    qn, sn = orc.daq(-x, R)
    assert np.array_equal(qn, -q0) and np.array_equal(sn, s0)


def test_daq_range_absmax_and_error_bound(orc):
    g = workload.rng("bound")
    for R in (1, 8, 32):
        x = workload.activations(32, 200, "bound", R, sigma=float(10.0 ** g.uniform(-3, 2)))
        q, s = orc.daq(x, R)
        assert q.min() >= -127 and q.max() <= 127
        xb = x.astype(np.float64).reshape(32 // R, R * 200)
        qb = q.astype(np.float64).reshape(32 // R, R * 200)
        amax = np.abs(xb).max(axis=1)
        # alpha = amax/127 to binary32 accuracy
        assert np.allclose(s.astype(np.float64), amax / 127.0, rtol=2.0 ** -23, atol=0)
        # the largest-magnitude element encodes to +-127
        idx = np.abs(xb).argmax(axis=1)
        assert np.all(np.abs(qb[np.arange(len(idx)), idx]) == 127)
        # mid-tread quantizer with step alpha: |x - alpha*q| <= alpha * (1/2 + 2^-16)
        err = np.abs(xb - s.astype(np.float64)[:, None] * qb)
        assert np.all(err <= s.astype(np.float64)[:, None] * (0.5 + 2.0 ** -16))


def test_daq_matches_exact_rational_rounding(orc):
    """code = round-half-even(127 x / amax) in exact arithmetic, except when that ratio lies
    within 2^-14 of a half-integer, where the two binary32 roundings may tip it either way."""
    x = workload.activations(6, 96, "rational", sigma=0.7)
    q, s = orc.daq(x, 1)
    near_tie = 0
    for m in range(x.shape[0]):
        row = [Fraction(float(v)) for v in x[m]]
        amax = max(abs(v) for v in row)
        for k, v in enumerate(row):
            t = 127 * v / amax
            lo = t.__floor__()
            frac = t - lo
            if abs(frac - Fraction(1, 2)) < Fraction(1, 2 ** 14):
                near_tie += 1
                assert int(q[m, k]) in (lo, lo + 1)
            else:
                assert int(q[m, k]) == (lo if frac < Fraction(1, 2) else lo + 1)
    assert near_tie < 8


def _fl32(fr):
    """Correctly rounded (nearest, ties to even) binary32 value of a positive rational, as a Fraction (normal range)."""
    e = 0
    while fr >= 2 ** 24:
        fr /= 2
        e += 1
    while fr < 2 ** 23:
        fr *= 2
        e -= 1
    n = fr.__floor__()
    rem = fr - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n % 2 == 1):
        n += 1
    return Fraction(n) * Fraction(2) ** e


def test_daq_divides_by_alpha_where_a_reciprocal_would_differ(orc):
    """Eq. (4) divides by alpha.  On the stored pairs the correctly rounded quotient and a multiplication by the rounded
    reciprocal give different codes; the expected code is derived here with exact rational arithmetic (two binary32
    roundings: alpha = fl(amax/127), t = fl(x/alpha), then round half to even), so an oracle that multiplied by
    1/alpha instead of dividing fails."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "daq_division_vs_reciprocal.txt")
    pairs = []
    for line in open(path):
        if line.startswith("#") or not line.strip():
            continue
        lhs, by_div, by_rcp = [t.strip() for t in line.split("|")]
        a, x = [int(t, 16) for t in lhs.split()]
        pairs.append((a, x, int(by_div), int(by_rcp)))
    assert len(pairs) >= 8
    for a_bits, x_bits, by_div, by_rcp in pairs:
        amax = Fraction(float(np.array([a_bits], np.uint16).view(np.float16)[0]))
        xv = Fraction(float(np.array([x_bits], np.uint16).view(np.float16)[0]))
        alpha = _fl32(amax / 127)
        t = _fl32(xv / alpha)
        lo = t.__floor__()
        frac = t - lo
        code = lo + 1 if (frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2 == 1)) else lo
        t_rcp = _fl32(xv * _fl32(1 / alpha))
        lo2 = t_rcp.__floor__()
        f2 = t_rcp - lo2
        code_rcp = lo2 + 1 if (f2 > Fraction(1, 2) or (f2 == Fraction(1, 2) and lo2 % 2 == 1)) else lo2
        assert code != code_rcp and (code, code_rcp) == (by_div, by_rcp)     # the pair does discriminate the two forms
        row = np.array([[a_bits, x_bits, x_bits ^ 0x8000, 0]], np.uint16).view(np.float16)
        q, s = orc.daq(row, 1)
        assert Fraction(float(s[0])) == alpha
        assert q[0].tolist() == [127, code, -code, 0]


def test_daq_granularities_agree_when_rows_share_absmax(orc):
    x = workload.activations(24, 64, "share", n_outlier=0)
    x = np.clip(x, -2.0, 2.0).astype(np.float16)
    x[:, 5] = f16(2.5)  # every row has the same absmax
    ref_q, ref_s = orc.daq(x, 1)
    for R in (4, 12, 24):
        q, s = orc.daq(x, R)
        assert np.array_equal(q, ref_q)
        assert np.all(s == ref_s[0])


def test_daq_block_boundaries(orc):
    # the scale of block b depends on rows [bR, bR+R) only
    x = workload.activations(12, 32, "blocks")
    q, s = orc.daq(x, 4)
    for b in range(3):
        qb, sb = orc.daq(x[4 * b:4 * b + 4], 4)
        assert np.array_equal(q[4 * b:4 * b + 4], qb) and s[b] == sb[0]
    with pytest.raises(ValueError):
        orc.daq(x, 5)


def test_daq_noise_model(orc):
    # Algorithm 1's noise term: a uniform quantizer of step Delta has error variance Delta^2 / 12
    x = workload.activations(64, 4096, "noise", n_outlier=0)
    q, s = orc.daq(x, 1)
    err = x.astype(np.float64) - s.astype(np.float64)[:, None] * q.astype(np.float64)
    ratio = (err ** 2).mean(axis=1) / (s.astype(np.float64) ** 2 / 12.0)
    assert abs(ratio.mean() - 1.0) < 0.03


# ---------------------------------------------------------------- the integer GEMM

def _brute_gemm(q, w):
    M, K = q.shape
    N = w.shape[0]
    out = [[0] * N for _ in range(M)]
    for m in range(M):
        for n in range(N):
            out[m][n] = sum(int(q[m, k]) * int(w[n, k]) for k in range(K))
    return np.array(out, dtype=np.int64)


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (16, 9, 13), (5, 16, 33)])
def test_gemm_brute_force(orc, M, N, K):
    g = workload.rng("brute", M, N, K)
    q = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    w = g.integers(-127, 128, size=(N, K), dtype=np.int8)
    assert np.array_equal(orc.gemm_i8(q, w).astype(np.int64), _brute_gemm(q, w))


def test_gemm_against_numpy_matmul(orc):
    g = workload.rng("npmm")
    q = g.integers(-127, 128, size=(70, 300), dtype=np.int8)
    w = g.integers(-127, 128, size=(45, 300), dtype=np.int8)
    want = q.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(orc.gemm_i8(q, w).astype(np.int64), want)
    assert np.array_equal(orc.gemm_i8(q, w, nthreads=4).astype(np.int64), want)


def test_gemm_closed_forms(orc):
    g = workload.rng("closed")
    K = 48
    q = g.integers(-127, 128, size=(9, K), dtype=np.int8)
    eye = np.eye(K, dtype=np.int8)
    assert np.array_equal(orc.gemm_i8(q, eye), q.astype(np.int32))            # W = I -> acc = Q
    ones = np.ones((3, K), np.int8)
    assert np.array_equal(orc.gemm_i8(q, ones), np.repeat(q.astype(np.int32).sum(1, keepdims=True), 3, 1))
    # W[n, k] = [k == n+1]: a shifted identity tells operand order and transposition apart
    sh = np.zeros((K - 1, K), np.int8)
    sh[np.arange(K - 1), np.arange(1, K)] = 1
    assert np.array_equal(orc.gemm_i8(q, sh), q[:, 1:].astype(np.int32))
    # permuting k in both operands changes nothing
    w = g.integers(-127, 128, size=(7, K), dtype=np.int8)
    p = g.permutation(K)
    assert np.array_equal(orc.gemm_i8(q, w), orc.gemm_i8(q[:, p], w[:, p]))
    # extreme fill at the largest DiT reduction length: 4608 * 127^2, no int32 overflow
    big = np.full((2, 4608), 127, np.int8)
    assert orc.gemm_i8(big, -big).tolist() == [[-74322432] * 2] * 2


# ---------------------------------------------------------------- 4-bit storage and GEMM

def test_w4_pack_format_and_roundtrip(orc):
    # the documented storage order: in each run of 8 k, byte j holds k=j (low) and k=4+j (high)
    w = np.array([[0, 1, 2, 3, 4, 5, 6, 7, -8, -7, -6, -5, -4, -3, -2, -1]], np.int8)
    assert orc.pack_w4(w).tolist() == [[0x40, 0x51, 0x62, 0x73, 0xC8, 0xD9, 0xEA, 0xFB]]
    # every byte value decodes and re-encodes to itself
    allb = np.arange(256, dtype=np.uint32).astype(np.uint8).reshape(1, 256)
    codes = orc.unpack_w4(allb, 512)
    assert codes.min() == -8 and codes.max() == 7
    assert np.array_equal(orc.pack_w4(codes), allb)
    with pytest.raises(ValueError):
        orc.pack_w4(np.full((1, 8), 8, np.int8))


def test_w4_gemm_one_hot_and_group_sum(orc):
    g = workload.rng("w4")
    K, N, M = 256, 6, 5
    q = g.integers(-127, 128, size=(M, K), dtype=np.int8)
    # one-hot weights: channel n picks k = pick[n]; the partial of the other group is 0
    pick = [0, 3, 4, 127, 128, 255]
    w = np.zeros((N, K), np.int8)
    for n, k in enumerate(pick):
        w[n, k] = 1
    P = orc.gemm_w4g128(q, orc.pack_w4(w))
    assert P.shape == (M, 2, N)
    for n, k in enumerate(pick):
        assert np.array_equal(P[:, k // 128, n], q[:, k].astype(np.int32))
        assert not P[:, 1 - k // 128, n].any()
    # random codes: partials are the per-group slices of the int8 GEMM on the unpacked codes
    w = workload.w4_codes(N, K, "t")
    P = orc.gemm_w4g128(q, orc.pack_w4(w))
    for gi in range(2):
        sl = slice(128 * gi, 128 * gi + 128)
        assert np.array_equal(P[:, gi, :].astype(np.int64), q[:, sl].astype(np.int64) @ w[:, sl].astype(np.int64).T)
    assert np.array_equal(P.sum(axis=1), orc.gemm_i8(q, w))
    assert np.array_equal(orc.gemm_w4g128(q, orc.pack_w4(w), nthreads=3), P)


# ---------------------------------------------------------------- dequantization epilogues

def test_epilogue_power_of_two_scales_is_exact_scaling(orc):
    # s_a * s_w = 2^j and no bias: y = binary16(acc * 2^j), one rounding
    acc = np.array([[1, -3, 2049, 2050, 2051, 4097, 65504, 65519, 65520, -74322432, 0, 4099]], np.int32)
    s_a = np.array([0.5], np.float32)
    s_w = np.full((acc.shape[1],), 2.0, np.float32)
    y = orc.epilogue_w8(acc, s_a, 1, s_w, None)
    # 2049 lies half-way between 2048 and 2050 -> even mantissa 2048; 2051 -> 2052; 4097 -> 4096;
    # 4099 -> 4100; 65519 -> 65504; 65520 and beyond -> inf
    want = [1, -3, 2048, 2050, 2052, 4096, 65504, 65504, np.inf, -np.inf, 0, 4100]
    assert y.astype(np.float64).tolist() == [[float(v) for v in want]]
    y = orc.epilogue_w8(acc, np.array([2.0 ** -20], np.float32), 1, np.ones(acc.shape[1], np.float32), None)
    assert np.array_equal(y, (acc.astype(np.float64) * 2.0 ** -20).astype(np.float16))


def test_epilogue_w8_scales_rows_columns_bias(orc):
    g = workload.rng("epi8")
    M, N, R = 12, 10, 4
    acc = g.integers(-10 ** 6, 10 ** 6, size=(M, N), dtype=np.int32)
    s_a = g.uniform(1e-3, 1e-1, M // R).astype(np.float32)
    s_w = workload.w8_scales(N, "epi")
    b = workload.bias(N, "epi")
    y = orc.epilogue_w8(acc, s_a, R, s_w, b)
    exact = acc.astype(np.float64) * np.repeat(s_a, R).astype(np.float64)[:, None] * s_w.astype(np.float64)[None, :] \
        + b.astype(np.float64)[None, :]
    # two binary32 roundings then one binary16 rounding: within 2^-11 (1 + small) relative
    assert np.all(np.abs(y.astype(np.float64) - exact) <= np.abs(exact) * (2.0 ** -11 + 2.0 ** -21) + 1e-12)
    # zero accumulators give exactly the bias; no bias gives exactly zero
    z = np.zeros((M, N), np.int32)
    assert np.array_equal(orc.epilogue_w8(z, s_a, R, s_w, b), np.repeat(b[None, :], M, 0))
    assert not orc.epilogue_w8(z, s_a, R, s_w, None).view(np.uint16).any()
    # without a bias the expression is two binary32 products: numpy's binary32 arithmetic agrees bit for bit
    u = acc.astype(np.float32) * np.repeat(s_a, R)[:, None]
    u = u * s_w[None, :]
    assert np.array_equal(orc.epilogue_w8(acc, s_a, R, s_w, None), u.astype(np.float16))
    # with a bias the last step is one fused multiply-add: t*s_w is exact in binary64, so the binary64
    # sum differs from the exact one by at most 2^-53 relative; allow the rare double-rounding flip
    t = (acc.astype(np.float32) * np.repeat(s_a, R)[:, None]).astype(np.float64)
    v = (t * s_w.astype(np.float64)[None, :] + b.astype(np.float64)[None, :]).astype(np.float32)
    assert (y != v.astype(np.float16)).sum() <= 1


def test_epilogue_w4_equal_power_of_two_groups_reduce_to_w8(orc):
    g = workload.rng("epi4")
    M, N, G, R = 8, 6, 3, 2
    P = g.integers(-130048, 130049, size=(M, G, N), dtype=np.int32)
    s_a = g.uniform(1e-3, 1e-1, M // R).astype(np.float32)
    b = workload.bias(N, "epi4")
    sw = np.full((N, G), 2.0 ** -5, np.float16)
    y4 = orc.epilogue_w4(P, s_a, R, sw, b)
    y8 = orc.epilogue_w8(P.sum(axis=1, dtype=np.int32), s_a, R, np.full((N,), 2.0 ** -5, np.float32), b)
    assert np.array_equal(y4, y8)
    # general group scales: compare with exact real arithmetic to accumulated-rounding accuracy
    sw = workload.w4_scales(N, 128 * G, "epi4")
    y = orc.epilogue_w4(P, s_a, R, sw, b).astype(np.float64)
    terms = P.astype(np.float64) * sw.astype(np.float64).T[None, :, :]
    exact = terms.sum(axis=1) * np.repeat(s_a, R).astype(np.float64)[:, None] + b.astype(np.float64)[None, :]
    mag = np.abs(terms).sum(axis=1) * np.repeat(s_a, R).astype(np.float64)[:, None] + np.abs(b.astype(np.float64))
    assert np.all(np.abs(y - exact) <= np.abs(exact) * 2.0 ** -11 + mag * 2.0 ** -21)
    # group order and indexing: a single non-zero group with scale 2^j
    for gi in range(G):
        Pz = np.zeros_like(P)
        Pz[:, gi, :] = P[:, gi, :]
        swz = workload.w4_scales(N, 128 * G, "z")
        swz[:, gi] = np.float16(0.25)
        want = orc.epilogue_w8(P[:, gi, :].copy(), s_a, R, np.full((N,), 0.25, np.float32), None)
        assert np.array_equal(orc.epilogue_w4(Pz, s_a, R, swz, None), want)


# ---------------------------------------------------------------- the whole layer

def test_layer_composition_and_zero_input(orc):
    M, K, N, R = 8, 128, 12, 4
    x = workload.activations(M, K, "layer")
    lw = workload.layer_weights("t", K, N, 8, "layer")
    out = orc.qlinear_w8a8(x, R, lw["w"], lw["s_w"], lw["bias"], nthreads=2)
    q, s = orc.daq(x, R)
    acc = orc.gemm_i8(q, lw["w"])
    assert np.array_equal(out["q"], q) and np.array_equal(out["s_a"], s) and np.array_equal(out["acc"], acc)
    assert np.array_equal(out["y"], orc.epilogue_w8(acc, s, R, lw["s_w"], lw["bias"]))
    # zero input: codes 0, scale 1, output is the bias
    z = orc.qlinear_w8a8(np.zeros((M, K), np.float16), R, lw["w"], lw["s_w"], lw["bias"])
    assert not z["q"].any() and np.all(z["s_a"] == 1.0) and np.array_equal(z["y"], np.repeat(lw["bias"][None], M, 0))
    l4 = workload.layer_weights("t", K, N, 4, "layer")
    w4 = orc.pack_w4(l4["w"])
    o4 = orc.qlinear_w4a8(x, R, w4, l4["s_w"], l4["bias"])
    assert np.array_equal(o4["q"], q) and np.array_equal(o4["P"], orc.gemm_w4g128(q, w4))
    assert np.array_equal(o4["y"], orc.epilogue_w4(o4["P"], s, R, l4["s_w"], l4["bias"]))
    z4 = orc.qlinear_w4a8(np.zeros((M, K), np.float16), R, w4, l4["s_w"], l4["bias"])
    assert np.array_equal(z4["y"], np.repeat(l4["bias"][None], M, 0))


@pytest.mark.parametrize("bits", [8, 4])
def test_layer_close_to_unquantized_linear(orc, bits):
    """Sanity, not parity: the layer approximates x @ (s_w * W)^T + b with the error a
    127-level activation quantizer predicts (relative Frobenius error ~ amax / (rms * 127 * sqrt(12)))."""
    M, K, N = 64, 1152, 96
    x = workload.activations(M, K, "sanity", n_outlier=0)
    lw = workload.layer_weights("s", K, N, bits, "sanity")
    if bits == 8:
        y = orc.qlinear_w8a8(x, 1, lw["w"], lw["s_w"], lw["bias"], want_debug=False)["y"]
        wr = lw["w"].astype(np.float64) * lw["s_w"].astype(np.float64)[:, None]
    else:
        y = orc.qlinear_w4a8(x, 1, orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"], want_debug=False)["y"]
        wr = lw["w"].astype(np.float64) * np.repeat(lw["s_w"].astype(np.float64), 128, axis=1)
    ref = x.astype(np.float64) @ wr.T + lw["bias"].astype(np.float64)[None]
    rel = np.linalg.norm(y.astype(np.float64) - ref) / np.linalg.norm(ref)
    assert 0.002 < rel < 0.02


def test_workload_outputs_stay_finite(orc):
    # the synthetic recipe must not overflow binary16 at the largest drift (sigma = 5)
    for name, K, N in workload.BLOCK_LAYERS:
        x = workload.activations(16, K, name, "fin", sigma=5.0)
        for bits in (8, 4):
            lw = workload.layer_weights(name, K, N, bits, 0)
            if bits == 8:
                y = orc.qlinear_w8a8(x, 1, lw["w"], lw["s_w"], lw["bias"], nthreads=8, want_debug=False)["y"]
            else:
                y = orc.qlinear_w4a8(x, 1, orc.pack_w4(lw["w"]), lw["s_w"], lw["bias"], nthreads=8,
                                     want_debug=False)["y"]
            assert np.isfinite(y.astype(np.float32)).all()
            assert np.abs(y.astype(np.float32)).max() < 30000
