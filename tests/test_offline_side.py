"""Offline side (Step 2 GPTQ packer, Step 4 timestep selection, Algorithm 2 Phase A planner), CPU only:
first the oracle (oracle/planning.py) against things other than itself, then the library's host code against the oracle."""
import itertools
import os

import numpy as np
import pytest

import workload
from oracle import planning as P

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def ql():
    import paper_2511_11446_amd as q
    q.lib()
    return q


# ------------------------------------------------------------------ Step 4, eqs. (5)-(6)

def test_schedule_topk_is_the_best_subset_containing_the_tail():
    """Eq. (6) by its meaning: among all subsets of size k that contain the protected tail, the schedule has the largest
    total delta (brute force over all subsets of a 10-step timeline)."""
    g = workload.rng("topk-brute")
    T, rho = 10, 0.3
    for trial in range(6):
        delta = g.uniform(0, 1, T)
        tail = [t for t in range(T) if t / T >= 1 - rho - 1e-12]
        assert tail == [7, 8, 9]
        for k in (3, 5, 8, 10):
            got = P.schedule_topk(delta, range(T), T, rho, k)
            best = max((s for s in itertools.combinations(range(T), k) if set(tail) <= set(s)), key=lambda s: delta[list(s)].sum())
            assert got == sorted(best)


def test_schedule_topk_worked_example_ties_and_errors():
    # T = 10, rho = 0.2: tail = {8, 9}.  delta decreasing in t: the three largest of the rest are 0, 1, 2.
    delta = np.arange(10, 0, -1.0)
    assert P.schedule_topk(delta, range(10), 10, 0.2, 5) == [0, 1, 2, 8, 9]
    # candidates may be a subset; a tie goes to the earlier step
    delta = np.array([1.0, 5.0, 5.0, 5.0, 0.0, 0.0, 0.0, 0.0, 9.0, 9.0])
    assert P.schedule_topk(delta, [0, 1, 2, 3, 9], 10, 0.2, 3) == [1, 2, 9]
    assert P.protected_tail(range(1000), 1000, 0.2) == list(range(800, 1000))      # the paper's rho on its 1000-step grid
    with pytest.raises(ValueError):
        P.schedule_topk(delta, range(10), 10, 0.2, 1)       # fewer than the tail
    with pytest.raises(ValueError):
        P.schedule_topk(delta, range(10), 10, 0.2, 11)


def test_library_schedule_matches_oracle(ql):
    g = workload.rng("topk-lib")
    for T, rho_ppm, k in [(10, 200000, 5), (1000, 200000, 500), (50, 0, 7), (37, 333333, 20), (25, 1000000, 25)]:
        delta = np.round(g.uniform(0, 1, T), 2)             # rounded: plenty of ties
        cand = np.sort(g.choice(T, size=max(k, T - 3), replace=False)) if T > 30 else np.arange(T)
        from fractions import Fraction
        want = P.schedule_topk(delta, cand, T, Fraction(rho_ppm, 1000000), k)
        got = ql.schedule_topk(delta, cand, T, rho_ppm, k)
        assert got.tolist() == want
    with pytest.raises(ql.QlError):
        ql.schedule_topk(np.zeros(10), np.arange(10), 10, 200000, 1)
    with pytest.raises(ql.QlError):
        ql.schedule_topk(np.zeros(10), np.array([0, 10]), 10, 200000, 1)


# ------------------------------------------------------------------ Algorithm 2, Phase A

def _read_hand_worked():
    rows = {}
    for line in open(os.path.join(GOLD, "plan_greedy_hand_worked.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        rows[tok[0]] = tok[1:]
    drift = [float(v) for v in rows["drift"]]
    c_step = [float(v) for v in rows["c_step"]]
    layers = []
    for name in ("layer0", "layer1"):
        t = rows[name]
        layers.append(dict(bits=[int(t[1]), int(t[2])], c_lat=[float(t[4]), float(t[5])], c_mem=[float(t[7]), float(t[8])],
                           sensitivity=float(t[10])))
    B_lat, B_mem, rho_ppm = float(rows["budget"][0]), float(rows["budget"][1]), int(rows["budget"][3])
    e = rows["expect"]
    expect = dict(bits=[int(e[1]), int(e[2])], kept=[int(e[4]), int(e[5])], C_lat=float(e[7]), C_mem=float(e[9]))
    return drift, c_step, layers, B_lat, B_mem, rho_ppm, expect


def _oracle_plan(drift, c_step, layers, B_lat, B_mem, rho_ppm, eps):
    from fractions import Fraction
    return P.plan_greedy(drift, c_step, [l["bits"] for l in layers],
                         [dict(zip(l["bits"], l["c_lat"])) for l in layers], [dict(zip(l["bits"], l["c_mem"])) for l in layers],
                         [l["sensitivity"] for l in layers], B_lat, B_mem, Fraction(rho_ppm, 1000000), eps)


def test_plan_greedy_hand_worked(ql):
    drift, c_step, layers, B_lat, B_mem, rho_ppm, expect = _read_hand_worked()
    r = _oracle_plan(drift, c_step, layers, B_lat, B_mem, rho_ppm, 0.0)
    assert [r["plan"][0], r["plan"][1]] == expect["bits"] and r["kept"] == expect["kept"]
    assert r["C_lat"] == expect["C_lat"] and r["C_mem"] == expect["C_mem"] and r["feasible"]
    assert r["trace"] == [("step", 1), ("bit", 1, 8, 4), ("step", 3), ("step", 2)]
    got = ql.plan_greedy(drift, c_step, layers, B_lat, B_mem, rho_ppm, eps=0.0)
    assert got["bits"].tolist() == expect["bits"] and np.flatnonzero(got["kept"]).tolist() == expect["kept"]
    assert got["C_lat"] == expect["C_lat"] and got["C_mem"] == expect["C_mem"] and got["feasible"]


def test_plan_greedy_special_cases():
    # budgets already met: nothing moves
    r = P.plan_greedy([1, 2, 3], [1, 1, 1], [[8, 4]], [{8: 5, 4: 2}], [{8: 4, 4: 2}], [1.0], 100, 100, 0.0)
    assert r["plan"] == {0: 8} and r["kept"] == [0, 1, 2] and r["trace"] == []
    # steps only (a single width per layer), equal step cost c: exactly ceil((C - B) / c) steps go, lowest drift first,
    # the protected tail stays
    drift = [5, 1, 7, 3, 2, 9, 4, 8, 6, 0.5]
    r = P.plan_greedy(drift, [2.0] * 10, [[8]], [{8: 0.0}], [{8: 0.0}], [1.0], 11.0, 1.0, 0.2)
    removed = sorted(set(range(10)) - set(r["kept"]))
    assert len(removed) == 5 and removed == sorted(sorted(range(8), key=lambda t: drift[t])[:5]) and {8, 9} <= set(r["kept"])
    # only the memory budget is violated: no step is pruned, layers narrow in order of their score
    r = P.plan_greedy([1, 1], [1, 1], [[8, 4], [8, 4]], [{8: 4, 4: 1}, {8: 9, 4: 1}], [{8: 4, 4: 2}, {8: 4, 4: 2}], [1.0, 1.0],
                      1e9, 6.0, 0.0)
    assert r["kept"] == [0, 1] and r["plan"] == {0: 8, 1: 4} and r["C_mem"] == 6.0
    # nothing left to take: reported infeasible, everything prunable pruned, everything narrowed
    r = P.plan_greedy([1, 2, 3, 4], [1] * 4, [[8, 4]], [{8: 4, 4: 2}], [{8: 4, 4: 2}], [1.0], 0.5, 0.5, 0.25)
    assert not r["feasible"] and r["kept"] == [3] and r["plan"] == {0: 4}


def test_plan_greedy_invariants_and_library_matches_oracle_on_random_instances(ql):
    g = workload.rng("greedy-random")
    for trial in range(40):
        T = int(g.integers(3, 40))
        L = int(g.integers(1, 12))
        rho_ppm = int(g.choice([0, 100000, 200000, 500000]))
        drift = np.round(g.uniform(0.01, 5, T), 1)
        c_step = np.round(g.uniform(0.5, 3, T), 1)
        layers = []
        for l in range(L):
            bits = list(g.permutation([16, 8, 4, 3])[:int(g.integers(1, 5))])
            order = sorted(bits, reverse=True)
            lat = np.sort(np.round(g.uniform(0.1, 9, len(bits)), 2))[::-1]
            mem = np.sort(np.round(g.uniform(0.1, 9, len(bits)), 2))[::-1]
            layers.append(dict(bits=[int(b) for b in bits], c_lat=[float(lat[order.index(b)]) for b in bits],
                               c_mem=[float(mem[order.index(b)]) for b in bits], sensitivity=float(np.round(g.uniform(0.1, 2), 2))))
        full_lat = c_step.sum() + sum(max(l["c_lat"]) for l in layers)
        full_mem = sum(max(l["c_mem"]) for l in layers)
        B_lat, B_mem = float(full_lat * g.uniform(0.2, 1.1)), float(full_mem * g.uniform(0.2, 1.1))
        want = _oracle_plan(drift, c_step, layers, B_lat, B_mem, rho_ppm, 1e-9)
        # invariants: the tail is kept, the totals are what the plan says, a feasible plan meets both budgets
        n_tail = rho_ppm * T // 1000000
        assert set(range(T - n_tail, T)) <= set(want["kept"])
        lat = sum(c_step[t] for t in want["kept"]) + sum(dict(zip(l["bits"], l["c_lat"]))[want["plan"][i]] for i, l in enumerate(layers))
        assert abs(lat - want["C_lat"]) < 1e-9
        if want["feasible"]:
            assert want["C_lat"] <= B_lat and want["C_mem"] <= B_mem
        got = ql.plan_greedy(drift, c_step, layers, B_lat, B_mem, rho_ppm, eps=1e-9)
        assert got["bits"].tolist() == [want["plan"][i] for i in range(L)]
        assert np.flatnonzero(got["kept"]).tolist() == want["kept"]
        assert got["feasible"] == want["feasible"] and abs(got["C_lat"] - want["C_lat"]) < 1e-9


# ------------------------------------------------------------------ Step 2: GPTQ

def _calib(K, n=400, key="gptq"):
    g = workload.rng(key, K)
    X = g.standard_normal((n, K)) * g.uniform(0.2, 3.0, K)
    for k in range(1, K, 3):
        X[:, k] += 0.8 * X[:, k - 1]          # correlated inputs: where the error compensation pays
    return X


def test_gptq_with_uncorrelated_inputs_is_round_to_nearest():
    """A diagonal H couples no two columns: U is diagonal, nothing is pushed forward, and GPTQ is plain rounding."""
    g = workload.rng("gptq-diag")
    W = g.standard_normal((6, 32))
    H = np.diag(g.uniform(0.5, 4.0, 32))
    for bits, sym in ((4, True), (8, True), (3, False), (4, False)):
        c, s, z, Wh = P.gptq_quantize(W, H, bits, 16, symmetric=sym, damp=0.0)
        cr, Whr = P.rtn_quantize(W, bits, 16, symmetric=sym)
        assert np.array_equal(c, cr) and np.allclose(Wh, Whr, rtol=0, atol=1e-12)
        assert np.allclose(Wh, (c - np.repeat(z, 16, 1)) * np.repeat(s, 16, 1))


def test_gptq_two_columns_closed_form():
    """K = 2, one group per column: the first column is rounded; its error d reaches the second column as
    w2 + d * H01 / H11 (the minimiser of the quadratic output error over w2 with column 1 fixed), which is then rounded."""
    H = np.array([[2.0, 0.9], [0.9, 1.5]])
    W = np.array([[0.37, -0.52], [-0.81, 0.44], [0.05, 0.93]])
    c, s, z, Wh = P.gptq_quantize(W, H, 4, 1, symmetric=True, damp=0.0)
    for n in range(3):
        s1 = float(np.float32(abs(W[n, 0]) / 7))
        q1 = np.clip(np.rint(W[n, 0] / s1), -8, 7)
        d = W[n, 0] - q1 * s1
        w2 = W[n, 1] + d * H[0, 1] / H[1, 1]
        s2 = float(np.float32(abs(w2) / 7))
        assert c[n, 0] == q1 and c[n, 1] == np.clip(np.rint(w2 / s2), -8, 7)
        assert abs(s[n, 1] - s2) < 1e-12


def test_gptq_compensation_is_the_least_squares_update():
    """After one column has been quantized, the compensated remaining weights minimise the output error over all choices
    of the remaining weights (checked against numpy's least-squares solution of that problem)."""
    K = 6
    X = _calib(K, 300, "gptq-ls")
    H = X.T @ X
    g = workload.rng("gptq-ls-w")
    w = g.standard_normal(K)
    # one row, group = K, 8 bits; read the compensated weights back from a 2-step run: quantizing column 0 only is not
    # exposed, so solve the same problem directly: fix w_hat0 = dequantized first code, minimise |X (w - v)|^2 over v[1:]
    c, s, z, Wh = P.gptq_quantize(w[None], H, 8, K, damp=0.0)
    v0 = Wh[0, 0]
    rhs = X @ w - X[:, 0] * v0
    v_rest = np.linalg.lstsq(X[:, 1:], rhs, rcond=None)[0]
    # GPTQ's second code is the rounding of the compensated second weight = the first entry of that minimiser
    assert c[0, 1] == np.clip(np.rint(v_rest[0] / s[0, 0]), -127, 127)


def test_gptq_beats_round_to_nearest_on_correlated_inputs_and_codes_stay_in_range():
    for K, bits, group, sym in ((64, 4, 32, True), (96, 3, 32, False), (128, 4, 128, True), (64, 8, 64, True)):
        X = _calib(K)
        H = X.T @ X
        W = workload.rng("gptq-w", K).standard_normal((16, K)) * 0.05
        c, s, z, Wh = P.gptq_quantize(W, H, bits, group, symmetric=sym, scale_fp16=True)
        cr, Whr = P.rtn_quantize(W, bits, group, symmetric=sym, scale_fp16=True)
        e_gptq, e_rtn = P.output_error(W, Wh, H), P.output_error(W, Whr, H)
        assert e_gptq < e_rtn, (K, bits, e_gptq, e_rtn)
        lo, hi = (-(2 ** (bits - 1)) if bits < 8 else -127, 2 ** (bits - 1) - 1) if sym else (0, 2 ** bits - 1)
        assert c.min() >= lo and c.max() <= hi
        assert np.array_equal(s.astype(np.float16).astype(np.float64), s)        # scales are binary16 values


def test_library_gptq_matches_oracle(ql):
    """The library's packer against the oracle: same algorithm in float64 on both sides; the two differ only in the
    summation order inside the factorisations, which can tip a code that sits within rounding of a half-way point, so
    the codes are compared on all but a handful of elements and the output error to 1e-6."""
    for K, N, bits, group, sym in ((64, 24, 4, 32, True), (128, 16, 4, 128, True), (96, 8, 3, 32, False), (256, 12, 8, 256, True),
                                   (64, 8, 6, 16, False)):
        X = _calib(K, key="gptq-lib")
        H = X.T @ X
        H[:, 5] = 0
        H[5, :] = 0                     # an input that never fires
        W = (workload.rng("gptq-lib-w", K).standard_normal((N, K)) * 0.05).astype(np.float32)
        c, s, z, Wh = P.gptq_quantize(W, H, bits, group, symmetric=sym, scale_fp16=(bits == 4))
        codes, scales, zeros = ql.gptq_quantize_host(W, H, bits, group, symmetric=sym, scale_fp16=(bits == 4))
        shift = 0 if sym else 2 ** (bits - 1)
        diff = int((codes.astype(np.int64) + shift != c).sum())
        assert diff <= max(2, c.size // 2000), (K, bits, diff)
        assert np.allclose(scales, s, rtol=1e-6, atol=0)
        if not sym:
            assert int((zeros + shift != z).sum()) <= 1
        Wh_lib = (codes.astype(np.float64) - np.repeat(zeros, group, 1)) * np.repeat(scales.astype(np.float64), group, 1)
        e_lib, e_orc = P.output_error(W, Wh_lib, H), P.output_error(W, Wh, H)
        assert abs(e_lib - e_orc) <= 1e-3 * e_orc
        assert (codes[:, 5] == (0 if sym else np.repeat(zeros, group, 1)[:, 5])).all()     # dropped input: weight 0
    with pytest.raises(ql.QlError):
        ql.gptq_quantize_host(np.zeros((2, 8), np.float32), np.eye(8), 9, 8)
    with pytest.raises(ql.QlError):
        ql.gptq_quantize_host(np.zeros((2, 8), np.float32), -np.eye(8), 4, 8)


def test_gptq_codes_feed_the_4bit_packer(ql):
    K, N = 128, 8
    X = _calib(K, key="gptq-pack")
    W = (workload.rng("gptq-pack-w").standard_normal((N, K)) * 0.05).astype(np.float32)
    codes, scales, _ = ql.gptq_quantize_host(W, X.T @ X, 4, 128, symmetric=True, scale_fp16=True)
    packed = ql.ql_pack_w4_host(codes)
    import oracle
    assert np.array_equal(oracle.unpack_w4(packed, K), codes)
    assert np.array_equal(scales.astype(np.float16).astype(np.float32), scales)
