"""CPU oracle for the offline side of the method: timestep selection (Step 4, eqs. (5)-(6)), the budgeted
greedy planner (Algorithm 2, Phase A) and the GPTQ weight packer (Step 2).

TEST INFRASTRUCTURE ONLY, like the rest of this package: plain Python / numpy in float64, no blocking, no shared code
with the product library, never imported by it.  Every function follows the steps of its passage in the paper's order
and notation; where the paper is silent the reading is stated in the docstring.
"""
import heapq
from fractions import Fraction

import numpy as np


def protected_tail(candidates, T, rho):
    """Step 4: T_tail = {t in C : t / T >= 1 - rho}.  rho is taken as an exact rational (a float rho is converted
    through its shortest decimal string), so that t / T >= 1 - rho is decided without rounding."""
    r = Fraction(str(rho)) if not isinstance(rho, Fraction) else rho
    return [t for t in candidates if Fraction(t, T) >= 1 - r]


def schedule_topk(delta, candidates, T, rho, k):
    """Eq. (6): S = T_tail  union  TopK(C \\ T_tail, delta, k - |T_tail|), |S| = k.
    delta: mapping / array indexed by timestep.  TopK takes the m largest delta; equal delta: the earlier timestep
    first (reading: the paper does not say).  k below |T_tail| or above |C| is an error.  Returns the kept steps sorted."""
    cand = sorted(set(int(t) for t in candidates))
    tail = protected_tail(cand, T, rho)
    m = k - len(tail)
    if m < 0 or k > len(cand):
        raise ValueError("k must lie between the tail size and the number of candidates")
    rest = [t for t in cand if t not in set(tail)]
    rest.sort(key=lambda t: (-float(delta[t]), t))
    return sorted(tail + rest[:m])


def plan_greedy(drift, c_step, bit_options, c_lat, c_mem, s_m, B_lat, B_mem, rho, eps=1e-12):
    """Algorithm 2, Phase A, step by step.

    drift[t], c_step[t]            per step, t = 0 .. T-1 (the last floor(rho*T) indices are the protected tail)
    bit_options[l]                 the layer's widths, any order; the plan starts at the largest
    c_lat[l][b], c_mem[l][b]       cost of layer l at width b (dicts keyed by width)
    s_m[l]                         sensitivity
    Readings (the paper's listing leaves them open):
      * C_lat = sum of c_step over kept steps + sum of c_lat(l, Pi(l)); C_mem = sum of c_mem(l, Pi(l)).
      * a layer's next move goes to its next smaller width; its score is S_bit = (c_lat(l,b) - c_lat(l,b')) / (eps + s_M(l)).
      * the bit candidate is the top of the heap; the listing's side condition on C_mem cannot hold while the memory
        budget is still far away, so it is read as: while ONLY the memory budget is violated, steps are not pruned
        (removing a step frees no memory).
      * S_step > S_bit removes the step, otherwise the bit move is taken; with one kind of candidate left, that kind is
        taken; with none left the loop stops and the plan is reported infeasible.
      * ties in the sort by drift: earlier step first; ties in the heap: smaller layer index first.
    Returns dict(plan = {l: width}, kept = sorted steps, C_lat, C_mem, feasible, trace = list of moves)."""
    T = len(drift)
    n_tail = int(np.floor(Fraction(str(rho)) * T))
    tail = set(range(T - n_tail, T))
    L = len(bit_options)
    opts = [sorted(set(o), reverse=True) for o in bit_options]
    pos = [0] * L
    plan = {l: opts[l][0] for l in range(L)}
    kept = set(range(T))
    C_lat = float(sum(c_step[t] for t in range(T))) + float(sum(c_lat[l][plan[l]] for l in range(L)))
    C_mem = float(sum(c_mem[l][plan[l]] for l in range(L)))
    R = sorted((t for t in range(T) if t not in tail), key=lambda t: (float(drift[t]), t))
    heap = []

    def push(l):
        if pos[l] + 1 < len(opts[l]):
            b, b2 = opts[l][pos[l]], opts[l][pos[l] + 1]
            d_lat = float(c_lat[l][b]) - float(c_lat[l][b2])
            heapq.heappush(heap, (-(d_lat / (eps + float(s_m[l]))), l, b, b2))

    for l in range(L):
        push(l)
    trace = []
    feasible = True
    while C_lat > B_lat or C_mem > B_mem:
        step_ok = bool(R) and C_lat > B_lat
        bit_ok = bool(heap)
        if not step_ok and not bit_ok:
            feasible = False
            break
        S_step = c_step[R[0]] / (eps + float(drift[R[0]])) if step_ok else None
        S_bit = -heap[0][0] if bit_ok else None
        if step_ok and (not bit_ok or S_step > S_bit):
            t = R.pop(0)
            kept.discard(t)
            C_lat -= float(c_step[t])
            trace.append(("step", t))
        else:
            _, l, b, b2 = heapq.heappop(heap)
            plan[l] = b2
            pos[l] += 1
            C_lat -= float(c_lat[l][b]) - float(c_lat[l][b2])
            C_mem -= float(c_mem[l][b]) - float(c_mem[l][b2])
            trace.append(("bit", l, b, b2))
            push(l)
    return dict(plan=plan, kept=sorted(kept), C_lat=C_lat, C_mem=C_mem, feasible=feasible, trace=trace)


def quant_grid(w_block, bits, symmetric):
    """Scale and zero point of one weight group (a 1-D float64 array), Step 2: symmetric: scale = max|w| / q_max with
    q_max = 2^(b-1) - 1 (b = 8: 127) or 2^(b-1) - 1 on the positive and -2^(b-1) on the negative side for b < 8
    (4 bits: codes in [-8, 7]), zero point 0; asymmetric: codes in [0, 2^b - 1], scale = (max - min) / (2^b - 1),
    zero = round(-min / scale) (min and max widened to include 0).  An all-zero group gets scale 1."""
    if symmetric:
        qmax = 2 ** (bits - 1) - 1
        qmin = -qmax if bits == 8 else -(2 ** (bits - 1))
        amax = float(np.max(np.abs(w_block))) if w_block.size else 0.0
        scale = amax / qmax if amax > 0 else 1.0
        return scale, 0, qmin, qmax
    lo, hi = min(float(np.min(w_block)), 0.0), max(float(np.max(w_block)), 0.0)
    levels = 2 ** bits - 1
    scale = (hi - lo) / levels if hi > lo else 1.0
    zero = int(np.rint(-lo / scale))
    return scale, zero, 0, levels


def _round_scale(s, scale_fp16):
    """The kernels read 4-bit group scales as binary16: with scale_fp16 the scale is rounded to it before it is used."""
    if not scale_fp16:
        return float(np.float32(s))
    h = float(np.float16(s))
    return h if h > 0 else float(np.float16(6e-8))


def gptq_quantize(W, H, bits, group, symmetric=True, damp=0.01, scale_fp16=False):
    """GPTQ (Step 2; Frantar et al.): quantize W [N, K] column by column so that the output error under the layer's
    input second-moment matrix H ~ X^T X [K, K] stays small.
      1. dead inputs (H_kk = 0): H_kk = 1, W[:, k] = 0;  H += damp * mean(diag H) * I
      2. U = the upper Cholesky factor of H^-1  (H^-1 = U^T U)
      3. for k = 0 .. K-1: at the start of a group its scale (and zero point) is taken from the CURRENT (already
         compensated) weights of the group's columns, per row; q = clamp(rne(w_k / scale) + zero); the rounding error
         e = (w_k - dequant(q)) / U_kk is pushed onto the columns not yet quantized: W[:, j] -= e * U_kj for j > k.
    Returns (codes int [N, K], scale float64 [N, K/group], zero int [N, K/group], W_hat float64 [N, K])."""
    W = np.array(W, dtype=np.float64)
    H = np.array(H, dtype=np.float64)
    N, K = W.shape
    assert H.shape == (K, K) and K % group == 0
    dead = np.diag(H) == 0
    H[dead, dead] = 1.0
    W[:, dead] = 0.0
    H[np.arange(K), np.arange(K)] += damp * float(np.mean(np.diag(H)))
    Hinv = np.linalg.inv(H)
    U = np.linalg.cholesky(Hinv).T            # upper: Hinv = U^T U
    codes = np.zeros((N, K), np.int64)
    scales = np.zeros((N, K // group), np.float64)
    zeros = np.zeros((N, K // group), np.int64)
    What = np.zeros((N, K), np.float64)
    _, _, qmin, qmax = quant_grid(np.zeros(1), bits, symmetric)
    for k in range(K):
        g = k // group
        if k % group == 0:
            for n in range(N):
                s, z, _, _ = quant_grid(W[n, k:k + group], bits, symmetric)
                s = _round_scale(s, scale_fp16)
                if not symmetric:
                    z = int(np.rint(-min(float(np.min(W[n, k:k + group])), 0.0) / s))
                scales[n, g], zeros[n, g] = s, z
        for n in range(N):
            s, z = scales[n, g], zeros[n, g]
            q = int(min(max(np.rint(W[n, k] / s) + z, qmin), qmax))
            codes[n, k] = q
            What[n, k] = (q - z) * s
        err = (W[:, k] - What[:, k]) / U[k, k]
        if k + 1 < K:
            W[:, k + 1:] -= np.outer(err, U[k, k + 1:])
    return codes, scales, zeros, What


def rtn_quantize(W, bits, group, symmetric=True, scale_fp16=False):
    """Round to nearest with the same grids, no error compensation (what GPTQ reduces to for a diagonal H)."""
    W = np.array(W, dtype=np.float64)
    N, K = W.shape
    codes = np.zeros((N, K), np.int64)
    What = np.zeros((N, K))
    for n in range(N):
        for g in range(K // group):
            blk = W[n, g * group:(g + 1) * group]
            s, z, qmin, qmax = quant_grid(blk, bits, symmetric)
            s = _round_scale(s, scale_fp16)
            if not symmetric:
                z = int(np.rint(-min(float(np.min(blk)), 0.0) / s))
            q = np.clip(np.rint(blk / s) + z, qmin, qmax).astype(np.int64)
            codes[n, g * group:(g + 1) * group] = q
            What[n, g * group:(g + 1) * group] = (q - z) * s
    return codes, What


def output_error(W, What, H):
    """tr((W - What) H (W - What)^T): the squared output error of the layer on the calibration inputs."""
    D = np.asarray(W, np.float64) - np.asarray(What, np.float64)
    return float(np.einsum("nk,kj,nj->", D, np.asarray(H, np.float64), D))
