"""CPU oracle for the quantized DiT linear layer (DiffPro, arXiv 2511.11446).

TEST INFRASTRUCTURE ONLY.  The arithmetic lives in ``diffpro_oracle.c`` (plain
scalar C); this module compiles it with gcc and exposes it on numpy arrays.
Nothing here imports, links or calls the HIP library, and the HIP library never
calls this.  Allowed callers: the test-suite, the smoke check, and the
benchmark's ``cpu_baseline`` leg.

Operations and the passages they follow:
  daq               Step 3, eq. (4) with tau = block absmax (percentile -> 100)
  gemm_i8           INT8 x INT8 -> INT32 GEMM (Step 3, Step 5, Section 6)
  gemm_w4g128       the same GEMM on 4-bit group-128 weights (Step 2)
  epilogue_w8/_w4   dequantization with per-channel / per-group weight scales
  daq_robust        eq. (4) as printed: nearest-rank percentile clipping, activation width from Step 6
  gemm_w4g          4-bit GEMM with weight groups of any size dividing K (Step 2, Algorithm 1)
  dequant_w8/_w4    the fp32 values before the fp16 rounding;  block_glue: activation, gate, residual on top of them
  linear_f16        a layer the plan leaves in FP16 (fp64 sum)
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "diffpro_oracle.c")
_LIB = os.path.join(_HERE, "libdiffpro_oracle.so")
CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC", "-std=c11"]


def _host_has_fma():
    try:
        with open("/proc/cpuinfo") as f:
            return " fma " in f.read()
    except OSError:
        return False

_lib = None


def build(force=False):
    """Compile the oracle with gcc (a second or two)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        # -mfma only turns the explicit fmaf() calls into one instruction (contraction stays off);
        # without it libm's fmaf gives the same correctly rounded result, slower
        extra = ["-mfma"] if _host_has_fma() else []
        subprocess.check_call(["gcc", *CFLAGS, *extra, _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_half_to_float.restype = ctypes.c_float
        L.orc_half_to_float.argtypes = [ctypes.c_uint16]
        L.orc_float_to_half.restype = ctypes.c_uint16
        L.orc_float_to_half.argtypes = [ctypes.c_float]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError("expected %s, got %s" % (np.dtype(dtype), a.dtype))
    return a


def _f16bits(a):
    """Accept float16 or uint16 arrays; hand the raw 16-bit patterns to C."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a.view(np.uint16)
    return _c(a, np.uint16)


def max_threads():
    return int(lib().orc_max_threads())


def half_to_float(bits):
    bits = _c(bits, np.uint16)
    out = np.empty(bits.shape, np.float32)
    lib().orc_half_to_float_array(_p(bits), _p(out), ctypes.c_int64(bits.size))
    return out


def float_to_half(f):
    f = _c(f, np.float32)
    out = np.empty(f.shape, np.uint16)
    lib().orc_float_to_half_array(_p(f), _p(out), ctypes.c_int64(f.size))
    return out


def daq(x, R, nthreads=1):
    """x [M,K] float16 -> (codes int8 [M,K], alpha float32 [M/R])."""
    xb = _f16bits(x)
    M, K = xb.shape
    q = np.empty((M, K), np.int8)
    s = np.empty((M // R if R > 0 else 0,), np.float32)
    rc = lib().orc_daq(_p(xb), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(R), _p(q), _p(s),
                       ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_daq rc=%d" % rc)
    return q, s


def daq_robust(x, R, p_ppm=999000, a_bits=8, nthreads=1):
    """Eq. (4) as printed: x [M,K] float16 -> (codes int8 [M,K], alpha float32 [M/R]) with
    tau = nearest-rank percentile (p_ppm parts per million) of |x| over each block of R rows, a_bits-bit codes."""
    xb = _f16bits(x)
    M, K = xb.shape
    q = np.empty((M, K), np.int8)
    s = np.empty((M // R if R > 0 else 0,), np.float32)
    rc = lib().orc_daq_robust(_p(xb), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(R), ctypes.c_int64(p_ppm),
                              ctypes.c_int(a_bits), _p(q), _p(s), ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_daq_robust rc=%d" % rc)
    return q, s


def gemm_i8(q, w, nthreads=1):
    """q [M,K] int8, w [N,K] int8 -> acc int32 [M,N]."""
    q = _c(q, np.int8)
    w = _c(w, np.int8)
    M, K = q.shape
    N, K2 = w.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    rc = lib().orc_gemm_i8(_p(q), _p(w), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _p(acc),
                           ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_gemm_i8 rc=%d" % rc)
    return acc


def pack_w4(w):
    """w [N,K] int8 codes in [-8,7] -> packed uint8 [N,K/2]."""
    w = _c(w, np.int8)
    N, K = w.shape
    out = np.empty((N, K // 2), np.uint8)
    rc = lib().orc_pack_w4(_p(w), ctypes.c_int64(N), ctypes.c_int64(K), _p(out))
    if rc:
        raise ValueError("orc_pack_w4 rc=%d" % rc)
    return out


def unpack_w4(packed, K):
    packed = _c(packed, np.uint8)
    N = packed.shape[0]
    assert packed.shape[1] * 2 == K
    out = np.empty((N, K), np.int8)
    rc = lib().orc_unpack_w4(_p(packed), ctypes.c_int64(N), ctypes.c_int64(K), _p(out))
    if rc:
        raise ValueError("orc_unpack_w4 rc=%d" % rc)
    return out


def gemm_w4g128(q, w4, nthreads=1):
    """q [M,K] int8, w4 packed [N,K/2] -> partials int32 [M,K/128,N]."""
    q = _c(q, np.int8)
    w4 = _c(w4, np.uint8)
    M, K = q.shape
    N = w4.shape[0]
    assert w4.shape[1] * 2 == K
    P = np.empty((M, K // 128, N), np.int32)
    rc = lib().orc_gemm_w4g128(_p(q), _p(w4), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _p(P),
                               ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_gemm_w4g128 rc=%d" % rc)
    return P


def gemm_w4g(q, w4, group, nthreads=1):
    """q [M,K] int8, w4 packed [N,K/2] -> P int32 [M,K/group,N] (weight groups of `group` consecutive k)."""
    q = _c(q, np.int8)
    w4 = _c(w4, np.uint8)
    M, K = q.shape
    N = w4.shape[0]
    assert w4.shape[1] * 2 == K and K % group == 0
    P = np.empty((M, K // group, N), np.int32)
    rc = lib().orc_gemm_w4g(_p(q), _p(w4), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), ctypes.c_int64(group),
                            _p(P), ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_gemm_w4g rc=%d" % rc)
    return P


def epilogue_w8(acc, s_a, R, s_w, bias):
    """-> y float16 [M,N]."""
    acc = _c(acc, np.int32)
    s_a = _c(s_a, np.float32)
    s_w = _c(s_w, np.float32)
    M, N = acc.shape
    assert s_a.size == M // R and s_w.size == N
    b = None if bias is None else _f16bits(bias)
    y = np.empty((M, N), np.uint16)
    rc = lib().orc_epilogue_w8(_p(acc), _p(s_a), ctypes.c_int64(R), _p(s_w), _p(b), ctypes.c_int64(M),
                               ctypes.c_int64(N), _p(y))
    if rc:
        raise ValueError("orc_epilogue_w8 rc=%d" % rc)
    return y.view(np.float16)


def epilogue_w4(P, s_a, R, s_w, bias):
    """P [M,G,N] int32, s_w float16 [N,G] -> y float16 [M,N]."""
    P = _c(P, np.int32)
    s_a = _c(s_a, np.float32)
    sw = _f16bits(s_w)
    M, G, N = P.shape
    assert sw.shape == (N, G) and s_a.size == M // R
    b = None if bias is None else _f16bits(bias)
    y = np.empty((M, N), np.uint16)
    rc = lib().orc_epilogue_w4(_p(P), _p(s_a), ctypes.c_int64(R), _p(sw), _p(b), ctypes.c_int64(M),
                               ctypes.c_int64(N), ctypes.c_int64(G), _p(y))
    if rc:
        raise ValueError("orc_epilogue_w4 rc=%d" % rc)
    return y.view(np.float16)


def linear_f16(x, w, bias=None, nthreads=1):
    """A layer left in FP16: x [M,K], w [N,K], bias [N] float16 -> y float16 [M,N] (fp64 sum, then fp32, then fp16)."""
    xb, wb = _f16bits(x), _f16bits(w)
    M, K = xb.shape
    N = wb.shape[0]
    assert wb.shape[1] == K
    b = None if bias is None else _f16bits(bias)
    y = np.empty((M, N), np.uint16)
    rc = lib().orc_linear_f16(_p(xb), _p(wb), _p(b), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), _p(y),
                              ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_linear_f16 rc=%d" % rc)
    return y.view(np.float16)


def dequant_w8(acc, s_a, R, s_w, bias):
    """The layer's fp32 values before the fp16 rounding, float32 [M,N]."""
    acc = _c(acc, np.int32)
    s_a = _c(s_a, np.float32)
    s_w = _c(s_w, np.float32)
    M, N = acc.shape
    b = None if bias is None else _f16bits(bias)
    u = np.empty((M, N), np.float32)
    rc = lib().orc_dequant_w8(_p(acc), _p(s_a), ctypes.c_int64(R), _p(s_w), _p(b), ctypes.c_int64(M), ctypes.c_int64(N), _p(u))
    if rc:
        raise ValueError("orc_dequant_w8 rc=%d" % rc)
    return u


def dequant_w4(P, s_a, R, s_w, bias):
    P = _c(P, np.int32)
    s_a = _c(s_a, np.float32)
    sw = _f16bits(s_w)
    M, G, N = P.shape
    b = None if bias is None else _f16bits(bias)
    u = np.empty((M, N), np.float32)
    rc = lib().orc_dequant_w4(_p(P), _p(s_a), ctypes.c_int64(R), _p(sw), _p(b), ctypes.c_int64(M), ctypes.c_int64(N),
                              ctypes.c_int64(G), _p(u))
    if rc:
        raise ValueError("orc_dequant_w4 rc=%d" % rc)
    return u


def block_glue(u, act=0, residual=None, gate=None, gate_rows=1):
    """u float32 [M,N] -> y float16 [M,N]: activation, gate and residual folded into the epilogue."""
    u = _c(u, np.float32)
    M, N = u.shape
    r = None if residual is None else _f16bits(residual)
    g = None if gate is None else _f16bits(gate)
    y = np.empty((M, N), np.uint16)
    rc = lib().orc_block_glue(_p(u), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int(act), _p(r), _p(g),
                              ctypes.c_int64(gate_rows), _p(y))
    if rc:
        raise ValueError("orc_block_glue rc=%d" % rc)
    return y.view(np.float16)


def qlinear_w8a8(x, R, w, s_w, bias, nthreads=1, want_debug=True):
    """Whole layer.  Returns dict(y, q, s_a, acc)."""
    xb = _f16bits(x)
    w = _c(w, np.int8)
    s_w = _c(s_w, np.float32)
    M, K = xb.shape
    N = w.shape[0]
    assert w.shape[1] == K and s_w.size == N
    b = None if bias is None else _f16bits(bias)
    y = np.empty((M, N), np.uint16)
    q = np.empty((M, K), np.int8) if want_debug else None
    s_a = np.empty((M // R,), np.float32) if want_debug else None
    acc = np.empty((M, N), np.int32) if want_debug else None
    rc = lib().orc_qlinear_w8a8(_p(xb), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(R), _p(w), _p(s_w),
                                _p(b), ctypes.c_int64(N), _p(y), _p(q), _p(s_a), _p(acc), ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_qlinear_w8a8 rc=%d" % rc)
    return dict(y=y.view(np.float16), q=q, s_a=s_a, acc=acc)


def qlinear_w4a8(x, R, w4, s_w, bias, nthreads=1, want_debug=True):
    """Whole layer on 4-bit group-128 weights.  Returns dict(y, q, s_a, P)."""
    xb = _f16bits(x)
    w4 = _c(w4, np.uint8)
    sw = _f16bits(s_w)
    M, K = xb.shape
    N = w4.shape[0]
    G = K // 128
    assert w4.shape[1] * 2 == K and sw.shape == (N, G)
    b = None if bias is None else _f16bits(bias)
    y = np.empty((M, N), np.uint16)
    q = np.empty((M, K), np.int8) if want_debug else None
    s_a = np.empty((M // R,), np.float32) if want_debug else None
    P = np.empty((M, G, N), np.int32) if want_debug else None
    rc = lib().orc_qlinear_w4a8(_p(xb), ctypes.c_int64(M), ctypes.c_int64(K), ctypes.c_int64(R), _p(w4), _p(sw),
                                _p(b), ctypes.c_int64(N), _p(y), _p(q), _p(s_a), _p(P), ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_qlinear_w4a8 rc=%d" % rc)
    return dict(y=y.view(np.float16), q=q, s_a=s_a, P=P)


def layernorm_modulate(x, shift=None, scale=None, rows_per_mod=1, eps=1e-6):
    """LayerNorm without affine parameters followed by the adaptive modulation of a DiT block, in float64, rounded once
    to binary32 and then to binary16 (Step 3: LayerNorm stays in higher precision in front of the quantized layers):
        mu = mean(x), var = mean((x - mu)^2), n = (x - mu) / sqrt(var + eps), h = n * (1 + scale[m / rows_per_mod]) + shift[...]
    x [M,K] float16; shift, scale [M/rows_per_mod, K] float16 or None.  Returns h float16 [M,K]."""
    xd = np.asarray(x, dtype=np.float16).astype(np.float64)
    M, K = xd.shape
    mu = xd.sum(axis=1, keepdims=True) / K
    var = ((xd - mu) ** 2).sum(axis=1, keepdims=True) / K
    n = (xd - mu) / np.sqrt(var + eps)
    g = 1.0 if scale is None else 1.0 + np.repeat(np.asarray(scale, np.float16).astype(np.float64), rows_per_mod, axis=0)
    b = 0.0 if shift is None else np.repeat(np.asarray(shift, np.float16).astype(np.float64), rows_per_mod, axis=0)
    return (n * g + b).astype(np.float32).astype(np.float16)


def row_absmax_bits(y):
    """The statistic a layer may leave for the DAQ of the layer that consumes its output (Step 3, eq. (4): tau is the
    largest magnitude of the scale block): per row of the fp16 matrix y, max_n |y[m,n]| as a binary16 bit pattern
    (uint32 [M]).  Written as the definition: magnitudes as numbers, the largest one, then its bit pattern."""
    y = np.asarray(y, dtype=np.float16)
    mag = np.abs(y.astype(np.float64)).max(axis=1)
    return mag.astype(np.float16).view(np.uint16).astype(np.uint32)


def gemm_i8g(q, w, group, nthreads=1):
    """int8 codes q [M,K] x int8 weight codes w [N,K] (any width up to 8 bits held as int8) -> int32 [M, K/group, N]."""
    q = _c(q, np.int8)
    w = _c(w, np.int8)
    M, K = q.shape
    N = w.shape[0]
    assert w.shape[1] == K and K % group == 0
    P = np.empty((M, K // group, N), np.int32)
    rc = lib().orc_gemm_i8g(_p(q), _p(w), ctypes.c_int64(M), ctypes.c_int64(N), ctypes.c_int64(K), ctypes.c_int64(group), _p(P),
                            ctypes.c_int(nthreads))
    if rc:
        raise ValueError("orc_gemm_i8g rc=%d" % rc)
    return P


def epilogue_cg(P, alpha, R, s_w, bias):
    """Dequantization with activation scales per (scale block, channel group): alpha float32 [M/R, G], s_w float16 [N, G]."""
    P = _c(P, np.int32)
    M, G, N = P.shape
    alpha = _c(alpha, np.float32)
    sw = _f16bits(s_w)
    assert alpha.shape == (M // R, G) and sw.shape == (N, G)
    b = None if bias is None else _f16bits(bias)
    y = np.empty((M, N), np.uint16)
    rc = lib().orc_epilogue_cg(_p(P), _p(alpha), ctypes.c_int64(R), _p(sw), _p(b), ctypes.c_int64(M), ctypes.c_int64(N),
                               ctypes.c_int64(G), _p(y))
    if rc:
        raise ValueError("orc_epilogue_cg rc=%d" % rc)
    return y.view(np.float16)


def daq_cg(x, R, group, nthreads=1):
    """Eq. (4) of Step 3 with its channel groups: one scale per block of R rows (a sample's tokens) AND group of `group`
    consecutive channels, tau = that sub-block's absolute maximum.  Written as the definition: every (row block, channel
    group) sub-matrix goes through daq() as one scale block.  Returns (codes int8 [M,K], alpha float32 [M/R, K/group])."""
    x = np.ascontiguousarray(x)
    M, K = x.shape
    assert M % R == 0 and K % group == 0
    q = np.empty((M, K), np.int8)
    alpha = np.empty((M // R, K // group), np.float32)
    for b in range(M // R):
        for g in range(K // group):
            sub = np.ascontiguousarray(x[b * R:(b + 1) * R, g * group:(g + 1) * group])
            qs, s = daq(sub, R, nthreads=nthreads)
            q[b * R:(b + 1) * R, g * group:(g + 1) * group] = qs
            alpha[b, g] = s[0]
    return q, alpha


def pack_bits(codes, bits):
    """Dense storage of b-bit two's-complement codes (b = 3 or 6: Algorithm 1's W3, Section 2.4's W6): the codes of a row
    are concatenated LSB first into a little-endian bit stream.  codes int8 [N,K] with K*bits % 8 == 0 -> uint8 [N, K*bits/8]."""
    codes = np.asarray(codes, np.int8)
    N, K = codes.shape
    assert (K * bits) % 8 == 0
    lo, hi = -(1 << (bits - 1)), (1 << (bits - 1)) - 1
    assert codes.min() >= lo and codes.max() <= hi
    u = (codes.astype(np.int64) & ((1 << bits) - 1))
    bitsarr = ((u[:, :, None] >> np.arange(bits)) & 1).reshape(N, K * bits).astype(np.uint8)
    return np.packbits(bitsarr, axis=1, bitorder="little")


def unpack_bits(packed, bits, K):
    packed = np.asarray(packed, np.uint8)
    N = packed.shape[0]
    b = np.unpackbits(packed, axis=1, bitorder="little")[:, :K * bits].reshape(N, K, bits).astype(np.int64)
    u = (b << np.arange(bits)).sum(axis=2)
    return np.where(u >= (1 << (bits - 1)), u - (1 << bits), u).astype(np.int8)
