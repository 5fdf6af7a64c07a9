"""Python binding of the MI355X quantized DiT linear layer (DiffPro, arXiv 2511.11446).

Argument marshalling only: every step (DAQ, INT8 GEMM, dequantization, plan walk)
runs inside ``libdiffpro_qlinear.so`` (hand-written HIP for gfx950) through the C
ABI of ``include/diffpro_qlinear.h``.  PyTorch supplies device memory and the
current stream, nothing else.  There is no CPU or PyTorch fallback: if the
library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdiffpro_qlinear.so")

QL_OK = 0
STATUS_NAMES = {0: "QL_OK", 1: "QL_ERR_NULL", 2: "QL_ERR_SHAPE", 3: "QL_ERR_ALIGN", 4: "QL_ERR_UNSUPPORTED",
                5: "QL_ERR_WORKSPACE", 6: "QL_ERR_DEVICE"}

# every symbol include/diffpro_qlinear.h declares
EXPORTS = ("ql_status_string", "ql_last_device_error", "ql_version", "daq_workspace_bytes", "daq_quantize",
           "qlinear_workspace_bytes", "qlinear_w8a8", "qlinear_w4a8", "qgemm_w8a8", "qgemm_w4a8",
           "ql_pack_w4_host", "ql_plan_create", "ql_plan_destroy", "ql_plan_num_layers",
           "ql_plan_workspace_bytes", "qlinear_plan_run", "ql_set_gemm_variant", "ql_num_gemm_variants",
           "ql_gemm_variant_name", "daq_quantize_robust", "qlinear_plan_run_robust", "ql_time_bin",
           "qlinear_w4a8_g", "qgemm_w4a8_g", "qlinear_w8a8_fused", "qlinear_w4a8_fused", "qlinear_f16", "ql_repack_w4_pairs_host", "ql_prepack_w4", "daq_quantize_rowmax", "qlinear_plan_run_ex", "qlinear_w8a8_noalloc", "qlinear_noalloc_max_bytes",
           "ql_schedule_topk", "ql_plan_greedy", "ql_gptq_quantize_host", "daq_quantize_ln",
           "daq_cg_workspace_bytes", "daq_quantize_cg", "qlinear_grouped_workspace_bytes", "qlinear_grouped", "ql_pack_bits_host",
           "ql_unpack_bits_host", "ql_zero_point_fold_host")


class QlError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        extra = ""
        if status == 6:
            extra = " (hipError %d)" % lib().ql_last_device_error()
        super().__init__("%s failed: %s%s" % (where, STATUS_NAMES.get(status, status), extra))


class ql_debug(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("a_scales", ctypes.c_void_p), ("acc", ctypes.c_void_p)]


class ql_layer_desc(ctypes.Structure):
    _fields_ = [("K", ctypes.c_int64), ("N", ctypes.c_int64), ("w_bits", ctypes.c_int32), ("group", ctypes.c_int32),
                ("w", ctypes.c_void_p), ("w_scale", ctypes.c_void_p), ("bias", ctypes.c_void_p)]


_lib = None
_i64, _vp, _sz, _int = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int


def ensure_built():
    """For the entry scripts (tests, smoke check, benchmark): compile the library if no built one is there.
    The binding itself never builds and never falls back: lib() raises when the library is missing."""
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    return LIB_PATH


def lib():
    """Load the HIP library (built in-tree by ``python -m paper_2511_11446_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2511_11446_amd.build` "
                          "(there is no fallback path)" % LIB_PATH)
    # PyTorch-ROCm ships its own HIP runtime (soname libamdhip64.so.7).  Loading torch first makes the
    # dynamic loader resolve this library's libamdhip64.so.7 dependency to that same copy, so torch's
    # device pointers and streams and this library's kernels live in ONE runtime.  The other order
    # would put two HIP runtimes in the process, and the second one finds no device.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    L.ql_status_string.restype = ctypes.c_char_p
    L.ql_status_string.argtypes = [_int]
    L.ql_gemm_variant_name.restype = ctypes.c_char_p
    L.ql_gemm_variant_name.argtypes = [_int]
    L.daq_workspace_bytes.restype = _sz
    L.daq_workspace_bytes.argtypes = [_i64, _i64, _i64]
    L.qlinear_workspace_bytes.restype = _sz
    L.qlinear_workspace_bytes.argtypes = [_i64, _i64, _i64]
    L.daq_quantize.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]
    lin = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _vp, ctypes.POINTER(ql_debug), _vp, _sz, _vp]
    L.qlinear_w8a8.argtypes = lin
    L.qlinear_w4a8.argtypes = lin
    gem = [_vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _vp, _vp, _vp]
    L.qgemm_w8a8.argtypes = gem
    L.qgemm_w4a8.argtypes = gem
    L.ql_pack_w4_host.argtypes = [_vp, _i64, _i64, _vp]
    L.ql_plan_create.argtypes = [ctypes.POINTER(ql_layer_desc), ctypes.c_int32, _i64, ctypes.POINTER(_vp)]
    L.ql_plan_destroy.argtypes = [_vp]
    L.ql_plan_destroy.restype = None
    L.ql_plan_num_layers.argtypes = [_vp]
    L.ql_plan_num_layers.restype = ctypes.c_int32
    L.ql_plan_workspace_bytes.argtypes = [_vp, _i64, _i64]
    L.ql_plan_workspace_bytes.restype = _sz
    L.qlinear_plan_run.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i64, _i64, _vp, _sz, _vp]
    L.qlinear_w4a8_g.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp, ctypes.POINTER(ql_debug), _vp, _sz, _vp]
    L.qlinear_w4a8_g.restype = _int
    L.qgemm_w4a8_g.argtypes = [_vp, _vp, _i64, _i64, _i64, _vp, _vp, _i64, _vp, _i64, _vp, _vp, _vp]
    L.qgemm_w4a8_g.restype = _int
    L.qlinear_w8a8_fused.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, ctypes.POINTER(ql_fusion), _vp, _vp, _sz, _vp]
    L.qlinear_w8a8_fused.restype = _int
    L.qlinear_w4a8_fused.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _i64, _vp, _i64, ctypes.POINTER(ql_fusion), _vp, _vp, _sz, _vp]
    L.qlinear_w4a8_fused.restype = _int
    L.ql_repack_w4_pairs_host.argtypes = [_vp, _i64, _i64, _vp]
    L.ql_repack_w4_pairs_host.restype = _int
    L.ql_prepack_w4.argtypes = [_vp, _i64, _i64, _vp, _vp]
    L.ql_prepack_w4.restype = _int
    L.daq_quantize_rowmax.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    L.daq_quantize_rowmax.restype = _int
    L.qlinear_plan_run_ex.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i64, _i64, _vp, ctypes.POINTER(ctypes.POINTER(ql_fusion)), _vp, _sz, _vp]
    L.qlinear_plan_run_ex.restype = _int
    L.qlinear_f16.argtypes = [_vp, _i64, _i64, _vp, _vp, _i64, ctypes.POINTER(ql_fusion), _vp, _vp]
    L.qlinear_f16.restype = _int
    L.qlinear_plan_run_robust.argtypes = [_vp, ctypes.POINTER(_vp), ctypes.POINTER(_vp), _i64, _i64, _vp, _vp, _sz, _vp]
    L.qlinear_plan_run_robust.restype = _int
    L.daq_quantize_robust.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    L.daq_quantize_robust.restype = _int
    L.ql_time_bin.argtypes = [_i64, _i64]
    L.ql_time_bin.restype = _int
    L.ql_set_gemm_variant.argtypes = [_int]
    L.qlinear_noalloc_max_bytes.restype = _sz
    L.qlinear_noalloc_max_bytes.argtypes = []
    L.qlinear_w8a8_noalloc.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _vp, _i64, _vp, _vp]
    L.qlinear_w8a8_noalloc.restype = _int
    _lib = L
    return L


def _check(status, where):
    if status != QL_OK:
        raise QlError(status, where)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _need(t, dtype, shape=None, name="tensor"):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous() or t.dtype != dtype:
        raise TypeError("%s must be a contiguous CUDA tensor of %s" % (name, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s has shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    return t


def workspace(nbytes, device="cuda"):
    """A 256-byte aligned scratch tensor of at least nbytes."""
    import torch
    return torch.empty((max(int(nbytes), 256),), dtype=torch.uint8, device=device)


def daq_workspace_bytes(M, K, R):
    return int(lib().daq_workspace_bytes(M, K, R))


def qlinear_workspace_bytes(M, K, R):
    return int(lib().qlinear_workspace_bytes(M, K, R))


def daq_quantize(x, R, q=None, scales=None, ws=None, stream=None):
    """x fp16 [M,K] -> (q int8 [M,K], scales fp32 [M/R])."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    if q is None:
        q = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if scales is None:
        scales = torch.empty((max(M // max(R, 1), 1),), dtype=torch.float32, device=x.device)
    if ws is None and R > 1:
        ws = workspace(daq_workspace_bytes(M, K, R), x.device)
    rc = lib().daq_quantize(_ptr(x), M, K, R, _ptr(q), _ptr(scales), _ptr(ws), 0 if ws is None else ws.numel(),
                            _stream(stream))
    _check(rc, "daq_quantize")
    return q, scales


def daq_quantize_rowmax(x, R, row_absmax, q=None, scales=None, ws=None, stream=None):
    """DAQ with the row maxima given (int32 [M], binary16 bit patterns, as a fused layer's row_absmax output leaves them)."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    _need(row_absmax, torch.int32, (M,), "row_absmax")
    if q is None:
        q = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if scales is None:
        scales = torch.empty((max(M // max(R, 1), 1),), dtype=torch.float32, device=x.device)
    if ws is None and R > 1:
        ws = workspace(daq_workspace_bytes(M, K, R), x.device)
    rc = lib().daq_quantize_rowmax(_ptr(x), M, K, R, _ptr(row_absmax), _ptr(q), _ptr(scales), _ptr(ws),
                                   0 if ws is None else ws.numel(), _stream(stream))
    _check(rc, "daq_quantize_rowmax")
    return q, scales


def daq_quantize_ln(x, R=1, shift=None, scale=None, rows_per_mod=1, eps=1e-6, want_h=False, want_q=True, ws=None, stream=None):
    """LayerNorm + modulation + DAQ: x fp16 [M,K] -> dict(q int8, scales fp32 [M/R], h fp16 (if want_h or R > 1))."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    out = {}
    if want_h or R > 1:
        out["h"] = torch.empty((M, K), dtype=torch.float16, device=x.device)
    if want_q:
        out["q"] = torch.empty((M, K), dtype=torch.int8, device=x.device)
        out["scales"] = torch.empty((max(M // max(R, 1), 1),), dtype=torch.float32, device=x.device)
    if ws is None and R > 1 and want_q:
        ws = workspace(daq_workspace_bytes(M, K, R), x.device)
    fn = lib().daq_quantize_ln
    fn.argtypes = [_vp, _i64, _i64, _i64, _vp, _vp, _i64, ctypes.c_float, _vp, _vp, _vp, _vp, _sz, _vp]
    rc = fn(_ptr(x), M, K, R, _ptr(shift), _ptr(scale), rows_per_mod, eps, _ptr(out.get("h")), _ptr(out.get("q")),
            _ptr(out.get("scales")), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(rc, "daq_quantize_ln")
    return out


def daq_quantize_cg(x, R, act_group, stream=None):
    """Eq. (4) with channel groups: x fp16 [M,K] -> (q int8 [M,K], alpha fp32 [M/R, K/act_group])."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    q = torch.empty((M, K), dtype=torch.int8, device=x.device)
    sc = torch.empty((M // R, K // act_group), dtype=torch.float32, device=x.device)
    L = lib()
    L.daq_cg_workspace_bytes.restype = _sz
    L.daq_cg_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64]
    ws = workspace(L.daq_cg_workspace_bytes(M, K, R, act_group), x.device)
    L.daq_quantize_cg.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _sz, _vp]
    _check(L.daq_quantize_cg(_ptr(x), M, K, R, act_group, _ptr(q), _ptr(sc), _ptr(ws), ws.numel(), _stream(stream)), "daq_quantize_cg")
    return q, sc


def qlinear_grouped(x, R, w, w_scale, group, bias=None, act_group=0, storage=8, debug=False, y=None, stream=None):
    """Group-scaled layer for any weight width: storage 8 = int8 codes [N,K], 4 = packed nibbles [N,K/2];
    act_group = 0 (row scales) or group (one activation scale per scale block and channel group)."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    N = w.shape[0]
    G = K // group
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    L = lib()
    L.qlinear_grouped_workspace_bytes.restype = _sz
    L.qlinear_grouped_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64]
    ws = workspace(L.qlinear_grouped_workspace_bytes(M, K, R, act_group), x.device)
    out, dbg = {"y": y}, None
    if debug:
        out["q"] = torch.empty((M, K), dtype=torch.int8, device=x.device)
        out["s_a"] = torch.empty((M // R,) if act_group == 0 else (M // R, G), dtype=torch.float32, device=x.device)
        out["P"] = torch.empty((M, G, N), dtype=torch.int32, device=x.device)
        dbg = ctypes.pointer(ql_debug(out["q"].data_ptr(), out["s_a"].data_ptr(), out["P"].data_ptr()))
    L.qlinear_grouped.argtypes = [_vp, _i64, _i64, _i64, _i64, _vp, ctypes.c_int32, _vp, _i64, _vp, _i64, _vp, ctypes.POINTER(ql_debug),
                                  _vp, _sz, _vp]
    rc = L.qlinear_grouped(_ptr(x), M, K, R, act_group, _ptr(w), storage, _ptr(w_scale), group, _ptr(bias), N, _ptr(y), dbg, _ptr(ws),
                           ws.numel(), _stream(stream))
    _check(rc, "qlinear_grouped")
    return out if debug else y


def pack_bits_host(codes, bits):
    import numpy as np
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    N, K = codes.shape
    out = np.empty((N, K * bits // 8), np.uint8)
    _check(lib().ql_pack_bits_host(codes.ctypes.data_as(_vp), _i64(N), _i64(K), ctypes.c_int32(bits), out.ctypes.data_as(_vp)), "ql_pack_bits_host")
    return out


def unpack_bits_host(packed, bits, K):
    import numpy as np
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    N = packed.shape[0]
    out = np.empty((N, K), np.int8)
    _check(lib().ql_unpack_bits_host(packed.ctypes.data_as(_vp), _i64(N), _i64(K), ctypes.c_int32(bits), out.ctypes.data_as(_vp)), "ql_unpack_bits_host")
    return out


def zero_point_fold_host(codes, zeros, group):
    import numpy as np
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    zeros = np.ascontiguousarray(zeros, dtype=np.int32)
    N, K = codes.shape
    out = np.empty((N, K), np.int8)
    _check(lib().ql_zero_point_fold_host(codes.ctypes.data_as(_vp), zeros.ctypes.data_as(_vp), _i64(N), _i64(K), _i64(group),
                                         out.ctypes.data_as(_vp)), "ql_zero_point_fold_host")
    return out


class ql_fusion(ctypes.Structure):
    _fields_ = [("act", ctypes.c_int32), ("reserved", ctypes.c_int32), ("residual", ctypes.c_void_p),
                ("gate", ctypes.c_void_p), ("gate_rows", ctypes.c_int64), ("row_absmax", ctypes.c_void_p)]


ACT_NONE, ACT_GELU_TANH = 0, 1


def qlinear_fused(x, R, w, w_scale, bias=None, bits=8, group=128, act=ACT_NONE, residual=None, gate=None, gate_rows=1,
                  y=None, ws=None, stream=None, row_absmax=None):
    """The layer with activation, gate and residual folded into its epilogue:
    h = fp16(act(u)); y = fp16(fma(gate, h, residual)).  bits = 8 (w int8 [N,K]) or 4 (w packed [N,K/2], group).
    row_absmax: int32 [M] device tensor that receives every row's largest |y| as a binary16 bit pattern, or None."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    N = w.shape[0]
    if residual is not None:
        _need(residual, torch.float16, (M, N), "residual")
    if gate is not None:
        _need(gate, torch.float16, (M // gate_rows, N), "gate")
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    if ws is None:
        ws = workspace(qlinear_workspace_bytes(M, K, R), x.device)
    if row_absmax is not None:
        _need(row_absmax, torch.int32, (M,), "row_absmax")
    fu = ql_fusion(act, 0, None if residual is None else residual.data_ptr(), None if gate is None else gate.data_ptr(), gate_rows,
                   None if row_absmax is None else row_absmax.data_ptr())
    if bits == 8:
        rc = lib().qlinear_w8a8_fused(_ptr(x), M, K, R, _ptr(w), _ptr(w_scale), _ptr(bias), N, ctypes.byref(fu), _ptr(y),
                                      _ptr(ws), ws.numel(), _stream(stream))
    else:
        rc = lib().qlinear_w4a8_fused(_ptr(x), M, K, R, _ptr(w), _ptr(w_scale), group, _ptr(bias), N, ctypes.byref(fu),
                                      _ptr(y), _ptr(ws), ws.numel(), _stream(stream))
    _check(rc, "qlinear_w%da8_fused" % bits)
    return y


def qlinear_f16(x, w, bias=None, act=ACT_NONE, residual=None, gate=None, gate_rows=1, y=None, stream=None, row_absmax=None):
    """A layer left in FP16: x fp16 [M,K], w fp16 [N,K] -> y fp16 [M,N] (fp32 accumulation)."""
    import torch
    _need(x, torch.float16, name="x")
    _need(w, torch.float16, name="w")
    M, K = x.shape
    N = w.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    fu = ql_fusion(act, 0, None if residual is None else residual.data_ptr(), None if gate is None else gate.data_ptr(), gate_rows,
                   None if row_absmax is None else row_absmax.data_ptr())
    _check(lib().qlinear_f16(_ptr(x), M, K, _ptr(w), _ptr(bias), N, ctypes.byref(fu), _ptr(y), _stream(stream)), "qlinear_f16")
    return y


class _DaqParams(ctypes.Structure):
    _fields_ = [("p_ppm", ctypes.c_int32), ("a_bits", ctypes.c_int32)]


def daq_quantize_robust(x, R, p_ppm=999000, a_bits=8, q=None, scales=None, ws=None, stream=None):
    """Percentile-clipped DAQ: x fp16 [M,K] -> (q int8 [M,K] with |q| <= 2^(a_bits-1)-1, scales fp32 [M/R])."""
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    if q is None:
        q = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if scales is None:
        scales = torch.empty((max(M // max(R, 1), 1),), dtype=torch.float32, device=x.device)
    if ws is None and R > 1:
        ws = workspace(daq_workspace_bytes(M, K, R), x.device)
    prm = _DaqParams(p_ppm, a_bits)
    rc = lib().daq_quantize_robust(_ptr(x), M, K, R, ctypes.byref(prm), _ptr(q), _ptr(scales), _ptr(ws),
                                   0 if ws is None else ws.numel(), _stream(stream))
    _check(rc, "daq_quantize_robust")
    return q, scales


def time_bin(step, num_steps):
    return int(lib().ql_time_bin(step, num_steps))


def _qlinear(fn_name, x, R, w, w_scale, bias, N, y, debug, ws, stream, group=128):
    import torch
    _need(x, torch.float16, name="x")
    M, K = x.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=x.device)
    if ws is None:
        ws = workspace(qlinear_workspace_bytes(M, K, R), x.device)
    dbg = None
    out = {"y": y}
    if debug:
        G = K // group
        out["q"] = torch.empty((M, K), dtype=torch.int8, device=x.device)
        out["s_a"] = torch.empty((M // R,), dtype=torch.float32, device=x.device)
        shape = (M, N) if fn_name == "qlinear_w8a8" else (M, G, N)
        out["acc" if fn_name == "qlinear_w8a8" else "P"] = acc = torch.empty(shape, dtype=torch.int32, device=x.device)
        dbg = ctypes.pointer(ql_debug(out["q"].data_ptr(), out["s_a"].data_ptr(), acc.data_ptr()))
    if fn_name == "qlinear_w4a8" and group != 128:
        fn_name = "qlinear_w4a8_g"
        rc = lib().qlinear_w4a8_g(_ptr(x), M, K, R, _ptr(w), _ptr(w_scale), group, _ptr(bias), N, _ptr(y), dbg, _ptr(ws),
                                  ws.numel(), _stream(stream))
    else:
        rc = getattr(lib(), fn_name)(_ptr(x), M, K, R, _ptr(w), _ptr(w_scale), _ptr(bias), N, _ptr(y), dbg, _ptr(ws),
                                     ws.numel(), _stream(stream))
    _check(rc, fn_name)
    return out if debug else y


def qlinear_w8a8(x, R, w, w_scale, bias=None, y=None, debug=False, ws=None, stream=None):
    """DAQ + INT8 GEMM + dequantization.  w int8 [N,K], w_scale fp32 [N], bias fp16 [N] or None."""
    import torch
    _need(w, torch.int8, name="w")
    _need(w_scale, torch.float32, (w.shape[0],), "w_scale")
    if bias is not None:
        _need(bias, torch.float16, (w.shape[0],), "bias")
    if w.shape[1] != x.shape[1]:
        raise ValueError("w must be [N,K]")
    return _qlinear("qlinear_w8a8", x, R, w, w_scale, bias, w.shape[0], y, debug, ws, stream)


def qlinear_w8a8_noalloc(x, R, w, w_scale, bias, y, stream=None):
    """qlinear_w8a8 on the library's own fixed scratch: the call allocates nothing; y is the caller's."""
    M, K = x.shape
    _check(lib().qlinear_w8a8_noalloc(_ptr(x), M, K, R, _ptr(w), _ptr(w_scale), _ptr(bias), w.shape[0], _ptr(y), _stream(stream)),
           "qlinear_w8a8_noalloc")
    return y


def qlinear_w4a8(x, R, w4, w_scale, bias=None, y=None, debug=False, ws=None, stream=None, group=128):
    """Same with packed 4-bit weights: w4 uint8 [N,K/2], w_scale fp16 [N,K/group]."""
    import torch
    _need(w4, torch.uint8, name="w4")
    K = x.shape[1]
    if w4.shape[1] * 2 != K:
        raise ValueError("w4 must be [N,K/2]")
    _need(w_scale, torch.float16, (w4.shape[0], K // group), "w_scale")
    if bias is not None:
        _need(bias, torch.float16, (w4.shape[0],), "bias")
    return _qlinear("qlinear_w4a8", x, R, w4, w_scale, bias, w4.shape[0], y, debug, ws, stream, group)


def _qgemm(fn_name, q, a_scales, R, w, w_scale, bias, N, y, acc, stream):
    import torch
    _need(q, torch.int8, name="q")
    _need(a_scales, torch.float32, name="a_scales")
    M, K = q.shape
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=q.device)
    rc = getattr(lib(), fn_name)(_ptr(q), _ptr(a_scales), M, K, R, _ptr(w), _ptr(w_scale), _ptr(bias), N, _ptr(y),
                                 _ptr(acc), _stream(stream))
    _check(rc, fn_name)
    return y


def qgemm_w8a8(q, a_scales, R, w, w_scale, bias=None, y=None, acc=None, stream=None):
    return _qgemm("qgemm_w8a8", q, a_scales, R, w, w_scale, bias, w.shape[0], y, acc, stream)


def qgemm_w4a8(q, a_scales, R, w4, w_scale, bias=None, y=None, acc=None, stream=None, group=128):
    if group == 128:
        return _qgemm("qgemm_w4a8", q, a_scales, R, w4, w_scale, bias, w4.shape[0], y, acc, stream)
    import torch
    M, K = q.shape
    N = w4.shape[0]
    if y is None:
        y = torch.empty((M, N), dtype=torch.float16, device=q.device)
    rc = lib().qgemm_w4a8_g(_ptr(q), _ptr(a_scales), M, K, R, _ptr(w4), _ptr(w_scale), group, _ptr(bias), N, _ptr(y),
                            _ptr(acc), _stream(stream))
    _check(rc, "qgemm_w4a8_g")
    return y


def ql_pack_w4_host(codes):
    """numpy int8 [N,K] in [-8,7] -> numpy uint8 [N,K/2] in the library's 4-bit storage order."""
    import numpy as np
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    N, K = codes.shape
    out = np.empty((N, K // 2), np.uint8)
    rc = lib().ql_pack_w4_host(codes.ctypes.data_as(_vp), N, K, out.ctypes.data_as(_vp))
    _check(rc, "ql_pack_w4_host")
    return out


class Plan:
    """A per-layer weight-bit plan (Algorithm 2, Phase B): list of dicts(K, N, bits, w, w_scale, bias[, group]) of CUDA
    tensors; group = k per weight scale of a 4-bit layer (default 128)."""

    def __init__(self, layers, M_max):
        self._keep = layers  # the plan stores raw pointers: keep the tensors alive
        arr = (ql_layer_desc * len(layers))()
        for i, l in enumerate(layers):
            arr[i] = ql_layer_desc(l["K"], l["N"], l["bits"], l.get("group", 128) if l["bits"] == 4 else 0, l["w"].data_ptr(),
                                   0 if l.get("w_scale") is None else l["w_scale"].data_ptr(),
                                   0 if l.get("bias") is None else l["bias"].data_ptr())
        h = _vp()
        _check(lib().ql_plan_create(arr, len(layers), M_max, ctypes.byref(h)), "ql_plan_create")
        self.handle = h
        self.L = len(layers)
        self.M_max = M_max

    def workspace_bytes(self, M, R):
        return int(lib().ql_plan_workspace_bytes(self.handle, M, R))

    def run(self, x_in, y_out, M, R, ws, stream=None):
        """x_in / y_out: lists of L CUDA tensors ([M,K_l] fp16 / [M,N_l] fp16)."""
        xs = (_vp * self.L)(*[t.data_ptr() for t in x_in])
        ys = (_vp * self.L)(*[t.data_ptr() for t in y_out])
        _check(lib().qlinear_plan_run(self.handle, xs, ys, M, R, _ptr(ws), ws.numel(), _stream(stream)),
               "qlinear_plan_run")

    def run_ptrs(self, xs, ys, M, R, ws, stream_ptr):
        """Same with pre-marshalled pointer arrays (keeps Python out of a timed loop)."""
        _check(lib().qlinear_plan_run(self.handle, xs, ys, M, R, _ptr(ws), ws.numel(), stream_ptr), "qlinear_plan_run")

    def run_ptrs_robust(self, xs, ys, M, R, p_ppm, a_bits, ws, stream_ptr):
        prm = _DaqParams(p_ppm, a_bits)
        _check(lib().qlinear_plan_run_robust(self.handle, xs, ys, M, R, ctypes.byref(prm), _ptr(ws), ws.numel(), stream_ptr),
               "qlinear_plan_run_robust")

    def run_ex(self, x_in, y_out, M, R, ws, fusions=None, p_ppm=None, a_bits=8, stream=None):
        """The plan walk with optional percentile DAQ (p_ppm) and per-layer glue: fusions = list of None or
        dict(act, residual, gate, gate_rows) per layer."""
        xs = (_vp * self.L)(*[t.data_ptr() for t in x_in])
        ys = (_vp * self.L)(*[t.data_ptr() for t in y_out])
        prm = None if p_ppm is None else ctypes.byref(_DaqParams(p_ppm, a_bits))
        fus = None
        keep = []
        if fusions is not None:
            arr = (ctypes.POINTER(ql_fusion) * self.L)()
            for i, f in enumerate(fusions):
                if f is None:
                    continue
                fu = ql_fusion(f.get("act", 0), 0, None if f.get("residual") is None else f["residual"].data_ptr(),
                               None if f.get("gate") is None else f["gate"].data_ptr(), f.get("gate_rows", 1),
                               None if f.get("row_absmax") is None else f["row_absmax"].data_ptr())
                keep.append(fu)
                arr[i] = ctypes.pointer(fu)
            fus = arr
        _check(lib().qlinear_plan_run_ex(self.handle, xs, ys, M, R, prm, fus, _ptr(ws), ws.numel(), _stream(stream)),
               "qlinear_plan_run_ex")

    def close(self):
        if self.handle:
            lib().ql_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ql_planner_layer(ctypes.Structure):
    _fields_ = [("n_options", ctypes.c_int32), ("reserved", ctypes.c_int32), ("bits", ctypes.POINTER(ctypes.c_int32)),
                ("c_lat", ctypes.POINTER(ctypes.c_double)), ("c_mem", ctypes.POINTER(ctypes.c_double)),
                ("sensitivity", ctypes.c_double)]


def schedule_topk(delta, candidates, T, rho_ppm, k):
    """Step 4, eq. (6): the k kept timesteps (ascending) = protected tail + the largest-delta steps of the rest."""
    import numpy as np
    d = np.ascontiguousarray(delta, dtype=np.float64)
    c = np.ascontiguousarray(candidates, dtype=np.int32)
    out = np.empty((max(k, 0),), np.int32)
    rc = lib().ql_schedule_topk(d.ctypes.data_as(_vp), c.ctypes.data_as(_vp), ctypes.c_int32(len(c)), ctypes.c_int32(T),
                                ctypes.c_int32(rho_ppm), ctypes.c_int32(k), out.ctypes.data_as(_vp))
    _check(rc, "ql_schedule_topk")
    return out


def plan_greedy(drift, c_step, layers, B_lat, B_mem, rho_ppm, eps=1e-12):
    """Algorithm 2, Phase A.  layers: list of dict(bits=[...], c_lat=[...], c_mem=[...], sensitivity=s).
    Returns dict(bits=[L], kept=[T] bool, C_lat, C_mem, feasible)."""
    import numpy as np
    dr = np.ascontiguousarray(drift, dtype=np.float64)
    cs = np.ascontiguousarray(c_step, dtype=np.float64)
    T, L = len(dr), len(layers)
    arr = (ql_planner_layer * L)()
    keep = []
    for i, l in enumerate(layers):
        b = np.ascontiguousarray(l["bits"], dtype=np.int32)
        cl = np.ascontiguousarray(l["c_lat"], dtype=np.float64)
        cm = np.ascontiguousarray(l["c_mem"], dtype=np.float64)
        keep += [b, cl, cm]
        arr[i] = ql_planner_layer(len(b), 0, b.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                  cl.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                  cm.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), float(l["sensitivity"]))
    bits = np.empty((L,), np.int32)
    kept = np.empty((T,), np.uint8)
    cl_out, cm_out, feas = ctypes.c_double(), ctypes.c_double(), ctypes.c_int32()
    fn = lib().ql_plan_greedy
    fn.argtypes = [_vp, _vp, ctypes.c_int32, ctypes.POINTER(ql_planner_layer), ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                   ctypes.c_int32, ctypes.c_double, _vp, _vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                   ctypes.POINTER(ctypes.c_int32)]
    rc = fn(dr.ctypes.data_as(_vp), cs.ctypes.data_as(_vp), T, arr, L, B_lat, B_mem, rho_ppm, eps, bits.ctypes.data_as(_vp),
            kept.ctypes.data_as(_vp), ctypes.byref(cl_out), ctypes.byref(cm_out), ctypes.byref(feas))
    _check(rc, "ql_plan_greedy")
    return dict(bits=bits, kept=kept.astype(bool), C_lat=cl_out.value, C_mem=cm_out.value, feasible=bool(feas.value))


def gptq_quantize_host(W, H, bits, group, symmetric=True, damp=0.01, scale_fp16=False):
    """Step 2, GPTQ: W fp32 [N,K], H float64 [K,K] -> (codes int8 [N,K], scales fp32 [N,K/group], zeros int32 [N,K/group])."""
    import numpy as np
    W = np.ascontiguousarray(W, dtype=np.float32)
    H = np.ascontiguousarray(H, dtype=np.float64)
    N, K = W.shape
    codes = np.empty((N, K), np.int8)
    scales = np.empty((N, K // group), np.float32)
    zeros = np.zeros((N, K // group), np.int32)
    fn = lib().ql_gptq_quantize_host
    fn.argtypes = [_vp, _i64, _i64, _vp, ctypes.c_int32, _i64, ctypes.c_int32, ctypes.c_double, ctypes.c_int32, _vp, _vp, _vp]
    rc = fn(W.ctypes.data_as(_vp), N, K, H.ctypes.data_as(_vp), bits, group, 1 if symmetric else 0, damp, 1 if scale_fp16 else 0,
            codes.ctypes.data_as(_vp), scales.ctypes.data_as(_vp), zeros.ctypes.data_as(_vp))
    _check(rc, "ql_gptq_quantize_host")
    return codes, scales, zeros


def set_gemm_variant(v):
    _check(lib().ql_set_gemm_variant(v), "ql_set_gemm_variant")


def gemm_variants():
    L = lib()
    return [L.ql_gemm_variant_name(i).decode() for i in range(L.ql_num_gemm_variants())]


def prepack_w4(pairs, stream=None):
    """Device uint8 [N,K/2] in pair order (low nibble = even k, high nibble = odd k) -> a new device tensor in the
    library's 4-bit storage order."""
    import torch
    N, K2 = pairs.shape
    out = torch.empty_like(pairs)
    _check(lib().ql_prepack_w4(_ptr(pairs), N, K2 * 2, _ptr(out), _stream(stream)), "ql_prepack_w4")
    return out


def ql_repack_w4_pairs_host(pairs):
    """uint8 [N,K/2] in pair order (low nibble = even k, high nibble = odd k) -> the library's 4-bit storage order."""
    import numpy as np
    pairs = np.ascontiguousarray(pairs, dtype=np.uint8)
    N, K2 = pairs.shape
    out = np.empty_like(pairs)
    _check(lib().ql_repack_w4_pairs_host(pairs.ctypes.data_as(_vp), N, K2 * 2, out.ctypes.data_as(_vp)), "ql_repack_w4_pairs_host")
    return out
