"""ctypes binding of ``libiptq.so``: argument marshalling only.

Every function has the name and the argument order of its C entry point
(``include/iptq.h``).  Device tensors are torch tensors on the GPU; only their
``data_ptr()`` crosses the boundary, together with the current torch stream.
There is no CPU fallback: if the library is missing, loading raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libiptq.so")
_lib = None

ALGO_AUTO = 0
ALGO_GENERIC = 1
ALGO_DYNAMIC = 2
ALGO_WIDE = 3
ALGO_SLAB = 4


class IptqError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__("%s failed: %s (code %d)" % (what, strerror(code), code))


class Dyadic(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("s", ctypes.c_int32), ("zp", ctypes.c_int32),
                ("qmin", ctypes.c_int32), ("qmax", ctypes.c_int32)]


class SoftmaxParams(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("i0", ctypes.c_int32), ("n_shift", ctypes.c_int32),
                ("m_bits", ctypes.c_int32), ("out_bits", ctypes.c_int32),
                ("pre_m", ctypes.c_int32), ("pre_s", ctypes.c_int32),
                ("post", Dyadic), ("out_is_signed", ctypes.c_int32), ("algo", ctypes.c_int32)]


class GeluParams(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("q_b", ctypes.c_int32), ("q_c", ctypes.c_int64),
                ("k", ctypes.c_int32), ("zp_in", ctypes.c_int32), ("max_abs_q", ctypes.c_int32),
                ("pre_m", ctypes.c_int32), ("pre_s", ctypes.c_int32), ("post", Dyadic),
                ("algo", ctypes.c_int32)]


class Metric(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("q_db", "p", "c", "n_q", "n_p", "n_c", "score")]


METRIC_LITERAL = 0
METRIC_PER_ELEMENT = 1


class SoftmaxProblem(ctypes.Structure):
    _fields_ = [("d_scores", ctypes.c_void_p), ("d_bias", ctypes.c_void_p),
                ("bias_period_rows", ctypes.c_int64), ("d_out", ctypes.c_void_p),
                ("rows", ctypes.c_int64), ("params", SoftmaxParams), ("d_mask", ctypes.c_void_p),
                ("n_windows", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("d_mask_bits", ctypes.c_void_p)]


class GeluProblem(ctypes.Structure):
    _fields_ = [("d_in", ctypes.c_void_p), ("d_out", ctypes.c_void_p), ("n", ctypes.c_int64),
                ("params", GeluParams)]


BATCH_MAX = 16


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load the shared library (built by ``python -m paper_2511_15369_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("libiptq.so is not built: run `python -m paper_2511_15369_amd.build` "
                          "(there is no fallback path)")
    # torch first: it brings its own copy of the HIP runtime, and the library must bind to that
    # one (the device buffers and streams come from it).  Loaded before torch, libiptq.so would
    # pull in the system's copy and every launch would go to a second runtime that has no device.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    lib.iptq_version.restype = ctypes.c_int
    lib.iptq_strerror.restype = ctypes.c_char_p
    lib.iptq_strerror.argtypes = [ctypes.c_int]
    lib.iptq_requant.argtypes = [vp, vp, i64, i32, ctypes.POINTER(Dyadic), vp]
    lib.iptq_softmax_i32.argtypes = [vp, vp, i64, vp, i64, i32, ctypes.POINTER(SoftmaxParams), vp]
    lib.iptq_softmax_i32_windowed.argtypes = [vp, vp, i64, vp, i32, i32, vp, i64, i32,
                                              ctypes.POINTER(SoftmaxParams), vp]
    lib.iptq_softmax_i32_windowed.restype = ctypes.c_int
    lib.iptq_softmax_i32_windowed_bits.argtypes = [vp, vp, i64, vp, i32, i32, vp, i64, i32,
                                                   ctypes.POINTER(SoftmaxParams), vp]
    lib.iptq_softmax_i32_windowed_bits.restype = ctypes.c_int
    lib.iptq_pack_window_mask.argtypes = [vp, i32, i32, vp, vp]
    lib.iptq_pack_window_mask.restype = ctypes.c_int
    lib.iptq_gelu_i8.argtypes = [vp, vp, i64, ctypes.POINTER(GeluParams), vp]
    lib.iptq_gelu_i32.argtypes = [vp, vp, i64, ctypes.POINTER(GeluParams), vp]
    lib.iptq_softmax_i32_layers.argtypes = [vp, i64, vp, i64, i64, i32, i32,
                                            ctypes.POINTER(SoftmaxParams), vp]
    lib.iptq_gelu_i8_layers.argtypes = [vp, i64, vp, i64, i64, i32, ctypes.POINTER(GeluParams), vp]
    lib.iptq_softmax_i32_batch.argtypes = [ctypes.POINTER(SoftmaxProblem), i32, i32, vp]
    lib.iptq_gelu_i8_batch.argtypes = [ctypes.POINTER(GeluProblem), i32, vp]
    lib.iptq_make_dyadic.argtypes = [ctypes.c_double, ctypes.POINTER(i32), ctypes.POINTER(i32)]
    lib.iptq_softmax_prepare.argtypes = [ctypes.c_double, i32, i32, i32,
                                         ctypes.POINTER(SoftmaxParams)]
    lib.iptq_gelu_prepare.argtypes = [ctypes.c_double, ctypes.c_double, i32, i32, i32, i32,
                                      ctypes.POINTER(GeluParams)]
    lib.iptq_unified_metric.argtypes = [vp, vp, i64, ctypes.c_double, i32, ctypes.POINTER(Metric)]
    lib.iptq_unified_metric.restype = ctypes.c_int
    lib.iptq_unified_select.argtypes = [ctypes.POINTER(Metric), i32, ctypes.POINTER(i32)]
    lib.iptq_unified_select.restype = ctypes.c_int
    lib.iptq_softmax_op_count.argtypes = [i32, i64, i32]
    lib.iptq_softmax_op_count.restype = ctypes.c_int64
    lib.iptq_gelu_op_count.argtypes = [i32, i64]
    lib.iptq_gelu_op_count.restype = ctypes.c_int64
    lib.iptq_softmax_kernel_family.argtypes = [i32, ctypes.POINTER(i32), ctypes.POINTER(i32),
                                               ctypes.POINTER(i32)]
    lib.iptq_softmax_kernel_family.restype = ctypes.c_int
    for name in ("iptq_requant", "iptq_softmax_i32", "iptq_gelu_i8", "iptq_gelu_i32",
                 "iptq_softmax_i32_layers", "iptq_gelu_i8_layers", "iptq_softmax_i32_batch",
                 "iptq_gelu_i8_batch", "iptq_make_dyadic",
                 "iptq_softmax_prepare", "iptq_gelu_prepare"):
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def version() -> int:
    return int(load().iptq_version())


def strerror(code: int) -> str:
    return load().iptq_strerror(int(code)).decode()


def _check(rc: int, what: str):
    if rc != 0:
        raise IptqError(rc, what)


_raw_stream = None


def _stream():
    """The current torch stream of the current device as a raw hipStream_t."""
    global _raw_stream
    import torch
    if _raw_stream is None:
        fast = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        if fast is not None:
            _raw_stream = lambda: fast(torch.cuda.current_device())
        else:
            _raw_stream = lambda: torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(_raw_stream())


def _dptr(t) -> Optional[int]:
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _need(t, dtype, what):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError("%s must be a contiguous %s tensor on the GPU" % (what, dtype))


# ----------------------------------------------------------------------------- host helpers
def make_dyadic(ratio: float):
    m, s = ctypes.c_int32(), ctypes.c_int32()
    _check(load().iptq_make_dyadic(ratio, ctypes.byref(m), ctypes.byref(s)), "iptq_make_dyadic")
    return m.value, s.value


def softmax_prepare(s_delta: float, cols: int, variant: int, out_is_signed: int = 0) -> SoftmaxParams:
    p = SoftmaxParams()
    _check(load().iptq_softmax_prepare(s_delta, cols, variant, out_is_signed, ctypes.byref(p)),
           "iptq_softmax_prepare")
    return p


def gelu_prepare(s_in: float, s_out: float, zp_in: int, zp_out: int, variant: int,
                 max_abs_q: int = 255) -> GeluParams:
    p = GeluParams()
    _check(load().iptq_gelu_prepare(s_in, s_out, zp_in, zp_out, variant, max_abs_q,
                                    ctypes.byref(p)), "iptq_gelu_prepare")
    return p


def unified_metric(x, x_hat, op_count: float, mode: int = METRIC_LITERAL) -> Metric:
    """x, x_hat: contiguous float64 numpy arrays of the same size (host)."""
    import numpy as np
    assert isinstance(x, np.ndarray) and isinstance(x_hat, np.ndarray)
    assert x.dtype == np.float64 and x_hat.dtype == np.float64 and x.size == x_hat.size
    assert x.flags["C_CONTIGUOUS"] and x_hat.flags["C_CONTIGUOUS"]
    out = Metric()
    _check(load().iptq_unified_metric(x.ctypes.data_as(ctypes.c_void_p), x_hat.ctypes.data_as(ctypes.c_void_p),
                                      x.size, float(op_count), mode, ctypes.byref(out)),
           "iptq_unified_metric")
    return out


def unified_select(candidates: Sequence[Metric]) -> int:
    arr = (Metric * max(len(candidates), 1))(*candidates)
    best = ctypes.c_int32()
    _check(load().iptq_unified_select(arr, len(candidates), ctypes.byref(best)), "iptq_unified_select")
    return best.value


def softmax_op_count(variant: int, rows: int, cols: int) -> int:
    return int(load().iptq_softmax_op_count(variant, rows, cols))


def gelu_op_count(variant: int, n: int) -> int:
    return int(load().iptq_gelu_op_count(variant, n))


# ----------------------------------------------------------------------------- device calls
def softmax_kernel_family(cols: int) -> str:
    """Which softmax kernel serves 16-byte aligned tensors of this row length."""
    fn = load().iptq_softmax_kernel_family
    fam, lanes, blocks = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    _check(fn(cols, ctypes.byref(fam), ctypes.byref(lanes), ctypes.byref(blocks)),
           "iptq_softmax_kernel_family")
    names = {0: "compiled row length", 1: "slab, %d lanes x %d blocks per row",
             2: "wavefront per row (%d lanes), %d passes", 3: "workgroup of %d lanes per row, %d passes",
             4: "three-pass"}
    text = names[fam.value]
    return text % (lanes.value, blocks.value) if "%d" in text else text


def requant(d_in, d_out, n: int, out_is_signed: int, p: Dyadic):
    import torch
    _need(d_in, torch.int32, "d_in")
    _need(d_out, torch.int8 if out_is_signed else torch.uint8, "d_out")
    assert d_in.numel() >= n and d_out.numel() >= n
    _check(load().iptq_requant(_dptr(d_in), _dptr(d_out), n, out_is_signed, ctypes.byref(p),
                               _stream()), "iptq_requant")


def softmax_i32(d_scores, d_bias, bias_period_rows: int, d_out, rows: int, cols: int,
                p: SoftmaxParams):
    import torch
    _need(d_scores, torch.int32, "d_scores")
    _need(d_out, torch.int8 if p.out_is_signed else torch.uint8, "d_out")
    assert d_scores.numel() >= rows * cols and d_out.numel() >= rows * cols
    if d_bias is not None:
        _need(d_bias, torch.int32, "d_bias")
        assert d_bias.numel() >= bias_period_rows * cols
    _check(load().iptq_softmax_i32(_dptr(d_scores), _dptr(d_bias), bias_period_rows, _dptr(d_out),
                                   rows, cols, ctypes.byref(p), _stream()), "iptq_softmax_i32")


def softmax_i32_windowed(d_scores, d_bias, bias_period_rows: int, d_mask, n_windows: int, heads: int,
                         d_out, rows: int, cols: int, p: SoftmaxParams):
    import torch
    _need(d_scores, torch.int32, "d_scores")
    _need(d_out, torch.int8 if p.out_is_signed else torch.uint8, "d_out")
    assert d_scores.numel() >= rows * cols and d_out.numel() >= rows * cols
    if d_bias is not None:
        _need(d_bias, torch.int32, "d_bias")
        assert d_bias.numel() >= bias_period_rows * cols
    if d_mask is not None:
        _need(d_mask, torch.int32, "d_mask")
        assert d_mask.numel() >= n_windows * cols * cols
    _check(load().iptq_softmax_i32_windowed(_dptr(d_scores), _dptr(d_bias), bias_period_rows,
                                            _dptr(d_mask), n_windows, heads, _dptr(d_out), rows,
                                            cols, ctypes.byref(p), _stream()),
           "iptq_softmax_i32_windowed")


def softmax_i32_windowed_bits(d_scores, d_bias, bias_period_rows: int, d_mask_bits, n_windows: int,
                              heads: int, d_out, rows: int, cols: int, p: SoftmaxParams):
    import torch
    _need(d_scores, torch.int32, "d_scores")
    _need(d_out, torch.int8 if p.out_is_signed else torch.uint8, "d_out")
    assert d_scores.numel() >= rows * cols and d_out.numel() >= rows * cols
    if d_bias is not None:
        _need(d_bias, torch.int32, "d_bias")
        assert d_bias.numel() >= bias_period_rows * cols
    if d_mask_bits is not None:
        _need(d_mask_bits, torch.int64, "d_mask_bits")        # torch has no uint64 arithmetic: the words travel as int64
        assert d_mask_bits.numel() >= n_windows * cols * ((cols + 63) // 64)
    _check(load().iptq_softmax_i32_windowed_bits(_dptr(d_scores), _dptr(d_bias), bias_period_rows,
                                                 _dptr(d_mask_bits), n_windows, heads, _dptr(d_out),
                                                 rows, cols, ctypes.byref(p), _stream()),
           "iptq_softmax_i32_windowed_bits")


def pack_window_mask(d_mask, n_windows: int, cols: int, d_mask_bits):
    import torch
    _need(d_mask, torch.int32, "d_mask")
    _need(d_mask_bits, torch.int64, "d_mask_bits")
    assert d_mask.numel() >= n_windows * cols * cols
    assert d_mask_bits.numel() >= n_windows * cols * ((cols + 63) // 64)
    _check(load().iptq_pack_window_mask(_dptr(d_mask), n_windows, cols, _dptr(d_mask_bits), _stream()),
           "iptq_pack_window_mask")


def gelu_i8(d_in, d_out, n: int, p: GeluParams):
    import torch
    _need(d_in, torch.int8, "d_in")
    _need(d_out, torch.int8, "d_out")
    assert d_in.numel() >= n and d_out.numel() >= n
    _check(load().iptq_gelu_i8(_dptr(d_in), _dptr(d_out), n, ctypes.byref(p), _stream()),
           "iptq_gelu_i8")


def gelu_i32(d_in, d_out, n: int, p: GeluParams):
    import torch
    _need(d_in, torch.int32, "d_in")
    _need(d_out, torch.int8, "d_out")
    assert d_in.numel() >= n and d_out.numel() >= n
    _check(load().iptq_gelu_i32(_dptr(d_in), _dptr(d_out), n, ctypes.byref(p), _stream()),
           "iptq_gelu_i32")


def softmax_i32_layers(d_scores, in_stride: int, d_out, out_stride: int, rows: int, cols: int,
                       n_layers: int, params: Sequence[SoftmaxParams]):
    import torch
    _need(d_scores, torch.int32, "d_scores")
    assert len(params) == n_layers
    signed = params[0].out_is_signed if n_layers else 0
    _need(d_out, torch.int8 if signed else torch.uint8, "d_out")
    if n_layers:
        assert d_scores.numel() >= (n_layers - 1) * in_stride + rows * cols
        assert d_out.numel() >= (n_layers - 1) * out_stride + rows * cols
    arr = (SoftmaxParams * max(n_layers, 1))(*params)
    _check(load().iptq_softmax_i32_layers(_dptr(d_scores), in_stride, _dptr(d_out), out_stride,
                                          rows, cols, n_layers, arr, _stream()),
           "iptq_softmax_i32_layers")


def gelu_i8_layers(d_in, in_stride: int, d_out, out_stride: int, n: int, n_layers: int,
                   params: Sequence[GeluParams]):
    import torch
    _need(d_in, torch.int8, "d_in")
    _need(d_out, torch.int8, "d_out")
    assert len(params) == n_layers
    if n_layers:
        assert d_in.numel() >= (n_layers - 1) * in_stride + n
        assert d_out.numel() >= (n_layers - 1) * out_stride + n
    arr = (GeluParams * max(n_layers, 1))(*params)
    _check(load().iptq_gelu_i8_layers(_dptr(d_in), in_stride, _dptr(d_out), out_stride, n,
                                      n_layers, arr, _stream()), "iptq_gelu_i8_layers")


def softmax_problem(d_scores, d_bias, bias_period_rows: int, d_out, rows: int, cols: int,
                    p: SoftmaxParams, d_mask=None, n_windows: int = 0, heads: int = 0,
                    d_mask_bits=None) -> SoftmaxProblem:
    """One entry of a softmax batch (same checks as softmax_i32)."""
    import torch
    _need(d_scores, torch.int32, "d_scores")
    _need(d_out, torch.int8 if p.out_is_signed else torch.uint8, "d_out")
    assert d_scores.numel() >= rows * cols and d_out.numel() >= rows * cols
    if d_bias is not None:
        _need(d_bias, torch.int32, "d_bias")
        assert d_bias.numel() >= bias_period_rows * cols
    if d_mask is not None:
        _need(d_mask, torch.int32, "d_mask")
        assert d_mask.numel() >= n_windows * cols * cols
    if d_mask_bits is not None:
        _need(d_mask_bits, torch.int64, "d_mask_bits")
        assert d_mask_bits.numel() >= n_windows * cols * ((cols + 63) // 64)
    return SoftmaxProblem(d_scores.data_ptr(), None if d_bias is None else d_bias.data_ptr(),
                          bias_period_rows, d_out.data_ptr(), rows, p,
                          None if d_mask is None else d_mask.data_ptr(), n_windows, heads,
                          None if d_mask_bits is None else d_mask_bits.data_ptr())


def gelu_problem(d_in, d_out, n: int, p: GeluParams) -> GeluProblem:
    import torch
    _need(d_in, torch.int8, "d_in")
    _need(d_out, torch.int8, "d_out")
    assert d_in.numel() >= n and d_out.numel() >= n
    return GeluProblem(d_in.data_ptr(), d_out.data_ptr(), n, p)


def softmax_i32_batch(problems, n_problems: int, cols: int):
    """problems: a ctypes array (SoftmaxProblem * n) or a sequence of SoftmaxProblem."""
    if not isinstance(problems, ctypes.Array):
        problems = (SoftmaxProblem * max(n_problems, 1))(*problems)
    _check(load().iptq_softmax_i32_batch(problems, n_problems, cols, _stream()),
           "iptq_softmax_i32_batch")


def gelu_i8_batch(problems, n_problems: int):
    if not isinstance(problems, ctypes.Array):
        problems = (GeluProblem * max(n_problems, 1))(*problems)
    _check(load().iptq_gelu_i8_batch(problems, n_problems, _stream()), "iptq_gelu_i8_batch")
