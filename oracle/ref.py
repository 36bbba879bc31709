"""TEST INFRASTRUCTURE - ctypes front end of the CPU oracle (``iptq_oracle.c``).

Builds the C file with gcc on first use and exposes numpy-in / numpy-out
functions.  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this module; it never touches the HIP library.
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "iptq_oracle.c")
_BUILD = os.path.join(_HERE, "_build")
_LIB = os.path.join(_BUILD, "libiptq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle (gcc -O2, no vectorisation flags beyond the default)."""
    os.makedirs(_BUILD, exist_ok=True)
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


class _Dyadic(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int32), ("s", ctypes.c_int32), ("zp", ctypes.c_int32),
                ("qmin", ctypes.c_int32), ("qmax", ctypes.c_int32)]


class _SoftmaxParams(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("i0", ctypes.c_int32), ("n_shift", ctypes.c_int32),
                ("m_bits", ctypes.c_int32), ("out_bits", ctypes.c_int32),
                ("pre_m", ctypes.c_int32), ("pre_s", ctypes.c_int32),
                ("post", _Dyadic), ("out_is_signed", ctypes.c_int32)]


class _GeluParams(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("q_b", ctypes.c_int32), ("q_c", ctypes.c_int64),
                ("k", ctypes.c_int32), ("zp_in", ctypes.c_int32), ("max_abs_q", ctypes.c_int32),
                ("pre_m", ctypes.c_int32), ("pre_s", ctypes.c_int32), ("post", _Dyadic)]


@dataclass
class Dyadic:
    m: int = 1
    s: int = 0
    zp: int = 0
    qmin: int = 0
    qmax: int = 255

    def c(self) -> _Dyadic:
        return _Dyadic(self.m, self.s, self.zp, self.qmin, self.qmax)


@dataclass
class SoftmaxParams:
    variant: int = 1
    i0: int = 128
    n_shift: int = 7
    m_bits: int = 30
    out_bits: int = 8
    pre_m: int = 1
    pre_s: int = 0
    post: Dyadic = field(default_factory=lambda: Dyadic(1, 0, 0, 0, 255))
    out_is_signed: int = 0

    def c(self) -> _SoftmaxParams:
        return _SoftmaxParams(self.variant, self.i0, self.n_shift, self.m_bits, self.out_bits,
                              self.pre_m, self.pre_s, self.post.c(), self.out_is_signed)


@dataclass
class GeluParams:
    variant: int = 1
    q_b: int = -62
    q_c: int = -13164466
    k: int = 2
    zp_in: int = 0
    max_abs_q: int = 255
    pre_m: int = 1
    pre_s: int = 0
    post: Dyadic = field(default_factory=lambda: Dyadic(-20880, 36, 0, -128, 127))

    def c(self) -> _GeluParams:
        return _GeluParams(self.variant, self.q_b, self.q_c, self.k, self.zp_in, self.max_abs_q,
                           self.pre_m, self.pre_s, self.post.c())


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p, vp = ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p
        lib.iptq_ref_requant.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32,
                                         ctypes.POINTER(_Dyadic)]
        lib.iptq_ref_softmax_i32.argtypes = [vp, vp, ctypes.c_int64, vp, ctypes.c_int64,
                                             ctypes.c_int32, ctypes.POINTER(_SoftmaxParams)]
        lib.iptq_ref_softmax_i32_windowed.argtypes = [vp, vp, ctypes.c_int64, vp, ctypes.c_int64,
                                                      ctypes.c_int64, vp, ctypes.c_int64,
                                                      ctypes.c_int32, ctypes.POINTER(_SoftmaxParams)]
        lib.iptq_ref_softmax_i32_windowed.restype = ctypes.c_int
        lib.iptq_ref_gelu_i8.argtypes = [vp, vp, ctypes.c_int64, ctypes.POINTER(_GeluParams)]
        lib.iptq_ref_gelu_i32.argtypes = [vp, vp, ctypes.c_int64, ctypes.POINTER(_GeluParams)]
        lib.iptq_ref_bit_exp.argtypes = [ctypes.c_int64, ctypes.POINTER(_SoftmaxParams)]
        lib.iptq_ref_bit_exp.restype = ctypes.c_int64
        lib.iptq_ref_bit_exp_array.argtypes = [vp, vp, ctypes.c_int64, ctypes.POINTER(_SoftmaxParams)]
        lib.iptq_ref_bit_exp_array.restype = ctypes.c_int
        for f in (lib.iptq_ref_requant, lib.iptq_ref_softmax_i32, lib.iptq_ref_gelu_i8,
                  lib.iptq_ref_gelu_i32):
            f.restype = ctypes.c_int
        del i32p
        _lib = lib
    return _lib


class OracleError(ValueError):
    pass


def _check(rc: int, what: str):
    if rc != 0:
        raise OracleError("%s rejected its arguments (code %d)" % (what, rc))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def requant(x: np.ndarray, d: Dyadic, out_is_signed: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int32)
    out = np.empty(x.shape, dtype=np.int8 if out_is_signed else np.uint8)
    dc = d.c()
    _check(_load().iptq_ref_requant(_ptr(x), _ptr(out), x.size, out_is_signed,
                                    ctypes.byref(dc)), "requant")
    return out


def softmax_i32(scores: np.ndarray, p: SoftmaxParams, bias: Optional[np.ndarray] = None,
                bias_period_rows: int = 0) -> np.ndarray:
    scores = np.ascontiguousarray(scores, dtype=np.int32)
    assert scores.ndim == 2
    rows, cols = scores.shape
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.int32)
        assert bias.shape == (bias_period_rows, cols)
    out = np.empty((rows, cols), dtype=np.int8 if p.out_is_signed else np.uint8)
    pc = p.c()
    _check(_load().iptq_ref_softmax_i32(_ptr(scores), _ptr(bias), bias_period_rows, _ptr(out),
                                        rows, cols, ctypes.byref(pc)), "softmax_i32")
    return out


def softmax_i32_windowed(scores: np.ndarray, p: SoftmaxParams, bias: Optional[np.ndarray],
                         bias_period_rows: int, mask: Optional[np.ndarray], heads: int) -> np.ndarray:
    """Rows ordered [image, window, head, query]; mask [n_windows, cols, cols] (0 / INT32_MIN
    or any additive int32), added beside the bias of period heads * cols."""
    scores = np.ascontiguousarray(scores, dtype=np.int32)
    rows, cols = scores.shape
    if bias is not None:
        bias = np.ascontiguousarray(bias, dtype=np.int32)
        assert bias.shape == (bias_period_rows, cols)
    n_windows = 0
    if mask is not None:
        mask = np.ascontiguousarray(mask, dtype=np.int32)
        assert mask.ndim == 3 and mask.shape[1:] == (cols, cols)
        n_windows = mask.shape[0]
    out = np.empty((rows, cols), dtype=np.int8 if p.out_is_signed else np.uint8)
    pc = p.c()
    _check(_load().iptq_ref_softmax_i32_windowed(_ptr(scores), _ptr(bias), bias_period_rows,
                                                 _ptr(mask), n_windows, heads, _ptr(out), rows,
                                                 cols, ctypes.byref(pc)), "softmax_i32_windowed")
    return out


def pack_window_mask(mask: np.ndarray) -> np.ndarray:
    """One bit per key of a 0 / INT32_MIN window mask [n_windows, cols, cols]: uint64
    [n_windows, cols, ceil(cols / 64)], bit (k mod 64) of word (k div 64) of row [w, q] set where
    mask[w, q, k] == INT32_MIN (any other value counts as "not masked").  Plain loops."""
    mask = np.asarray(mask, dtype=np.int32)
    n_w, cols, cols2 = mask.shape
    assert cols == cols2
    words = (cols + 63) // 64
    out = np.zeros((n_w, cols, words), dtype=np.uint64)
    for w in range(n_w):
        for q in range(cols):
            for k in range(cols):
                if int(mask[w, q, k]) == -(2 ** 31):
                    out[w, q, k // 64] |= np.uint64(1) << np.uint64(k % 64)
    return out


def unpack_window_mask(bits: np.ndarray, cols: int) -> np.ndarray:
    """The 0 / INT32_MIN mask a packed one stands for (bits beyond `cols` are ignored)."""
    bits = np.asarray(bits, dtype=np.uint64)
    n_w = bits.shape[0]
    out = np.zeros((n_w, cols, cols), dtype=np.int32)
    for w in range(n_w):
        for q in range(cols):
            for k in range(cols):
                if (int(bits[w, q, k // 64]) >> (k % 64)) & 1:
                    out[w, q, k] = -(2 ** 31)
    return out


def softmax_i32_windowed_bits(scores, p, bias, bias_period_rows, bits, heads) -> np.ndarray:
    """The windowed softmax with the mask given one bit per key: by definition the windowed
    softmax with the 0 / INT32_MIN mask those bits stand for."""
    cols = scores.shape[1]
    return softmax_i32_windowed(scores, p, bias, bias_period_rows, unpack_window_mask(bits, cols), heads)


def gelu_i8(x: np.ndarray, p: GeluParams) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int8)
    out = np.empty(x.shape, dtype=np.int8)
    pc = p.c()
    _check(_load().iptq_ref_gelu_i8(_ptr(x), _ptr(out), x.size, ctypes.byref(pc)), "gelu_i8")
    return out


def gelu_i32(x: np.ndarray, p: GeluParams) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.int32)
    out = np.empty(x.shape, dtype=np.int8)
    pc = p.c()
    _check(_load().iptq_ref_gelu_i32(_ptr(x), _ptr(out), x.size, ctypes.byref(pc)), "gelu_i32")
    return out


def bit_exp(delta: int, p: SoftmaxParams) -> int:
    pc = p.c()
    return int(_load().iptq_ref_bit_exp(int(delta), ctypes.byref(pc)))


def bit_exp_array(delta: np.ndarray, p: SoftmaxParams) -> np.ndarray:
    """Q_exp of every stabilised score in `delta` (<= 0), with the clamp at -2^30."""
    delta = np.ascontiguousarray(delta, dtype=np.int64)
    out = np.empty(delta.shape, dtype=np.int64)
    pc = p.c()
    _check(_load().iptq_ref_bit_exp_array(_ptr(delta), _ptr(out), delta.size, ctypes.byref(pc)),
           "bit_exp_array")
    return out
