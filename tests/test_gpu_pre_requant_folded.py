"""The requantization in front of the softmax folded into Eq. 6 (one multiply-add per score on
the raw difference to the row maximum instead of a 64-bit requantization of every score):
bit-exact against the oracle's requantize-then-subtract on the parameter range that enables
it, at rounding ties, with masked entries and with rows near INT32_MIN that must fall back."""
import ctypes

import numpy as np
import pytest

import paper_2511_15369_amd as ip
from oracle import ref
from tests.helpers import gpu_softmax, lib_softmax

pytestmark = pytest.mark.gpu
INT32_MIN = -(2 ** 31)


def _folded(p, cols):
    fn = ip.load().iptq_debug_softmax_plan
    fn.argtypes = [ctypes.POINTER(ip.SoftmaxParams), ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                   ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
    out = (ctypes.c_int64 * 12)()
    lp = lib_softmax(p)
    assert fn(ctypes.byref(lp), 1, cols, 0, 0, out) == 0
    return int(out[11])


@pytest.mark.parametrize("cols", [197, 49, 144, 257])
def test_folded_requant_parameter_sweep(cols):
    rng = np.random.default_rng(cols)
    used = 0
    for trial in range(60):
        i0 = int(rng.choice([16, 17, 23, 40, 64, 100, 181]))
        n = int(rng.integers(0, 15 - i0.bit_length() + 1))
        pre_s = int(rng.integers(16, 32))
        pre_m = int(rng.integers(1, 32768))
        signed = int(rng.integers(0, 2))
        p = ref.SoftmaxParams(variant=int(rng.integers(0, 2)), i0=i0, n_shift=n, pre_m=pre_m, pre_s=pre_s,
                              post=ref.Dyadic(1, 0, 0, 0, 127 if signed else 255), out_is_signed=signed)
        dmax = _folded(p, cols)
        used += dmax > 0
        ratio = pre_m / 2.0 ** pre_s
        rows = int(rng.integers(20, 90))
        # requantized scores spread over a few units of 1 / S_delta
        x = np.rint(rng.standard_normal((rows, cols)) * 2.0 * i0 / ratio)
        x += np.rint(rng.uniform(-2 ** 30, 2 ** 30))
        x = np.clip(x, INT32_MIN + 1, 2 ** 31 - 1).astype(np.int64)
        if dmax:
            # entries exactly at, one below and one above the clamp of the raw difference
            x[0, 1:4] = x[0].max() - np.array([dmax - 1, dmax, dmax + 1])
            # rounding ties: raw values whose product with m lands on odd multiples of 2^(s-1)
            k = np.arange(cols)
            x[1] = x[1].max() - ((k * (1 << pre_s) + (1 << (pre_s - 1))) // pre_m)
            x[2] = x[2].max() - (-(-(k * (1 << pre_s) + (1 << (pre_s - 1))) // pre_m))
        x = np.clip(x, INT32_MIN + 1, 2 ** 31 - 1).astype(np.int32)
        x[rng.random(x.shape) < 0.03] = INT32_MIN
        x[3, :] = INT32_MIN                                        # all masked
        x[4, :] = INT32_MIN + 1 + rng.integers(0, 40, cols)       # a row next to the sentinel: falls back
        x[4, ::3] = INT32_MIN
        x[5, :] = 2 ** 31 - 1 - rng.integers(0, 40, cols)
        want = ref.softmax_i32(x, p)
        for algo in (0, 4):
            assert np.array_equal(gpu_softmax(x, p, algo=algo), want), (trial, p, dmax, algo)
    assert used >= 20                                              # the folded form was exercised


def test_folded_requant_is_what_the_benchmark_leg_runs():
    p = ref.SoftmaxParams(variant=1, i0=16, n_shift=10, pre_m=20000, pre_s=24)
    assert _folded(p, 197) > 0
    # not with shifts below 16, shifts above 31, or a scale too fine for the product to fit 32 bits
    assert _folded(ref.SoftmaxParams(variant=1, i0=16, n_shift=10, pre_m=20000, pre_s=15), 197) == 0
    assert _folded(ref.SoftmaxParams(variant=1, i0=16, n_shift=10, pre_m=20000, pre_s=40), 197) == 0
    assert _folded(ref.SoftmaxParams(variant=1, i0=1000, n_shift=4, pre_m=20000, pre_s=28), 197) == 0
