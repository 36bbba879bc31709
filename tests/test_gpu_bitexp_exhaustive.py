"""Both arithmetic paths of the softmax kernels (32-bit lanes and packed 16-bit lanes)
against the oracle's exponential for EVERY stabilised score from 0 down past the clamp,
over a sweep of i0 (every value up to 300, then a dense sample up to 2^24), all three variants,
default and zero guard bits.  Uses the library's debug entry that runs the kernels' own
device functions on an array of deltas."""
import ctypes

import numpy as np
import pytest

import paper_2511_15369_amd as ip
from oracle import ref
from tests.helpers import lib_softmax

pytestmark = pytest.mark.gpu
INT32_MIN = -(2 ** 31)


def _run(deltas, p):
    import torch
    lib = ip.load()
    fn = lib.iptq_debug_bit_exp
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                   ctypes.POINTER(ip.SoftmaxParams), ctypes.c_void_p]
    d = torch.from_numpy(deltas.astype(np.int32)).cuda()
    o32 = torch.zeros(d.numel(), dtype=torch.int32, device="cuda")
    o16 = torch.zeros(d.numel(), dtype=torch.int32, device="cuda")
    lp = lib_softmax(p)
    rc = fn(d.data_ptr(), o32.data_ptr(), o16.data_ptr(), d.numel(), ctypes.byref(lp),
            ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    assert rc == 0
    torch.cuda.synchronize()
    return o32.cpu().numpy().astype(np.int64) & 0xFFFFFFFF, o16.cpu().numpy().astype(np.int64) & 0xFFFFFFFF


def _i0_sweep():
    rng = np.random.default_rng(0)
    vals = set(range(16, 301)) | {2 ** k for k in range(4, 24)} | {2 ** k - 1 for k in range(5, 25)}
    vals |= {2 ** k + 1 for k in range(4, 24)}
    vals |= set(int(v) for v in rng.integers(300, 3300, size=120))
    vals |= set(int(v) for v in rng.integers(3300, 2 ** 24, size=60))
    return sorted(v for v in vals if 16 <= v < 2 ** 24)


def test_every_delta_both_paths():
    packed_checked = 0
    for i0 in _i0_sweep():
        for n_shift in sorted({max(0, 15 - i0.bit_length()), 0, max(0, 23 - i0.bit_length())}):
            for variant in (0, 1, 2):
                if variant == 2 and i0 >= 2 ** 16:       # the second-degree form's domain
                    continue
                p = ref.SoftmaxParams(variant=variant, i0=i0, n_shift=n_shift, m_bits=31)
                # everything down to the point where the oracle is identically zero, then extremes
                zero_from = int(np.ceil(33 * i0 / 1.4375)) + 40
                span = min(zero_from, 600000)
                d = -np.arange(0, span + (span & 1), dtype=np.int64)
                tail = np.array([-zero_from, -zero_from - 1, -(2 ** 24), -(2 ** 30), -(2 ** 30) - 1,
                                 INT32_MIN + 1, INT32_MIN, -(2 ** 31) + 2], dtype=np.int64)
                d = np.concatenate([d, tail])
                want = ref.bit_exp_array(d, p)
                want[d == INT32_MIN] = 0
                got32, got16 = _run(d, p)
                assert np.array_equal(got32, want), (i0, n_shift, variant, "32-bit lanes")
                if not (got16 == 0xFFFFFFFF).all():
                    assert np.array_equal(got16, want), (i0, n_shift, variant, "packed lanes")
                    packed_checked += 1
    assert packed_checked > 750
