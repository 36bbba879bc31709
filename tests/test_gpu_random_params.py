"""GPU parity on random parameter sets drawn from the whole documented domain (not only the
values the derivation helpers produce): every softmax kernel family and arithmetic mode, the
int8 / int32 GELU with arbitrary constants, against the oracle, bit for bit."""
import numpy as np
import pytest

from oracle import ref
from oracle import prepare
from tests.helpers import gpu_gelu_i8, gpu_gelu_i32, gpu_softmax, lib_softmax

pytestmark = pytest.mark.gpu
I32_MIN, I32_MAX = -(2 ** 31), 2 ** 31 - 1


@pytest.mark.parametrize("seed", range(5))
def test_softmax_random_domain(seed):
    rng = np.random.default_rng(1000 + seed)
    for _ in range(40):
        cols = int(rng.choice([49, 197, 198, 144, 257, 577, 31, 64, 100, 333, 830, 1025, 2047, 4097, 6001,
                               14002, 30001]))
        rows = int(rng.integers(1, 150)) if cols < 1000 else int(rng.integers(1, 12))
        i0 = int(rng.choice([16, 17, 31, 100, 181, 255, 256, 257, 1000, 3139, 3141, 4095, 65536,
                             2 ** 20 + 3, 2 ** 24 - 1]))
        out_bits = int(rng.integers(2, 9))
        n_max = 0
        while ((i0 << (n_max + 1)) < 2 ** 24) and n_max < 20:
            n_max += 1
        n_shift = int(rng.integers(0, n_max + 1))
        need = (cols * (i0 << n_shift)).bit_length()
        if need > 31:
            n_shift = 0
            need = (cols * i0).bit_length()
            if need > 31:
                continue
        m_bits = int(rng.integers(max(out_bits - 1, need), 32))
        if cols * (i0 << n_shift) > (1 << m_bits):
            continue
        signed = int(rng.integers(0, 2))
        lo, hi = (-128, 127) if signed else (0, 255)
        choice = rng.integers(0, 3)
        if choice == 0:
            post = ref.Dyadic(1, 0, 0, 0 if not signed else int(rng.integers(-128, 1)), hi)
        elif choice == 1:
            post = ref.Dyadic(1, 0, 0, 0, 127)
        else:
            post = ref.Dyadic(int(rng.integers(-32767, 32768)), int(rng.integers(0, 63)),
                              int(rng.integers(-200, 200)), lo, hi)
        pre = (1, 0) if rng.integers(0, 3) else (int(rng.integers(1, 32768)), int(rng.integers(0, 63)))
        variant = int(rng.integers(0, 3))
        if variant == 2 and i0 >= 2 ** 16:                   # the second-degree form's domain
            variant = 1
        p = ref.SoftmaxParams(variant=variant, i0=i0, n_shift=n_shift, m_bits=m_bits,
                              out_bits=out_bits, pre_m=pre[0], pre_s=pre[1], post=post,
                              out_is_signed=signed)
        kind = rng.integers(0, 3)
        if kind == 0:
            x = rng.integers(I32_MIN, I32_MAX + 1, size=(rows, cols))
        elif kind == 1:
            x = np.rint(rng.standard_normal((rows, cols)) * 3.0 * i0)
        else:
            x = np.rint(rng.standard_normal((rows, cols)) * 40.0 * i0) + rng.integers(-2 ** 30, 2 ** 30)
        x = np.clip(x, I32_MIN, I32_MAX).astype(np.int32)
        x[rng.random((rows, cols)) < 0.05] = I32_MIN
        bias, period = None, 0
        if rng.integers(0, 2):
            period = int(rng.choice([1, 3, 64, 96]))
            bias = np.rint(rng.standard_normal((period, cols)) * 2.0 * i0).astype(np.int32)
            bias[rng.random((period, cols)) < 0.02] = I32_MIN
        want = ref.softmax_i32(x, p, bias, period)
        for algo in (0, 1, 2, 3, 4):
            got = gpu_softmax(x, p, bias, period, algo=algo)
            assert np.array_equal(got, want), (algo, cols, rows, p)


@pytest.mark.parametrize("seed", range(4))
def test_softmax_random_row_lengths_and_views(seed):
    """Row lengths drawn from 1 to 41000 (every layout of the run-time-length kernels), row
    counts that leave partial slabs, additive tables of several periods, and views that start
    off the 16-byte grid at the same element of the score and output buffers: bit-exact, and no
    byte outside the view written."""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(3000 + seed)
    for it in range(250):
        cols = int(np.exp(rng.uniform(0, np.log(41000)))) if rng.integers(0, 4) else int(rng.integers(1, 900))
        cols = max(1, min(cols, 41000))
        rows = int(rng.integers(1, 300)) if cols < 1000 else int(rng.integers(1, 7))
        signed = int(rng.integers(0, 2))
        p = prepare.softmax_prepare(2.0 ** rng.uniform(-10, -4), cols, int(rng.integers(0, 2)), out_is_signed=signed)
        if rng.integers(0, 4) == 0:
            p.post = ref.Dyadic(int(rng.integers(1, 300)), int(rng.integers(0, 9)), int(rng.integers(-5, 6)),
                                -128 if signed else 0, 127 if signed else 255)
        if rng.integers(0, 4) == 0:
            p.pre_m, p.pre_s = int(rng.integers(1, 32768)), int(rng.integers(8, 30))
        kind = rng.integers(0, 3)
        scale = (3.0 if kind == 0 else 40.0) * p.i0
        if (p.pre_m, p.pre_s) != (1, 0):
            scale *= 2.0 ** p.pre_s / p.pre_m
        x = np.rint(rng.standard_normal((rows, cols)) * min(scale, 2.0 ** 30))
        if kind == 2:
            x += rng.integers(-2 ** 30, 2 ** 30)
        x = np.clip(x, I32_MIN, I32_MAX).astype(np.int32)
        x[rng.random((rows, cols)) < 0.03] = I32_MIN
        if rng.integers(0, 8) == 0:
            x[rng.integers(0, rows)] = I32_MIN
        bias, period, off = None, 0, 0
        if rng.integers(0, 3) == 0:
            period = int(rng.choice([1, 2, 3, 4, 8, 64, 65, 147]))
            bias = np.rint(rng.standard_normal((period, cols)) * 2.0 * p.i0).astype(np.int32)
            bias[rng.random((period, cols)) < 0.02] = I32_MIN
        elif rng.integers(0, 2):
            off = int(rng.integers(1, 8))
        ooff = off if rng.integers(0, 2) else int(rng.integers(0, 17))      # output view: same or another offset
        want = ref.softmax_i32(x, p, bias, period).view(np.uint8).reshape(-1)
        n = rows * cols
        d_in = torch.zeros(n + 16, dtype=torch.int32, device="cuda")
        d_in[off:off + n] = torch.from_numpy(x.reshape(-1)).cuda()
        d_bias = torch.from_numpy(bias).cuda() if bias is not None else None
        for algo in (0, 2, 3, 4):
            d_out = torch.full((n + 32,), 0x5A, dtype=torch.uint8, device="cuda").view(torch.int8 if signed else torch.uint8)
            ip.softmax_i32(d_in[off:off + n], d_bias, period, d_out[ooff:ooff + n], rows, cols, lib_softmax(p, algo))
            torch.cuda.synchronize()
            got = d_out.view(torch.uint8).cpu().numpy()
            assert np.array_equal(got[ooff:ooff + n], want), (it, cols, rows, algo, off, ooff, period, p)
            assert (got[:ooff] == 0x5A).all() and (got[ooff + n:] == 0x5A).all(), (it, cols, rows, algo, off, ooff)


@pytest.mark.parametrize("seed", range(3))
def test_gelu_random_domain(seed):
    rng = np.random.default_rng(2000 + seed)
    done = 0
    while done < 60:
        variant = int(rng.integers(0, 2))
        q_b = -int(rng.integers(1, 2 ** int(rng.integers(2, 15 if variant else 30))))
        q_c = -int(rng.integers(1, 2 ** int(rng.integers(2, 60))))
        max_abs_q = int(rng.choice([1, 127, 255, 4000, 10 ** 6]))
        tp = q_b ** 2 if variant == 0 else q_b ** 4
        if tp >= 2 ** 61:
            continue
        k = 0
        while -(-(tp + 2 * -q_c) >> k) * max_abs_q >= 2 ** 31:     # ceiling: |v| can reach it
            k += 1
        if k > 62:
            continue
        k = min(62, k + int(rng.integers(0, 3)))
        post = ref.Dyadic(int(rng.integers(-32767, 32768)), int(rng.integers(0, 63)),
                          int(rng.integers(-300, 300)), -128, 127)
        pre = (1, 0) if rng.integers(0, 2) else (int(rng.integers(1, 32768)), int(rng.integers(0, 63)))
        p = ref.GeluParams(variant, q_b, q_c, k, int(rng.integers(-128, 129)), max_abs_q, pre[0], pre[1], post)
        n = int(rng.choice([7, 64, 1000, 4099]))
        x8 = rng.integers(-128, 128, size=n, dtype=np.int8)
        x32 = rng.integers(I32_MIN, I32_MAX + 1, size=n).astype(np.int32)
        x32[: n // 2] = np.rint(rng.standard_normal(n // 2) * max_abs_q).astype(np.int32)
        try:
            want8 = ref.gelu_i8(x8, p)
        except ref.OracleError:
            continue
        assert np.array_equal(gpu_gelu_i8(x8, p), want8), p
        assert np.array_equal(gpu_gelu_i8(x8, p, algo=1), want8), p
        assert np.array_equal(gpu_gelu_i32(x32, p), ref.gelu_i32(x32, p)), p
        done += 1
