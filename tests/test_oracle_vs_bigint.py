"""Differential check of the C oracle against the same equations in unbounded Python
integers (// and >> floor on any sign, no overflow possible), on random parameter sets that
stress the 64-bit intermediates: large i0, extreme scores, every requantization shift.
This is a cross-check of the C code's integer handling, not a pin of the method."""
import numpy as np
import pytest

from oracle import ref

I32_MIN, I32_MAX = -(2 ** 31), 2 ** 31 - 1


def rshr_round(v, s):
    return v if s == 0 else (v + (1 << (s - 1))) >> s


def requant(x, d):
    return min(max(rshr_round(x * d.m, d.s) + d.zp, d.qmin), d.qmax)


def sat32(v):
    return min(max(v, I32_MIN), I32_MAX)


def softmax_row(row, bias_row, p):
    x = []
    for j, v in enumerate(row):
        v = int(v)
        if bias_row is not None:
            b = int(bias_row[j])
            v = I32_MIN if (v == I32_MIN or b == I32_MIN) else sat32(v + b)
        if v != I32_MIN and not (p.pre_m == 1 and p.pre_s == 0):
            v = sat32(rshr_round(v * p.pre_m, p.pre_s))
        x.append(v)
    mx = max(x)
    qexp = []
    for v in x:
        if v == I32_MIN:
            qexp.append(0)
            continue
        d = max(v - mx, -(2 ** 30))
        qp = d + (d >> 1) - (d >> 4)
        q, r = divmod(-qp, p.i0)
        fr = ((-r) >> 1) if p.variant == 0 else ((-r) >> 1) + ((-r) >> 3) + ((-r) >> 4)
        if p.variant == 2:
            fr += (fr * fr) // (2 * p.i0)
        qexp.append(0 if q >= 32 else ((fr + p.i0) << p.n_shift) >> q)
    total = sum(qexp)
    f = (1 << p.m_bits) // total if total > 0 else 0
    return [requant((f * e) >> (p.m_bits - (p.out_bits - 1)), p.post) for e in qexp]


def gelu_value(v, p, with_pre):
    v = int(v)
    if with_pre and not (p.pre_m == 1 and p.pre_s == 0):
        v = sat32(rshr_round(v * p.pre_m, p.pre_s))
    q = min(max(v - p.zp_in, -p.max_abs_q), p.max_abs_q)
    sgn = (q > 0) - (q < 0)
    t = min(abs(q), -p.q_b) + p.q_b
    tp = t * t if p.variant == 0 else t ** 4
    vv = (sgn * (tp + p.q_c) + p.q_c) >> p.k
    return requant(q * vv, p.post)


@pytest.mark.parametrize("seed", range(6))
def test_softmax_random_parameters(seed):
    rng = np.random.default_rng(seed)
    for _ in range(60):
        cols = int(rng.integers(1, 40))
        rows = 5
        i0 = int(rng.choice([16, 17, 100, 181, 4095, 65535, 65536, 2 ** 20 + 3, 2 ** 24 - 1]))
        n_max = 0
        while ((i0 << (n_max + 1)) < 2 ** 24) and n_max < 20:
            n_max += 1
        n_shift = int(rng.integers(0, n_max + 1))
        out_bits = int(rng.integers(2, 9))
        m_bits = int(rng.integers(max(out_bits - 1, (cols * (i0 << n_shift)).bit_length()), 32))
        if cols * (i0 << n_shift) > (1 << m_bits):
            continue
        signed = int(rng.integers(0, 2))
        lo, hi = (-128, 127) if signed else (0, 255)
        post = ref.Dyadic(int(rng.integers(-32767, 32768)), int(rng.integers(0, 63)),
                          int(rng.integers(-200, 200)), lo, hi)
        if rng.integers(0, 3) == 0:
            post = ref.Dyadic(1, 0, 0, 0 if not signed else -128, hi)
        pre = (1, 0) if rng.integers(0, 2) else (int(rng.integers(1, 32768)), int(rng.integers(0, 63)))
        p = ref.SoftmaxParams(variant=int(rng.integers(0, 3 if i0 < 2 ** 16 else 2)), i0=i0, n_shift=n_shift, m_bits=m_bits,
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
        x[rng.random((rows, cols)) < 0.1] = I32_MIN
        bias, period = None, 0
        if rng.integers(0, 2):
            period = int(rng.integers(1, 4))
            bias = rng.integers(I32_MIN, I32_MAX + 1, size=(period, cols)).astype(np.int32)
            if rng.integers(0, 2):
                bias = (bias // 2 ** 20).astype(np.int32)
            bias[rng.random(bias.shape) < 0.15] = I32_MIN
        got = ref.softmax_i32(x, p, bias, period).astype(np.int64)
        for r in range(rows):
            want = softmax_row(x[r], None if bias is None else bias[r % period], p)
            assert got[r].tolist() == want, (p, x[r].tolist())


@pytest.mark.parametrize("seed", range(4))
def test_gelu_random_parameters(seed):
    rng = np.random.default_rng(100 + seed)
    done = 0
    while done < 80:
        variant = int(rng.integers(0, 2))
        q_b = -int(rng.integers(1, 2 ** 15 if variant else 2 ** 30))
        q_c = -int(rng.integers(1, 2 ** int(rng.integers(2, 60))))
        max_abs_q = int(rng.choice([1, 127, 255, 4000, 10 ** 6]))
        tp = q_b ** 2 if variant == 0 else q_b ** 4
        if tp >= 2 ** 61:
            continue
        k = 0
        while -(-(tp + 2 * -q_c) >> k) * max_abs_q >= 2 ** 31:     # ceiling: |v| can reach it
            k += 1
        k = min(62, k + int(rng.integers(0, 3)))
        post = ref.Dyadic(int(rng.integers(-32767, 32768)), int(rng.integers(0, 63)),
                          int(rng.integers(-300, 300)), -128, 127)
        pre = (1, 0) if rng.integers(0, 2) else (int(rng.integers(1, 32768)), int(rng.integers(0, 63)))
        p = ref.GeluParams(variant, q_b, q_c, k, int(rng.integers(-128, 129)), max_abs_q, pre[0], pre[1], post)
        x8 = rng.integers(-128, 128, size=64, dtype=np.int8)
        x32 = rng.integers(I32_MIN, I32_MAX + 1, size=64).astype(np.int32)
        x32[:8] = np.rint(rng.standard_normal(8) * max_abs_q).astype(np.int32)
        try:
            y8 = ref.gelu_i8(x8, p)
        except ref.OracleError:
            continue
        y32 = ref.gelu_i32(x32, p)
        assert y8.tolist() == [gelu_value(v, p, False) for v in x8], p
        assert y32.tolist() == [gelu_value(v, p, True) for v in x32], p
        done += 1
