"""The paper's two approximation-error tables, reproduced from the real-valued formulas.

They fix how the printed equations are read: Eq. 3 as sign(x) * [a (min(|x|, -b) + b)^4 + 1],
"L2 error" as the RMS error on a uniform grid over the stated open interval, the
second-order erf of Eq. 2 with the I-BERT coefficients, and the two fractional-part
approximations of 2^x (Eq. 10 and Eq. 12).
"""
import math

import numpy as np

A4, B4 = -0.019913, -2.698088       # Section 4.3, printed below Eq. 2
A2, B2 = -0.2888, -1.769            # second-order erf fit that Eq. 2 refers to

erf = np.vectorize(math.erf)


def l_poly(x, a, b, p):
    return np.sign(x) * (a * (np.minimum(np.abs(x), -b) + b) ** p + 1.0)


def errs(f, g, lo, hi, n=600001):
    x = np.linspace(lo, hi, n)[1:-1]
    d = f(x) - g(x)
    return float(np.sqrt(np.mean(d * d))), float(np.abs(d).max())


def gelu(x):
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def test_table_erf_and_gelu_errors():
    # Table "erf / GELU approximation error", range (-3, 3)
    l2, li = errs(lambda x: l_poly(x, A2, B2, 2), erf, -3, 3)
    assert round(l2, 4) == 0.0264 and round(li, 4) == 0.0962
    l2, li = errs(lambda x: l_poly(x, A4, B4, 4), erf, -3, 3)
    assert round(l2, 4) == 0.0098 and abs(li - 0.0550) < 3e-4
    l2, li = errs(lambda x: 0.5 * x * (1 + l_poly(x / math.sqrt(2), A2, B2, 2)), gelu, -3, 3)
    assert round(l2, 4) == 0.0094 and round(li, 4) == 0.0182
    l2, li = errs(lambda x: 0.5 * x * (1 + l_poly(x / math.sqrt(2), A4, B4, 4)), gelu, -3, 3)
    assert round(l2, 4) == 0.0051 and round(li, 4) == 0.0093


def test_table_base2_exp_errors():
    # Table "base-2 exponential approximation", range (-1, 1)
    two = lambda x: np.exp2(x)
    l2, li = errs(lambda x: 1 + x / 2, two, -1, 1)
    assert round(l2, 4) == 0.1717 and round(li, 3) == 0.5
    l2, li = errs(lambda x: 1 + math.log(2) * x, two, -1, 1)
    assert round(l2, 4) == 0.1126 and round(li, 4) == 0.3069
    # the shift-add constant of Eq. 13: (0.1011)b = 1/2 + 1/8 + 1/16
    assert 0.5 + 0.125 + 0.0625 == 0.6875 and abs(0.6875 - math.log(2)) < 0.006
    # the base change constant of Eq. 7: (1.0111)b = 1 + 1/2 - 1/16
    assert abs(1.4375 - math.log2(math.e)) < 0.0053
