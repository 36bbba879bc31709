"""TEST INFRASTRUCTURE - the oracle's own derivation of the integer constants.

Real-valued scales become integers once, before inference (Section 4.3: the
polynomial coefficients are pre-quantized constants; Eq. 14: floor(1/S)).
Written independently of the HIP library's host helpers; the tests compare the
two.  Floating point is IEEE double throughout and the operations are done in
the order stated in each docstring, so that an independent implementation that
follows the same statement gets the same integers.
"""

from __future__ import annotations

import math

from .ref import Dyadic, GeluParams, SoftmaxParams

# erf polynomial coefficients: degree 4 from Section 4.3 (text below Eq. 2);
# degree 2 is the I-BERT second-order fit that Eq. 2 refers to (its values are
# not printed in the paper; they reproduce the paper's error table).
POLY = {0: (2, -0.2888, -1.769), 1: (4, -0.019913, -2.698088)}


def make_dyadic(ratio: float):
    """(m, s) with ratio ~ m / 2^s, |m| < 2^15 and s the largest value <= 62.

    |ratio| = f * 2^e with f in [0.5, 1) (frexp); m = floor(f * 2^15 + 0.5),
    s = 15 - e; m == 2^15 is renormalised to (2^14, s - 1).  If s would exceed
    62, m = floor(|ratio| * 2^62 + 0.5) and s = 62.  Ratios >= 2^15 are refused.
    """
    a = abs(ratio)
    if not (a > 0.0) or math.isinf(a):
        raise ValueError("ratio must be finite and non-zero")
    f, e = math.frexp(a)
    m = int(math.floor(f * 32768.0 + 0.5))
    s = 15 - e
    if m == 32768:
        m, s = 16384, s - 1
    if s > 62:
        m, s = int(math.floor(math.ldexp(a, 62) + 0.5)), 62
    if s < 0:
        raise ValueError("ratio too large for a 15-bit multiplier")
    return (-m if ratio < 0 else m), s


def softmax_prepare(s_delta: float, cols: int, variant: int, out_is_signed: int = 0
                    ) -> SoftmaxParams:
    """i0 = floor(1 / s_delta) (Eq. 14); N = max(0, 15 - bitlen(i0)) lowered until
    cols * (i0 << N) <= 2^M; M = 30; b = 8; identity pre- and post-requantization
    (the int8 form saturates the code 128 to 127)."""
    i0 = int(math.floor(1.0 / s_delta))
    n = max(0, 15 - i0.bit_length())
    m_bits = 30
    while n > 0 and cols * (i0 << n) > (1 << m_bits):
        n -= 1
    post = Dyadic(1, 0, 0, 0, 127) if out_is_signed else Dyadic(1, 0, 0, 0, 255)
    return SoftmaxParams(variant=variant, i0=i0, n_shift=n, m_bits=m_bits, out_bits=8,
                         pre_m=1, pre_s=0, post=post, out_is_signed=out_is_signed)


def gelu_prepare(s_in: float, s_out: float, zp_in: int, zp_out: int, variant: int,
                 max_abs_q: int = 255) -> GeluParams:
    """S_e = s_in / sqrt(2); q_b = floor(b / S_e); S_L = a * S_e^p with the power
    formed as (S_e*S_e) or (S_e*S_e)*(S_e*S_e); q_c = floor(1 / S_L);
    k = smallest shift with ceil((|q_b|^p + 2|q_c|) / 2^k) * max_abs_q < 2^31 (the ceiling:
    a negative numerator is floored away from zero, so |v| can reach it);
    output ratio = ((s_in * S_L) * 2^k / 2) / s_out -> dyadic (negative m)."""
    p, a, b = POLY[variant]
    s_e = s_in / math.sqrt(2.0)
    q_b = int(math.floor(b / s_e))
    sq = s_e * s_e
    s_l = a * (sq if p == 2 else sq * sq)
    q_c = int(math.floor(1.0 / s_l))
    vmax = abs(q_b) ** p + 2 * abs(q_c)
    k = 0
    while -((-vmax) >> k) * max_abs_q >= (1 << 31):
        k += 1
    ratio = ((s_in * s_l) * math.ldexp(1.0, k) / 2.0) / s_out
    m, s = make_dyadic(ratio)
    return GeluParams(variant=variant, q_b=q_b, q_c=q_c, k=k, zp_in=zp_in, max_abs_q=max_abs_q,
                      pre_m=1, pre_s=0, post=Dyadic(m, s, zp_out, -128, 127))
