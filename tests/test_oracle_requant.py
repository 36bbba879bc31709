"""Pins for the oracle's dyadic requantization: exact rationals, hand values, bounds."""
from fractions import Fraction
import math

import numpy as np
import pytest

from oracle import prepare, ref


def exact_requant(x, m, s, zp, qmin, qmax):
    y = math.floor(Fraction(x * m, 2 ** s) + Fraction(1, 2)) + zp
    return min(max(y, qmin), qmax)


def test_hand_values_ties_go_up():
    # (x, m, s) -> round-half-up of x*m/2^s, worked by hand: 2.5 -> 3, -2.5 -> -2,
    # -0.5 -> 0, -1.5 -> -1, 21/4 -> 5, -21/4 -> -5
    cases = [((5, 1, 1), 3), ((-5, 1, 1), -2), ((-1, 1, 1), 0), ((-3, 1, 1), -1),
             ((7, 3, 2), 5), ((-7, 3, 2), -5)]
    for (x, m, s), want in cases:
        got = ref.requant(np.array([x], np.int32), ref.Dyadic(m, s, 0, -128, 127), 1)
        assert int(got[0]) == want


def test_identity_and_clip():
    x = np.arange(-300, 300, dtype=np.int32)
    got = ref.requant(x, ref.Dyadic(1, 0, 0, -128, 127), 1)
    assert np.array_equal(got, np.clip(x, -128, 127).astype(np.int8))
    got = ref.requant(x, ref.Dyadic(1, 0, 0, 0, 255), 0)
    assert np.array_equal(got, np.clip(x, 0, 255).astype(np.uint8))


@pytest.mark.parametrize("seed", range(4))
def test_matches_exact_rational(seed):
    rng = np.random.default_rng(seed)
    for _ in range(40):
        m = int(rng.integers(-32767, 32768))
        s = int(rng.integers(0, 63))
        zp = int(rng.integers(-128, 128))
        signed = int(rng.integers(0, 2))
        lo, hi = (-128, 127) if signed else (0, 255)
        x = rng.integers(-2 ** 31, 2 ** 31, size=64).astype(np.int32)
        x[:4] = [-2 ** 31, 2 ** 31 - 1, 0, -1]
        d = ref.Dyadic(m, s, zp, lo, hi)
        got = ref.requant(x, d, signed)
        want = [exact_requant(int(v), m, s, zp, lo, hi) for v in x]
        assert got.tolist() == want


def test_error_bound_and_monotone():
    # y tracks x*ratio to within 1/2 (rounding) + |x| * 2^-15 * ratio (15-bit multiplier)
    ratio = 0.0123456
    m, s = prepare.make_dyadic(ratio)
    assert 2 ** 14 <= m < 2 ** 15
    x = np.arange(-9000, 9000, dtype=np.int32)
    y = ref.requant(x, ref.Dyadic(m, s, 0, -128, 127), 1).astype(np.int64)
    assert np.all(np.diff(y) >= 0)
    err = np.abs(y - x * ratio)
    assert np.all(err <= 0.5 + np.abs(x) * ratio * 2.0 ** -15 + 1e-9)


def test_make_dyadic_powers_of_two_exact():
    assert prepare.make_dyadic(2.0 ** -6) == (16384, 20)
    assert prepare.make_dyadic(1.0) == (16384, 14)
    assert prepare.make_dyadic(-0.5) == (-16384, 15)
    m, s = prepare.make_dyadic(3.0)
    assert m / 2 ** s == 3.0
    with pytest.raises(ValueError):
        prepare.make_dyadic(40000.0)
    with pytest.raises(ValueError):
        prepare.make_dyadic(0.0)


def test_rejects_bad_params():
    x = np.zeros(4, np.int32)
    for d in (ref.Dyadic(32768, 0, 0, 0, 255), ref.Dyadic(1, 63, 0, 0, 255),
              ref.Dyadic(1, -1, 0, 0, 255), ref.Dyadic(1, 0, 0, 5, 4), ref.Dyadic(1, 0, 0, -1, 255)):
        with pytest.raises(ref.OracleError):
            ref.requant(x, d, 0)
