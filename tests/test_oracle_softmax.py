"""Pins for the oracle's integer softmax (Section 4.4, Eq. 6-15).

What fixes the oracle here is not the oracle: hand-worked rows (tests/golden),
closed forms, the real-valued statement of Eq. 7-14, exact rational brackets
around IntDiv (Eq. 15), and the invariances that Eq. 6 implies.
"""
from fractions import Fraction
import math
import os

import numpy as np
import pytest

from oracle import prepare, ref

INT32_MIN = -(2 ** 31)
PARAM_SETS = [(16, 0), (64, 8), (128, 7), (181, 7), (1000, 5), (23, 0), (5000, 2)]


def params(variant, i0, n, **kw):
    return ref.SoftmaxParams(variant=variant, i0=i0, n_shift=n, **kw)


def _golden_rows(golden_dir):
    out = []
    with open(os.path.join(golden_dir, "softmax_rows.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, row, want = [part.split() for part in line.split("|")]
            out.append((int(head[0]), int(head[1]), int(head[2]),
                        [int(v) for v in row], [int(v) for v in want]))
    return out


def test_hand_worked_rows(golden_dir):
    rows = _golden_rows(golden_dir)
    assert len(rows) >= 8
    for variant, i0, n, row, want in rows:
        got = ref.softmax_i32(np.array([row], np.int32), params(variant, i0, n))
        assert got[0].tolist() == want, (variant, i0, n, row)


# ----------------------------------------------------------------- the exponential
def real_bit_exp(delta, i0, variant):
    """Eq. 7-14 over the reals: base change by (1.0111)b, split into integer and
    fractional parts, linear fractional part; no floors anywhere."""
    y = 1.4375 * (-delta) / i0
    q = math.floor(y)
    x = y - q
    c = 0.5 if variant == 0 else 0.6875
    return 2.0 ** (-q) * (1.0 - c * x)


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("i0,n", PARAM_SETS)
def test_bit_exp_tracks_real_valued_equations(variant, i0, n):
    p = params(variant, i0, n)
    one = i0 << n
    assert ref.bit_exp(0, p) == one                      # delta 0: 2^0 = 1 exactly
    # floors perturb Qp by < 1 and base by < 2.4 (three floors) and the result by < 1
    tol = (1.4375 + 2.4) / i0 + 1.0 / one
    for delta in range(0, -40 * i0, -max(1, i0 // 37)):
        got = ref.bit_exp(delta, p) / one
        # variant 1 jumps at segment ends: compare against the nearer side
        cands = [real_bit_exp(delta + e, i0, variant) for e in (-1.0, 0.0, 1.0)]
        assert min(abs(got - c) for c in cands) <= tol, (delta, got, cands)


@pytest.mark.parametrize("variant,bound", [(0, 0.0431), (1, 0.1875)])
def test_bit_exp_close_to_exp(variant, bound):
    # worst case of 1 - c x against 2^-x on [0, 1) is `bound`; the (1.0111)b base
    # change adds < 0.0014 (max of 0.0036 z e^-z); floors add < 4 / i0
    i0, n = 4096, 3
    p = params(variant, i0, n)
    worst = 0.0
    for delta in range(0, -12 * i0, -7):
        got = ref.bit_exp(delta, p) / (i0 << n)
        worst = max(worst, abs(got - math.exp(delta / i0)))
    assert worst <= bound + 0.0014 + 4.0 / i0
    assert worst >= bound * 0.8        # and the bound is attained, not vacuous


def test_bit_exp_closed_form_on_multiples_of_16():
    # delta = -16 a makes Eq. 7 exact (Qp = -23 a); with i0 = 23: q = a, r = 0
    for variant in (0, 1):
        for n in (0, 5, 10):
            p = params(variant, 23, n)
            for a in range(0, 40):
                want = ((23 << n) >> a) if a < 32 else 0
                assert ref.bit_exp(-16 * a, p) == want


@pytest.mark.parametrize("i0,n", PARAM_SETS)
def test_variant0_monotone_and_variant1_segmentwise(i0, n):
    p0, p1 = params(0, i0, n), params(1, i0, n)
    prev = None
    for delta in range(0, -34 * i0, -1):
        v = ref.bit_exp(delta, p0)
        assert v >= 0
        if prev is not None:
            assert v <= prev
        prev = v
    # variant 1 is non-increasing inside a segment (fixed q) and segment heads halve
    for q in range(0, 6):
        head = ref.bit_exp(-math.ceil(q * i0 / 1.4375) - 2, p1)
        assert abs(head - ((i0 << n) >> q)) <= (4 << n >> q) + 1


def test_far_tail_is_zero_and_delta_clamp():
    p = params(1, 16, 0)
    assert ref.bit_exp(-400, p) == 0          # q = 35 >= 32
    assert ref.bit_exp(-(2 ** 30), p) == 0
    row = np.array([[2 ** 31 - 1, -(2 ** 31) + 1, 0]], np.int32)
    got = ref.softmax_i32(row, p)
    assert got[0].tolist() == [128, 0, 0]


# ----------------------------------------------------------------- IntDiv (Eq. 15)
@pytest.mark.parametrize("variant", [0, 1])
def test_intdiv_brackets_exact(variant):
    rng = np.random.default_rng(11 + variant)
    for trial in range(60):
        i0, n = PARAM_SETS[trial % len(PARAM_SETS)]
        cols = int(rng.integers(1, 70))
        spread = float(rng.choice([0.3, 1.0, 3.0, 10.0])) * i0
        row = np.rint(rng.standard_normal(cols) * spread).astype(np.int32)
        p = params(variant, i0, n)
        got = ref.softmax_i32(row[None, :], p)[0].astype(np.int64)
        mx = int(row.max())
        qexp = [ref.bit_exp(int(v) - mx, p) for v in row]
        sigma = sum(qexp)
        assert sigma >= (i0 << n)
        unit = 2 ** (30 - 7)
        for pj, qe in zip(got.tolist(), qexp):
            ideal = Fraction(128 * qe, sigma)
            assert ideal - 1 - Fraction(qe, unit) < pj <= ideal
        assert 128 - cols - math.ceil(Fraction(sigma, unit)) < int(got.sum()) <= 128


def test_invariance_to_row_shift_and_permutation():
    rng = np.random.default_rng(5)
    for variant in (0, 1):
        p = params(variant, 181, 7)
        rows = np.rint(rng.standard_normal((20, 33)) * 400).astype(np.int32)
        base = ref.softmax_i32(rows, p)
        for c in (1, -977, 2 ** 30, -(2 ** 30)):
            assert np.array_equal(ref.softmax_i32(rows + np.int32(c), p), base)
        perm = rng.permutation(33)
        assert np.array_equal(ref.softmax_i32(rows[:, perm], p), base[:, perm])


def test_monotone_in_the_input_for_variant0():
    # larger score -> not smaller probability, within a row
    rng = np.random.default_rng(6)
    p = params(0, 128, 7)
    rows = np.rint(rng.standard_normal((50, 49)) * 300).astype(np.int32)
    out = ref.softmax_i32(rows, p).astype(np.int64)
    for r, o in zip(rows, out):
        order = np.argsort(r, kind="stable")
        assert np.all(np.diff(o[order]) >= 0)


@pytest.mark.parametrize("variant,tol", [(0, 0.03), (1, 0.06)])
def test_close_to_float_softmax(variant, tol):
    rng = np.random.default_rng(7)
    s_delta = 1.0 / 181.3
    p = prepare.softmax_prepare(s_delta, 49, variant)
    assert (p.i0, p.n_shift) == (181, 7)
    rows = np.rint(rng.standard_normal((200, 49)) * 2.0 / s_delta).astype(np.int32)
    got = ref.softmax_i32(rows, p).astype(np.float64) / 128.0
    z = rows * s_delta
    e = np.exp(z - z.max(axis=1, keepdims=True))
    want = e / e.sum(axis=1, keepdims=True)
    assert np.abs(got - want).max() <= tol


def test_flat_long_row_is_all_zero():
    # 197 equal scores: 128 / 197 < 1 floors to 0 everywhere - the defined result of Eq. 15
    p = params(1, 128, 7)
    got = ref.softmax_i32(np.full((1, 197), 42, np.int32), p)
    assert not got.any()


# ----------------------------------------------------------------- mask, bias, requant
def test_mask_semantics():
    p = params(1, 16, 0)
    row = np.array([[3, INT32_MIN, -2, INT32_MIN, 3]], np.int32)
    got = ref.softmax_i32(row, p)[0]
    ref_row = ref.softmax_i32(np.array([[3, -2, 3]], np.int32), p)[0]
    assert got.tolist() == [ref_row[0], 0, ref_row[1], 0, ref_row[2]]
    # a fully masked row gives the requantized zero
    allm = np.full((1, 7), INT32_MIN, np.int32)
    assert not ref.softmax_i32(allm, p).any()
    p2 = params(1, 16, 0, post=ref.Dyadic(1, 0, 9, 0, 255))
    assert ref.softmax_i32(allm, p2)[0].tolist() == [9] * 7
    # a row whose only live entry sits next to INT32_MIN still treats the sentinel as masked
    near = np.array([[INT32_MIN + 1, INT32_MIN, INT32_MIN + 1]], np.int32)
    assert ref.softmax_i32(near, p)[0].tolist() == [64, 0, 64]


def test_bias_is_added_before_the_max_and_wraps_by_period():
    rng = np.random.default_rng(8)
    p = params(0, 64, 8)
    rows = np.rint(rng.standard_normal((12, 9)) * 150).astype(np.int32)
    bias = np.rint(rng.standard_normal((4, 9)) * 100).astype(np.int32)
    got = ref.softmax_i32(rows, p, bias=bias, bias_period_rows=4)
    want = ref.softmax_i32(rows + np.tile(bias, (3, 1)), p)
    assert np.array_equal(got, want)
    # masked entries ignore the bias; the sum saturates instead of wrapping
    rows2 = np.array([[INT32_MIN, 5, 2 ** 31 - 1]], np.int32)
    bias2 = np.array([[1000, 0, 1000]], np.int32)
    got2 = ref.softmax_i32(rows2, p, bias=bias2, bias_period_rows=1)
    # 64 << 8 = 2^14 is a power of two, so the lone survivor gets exactly 2^(b-1)
    assert got2[0].tolist() == [0, 0, 128]


def test_pre_requant_happens_before_the_max():
    rng = np.random.default_rng(9)
    p = params(1, 128, 7, pre_m=20000, pre_s=18)
    rows = np.rint(rng.standard_normal((8, 21)) * 9000).astype(np.int32)
    got = ref.softmax_i32(rows, p)
    pre = np.array([[math.floor(Fraction(int(v) * 20000, 2 ** 18) + Fraction(1, 2)) for v in r]
                    for r in rows], np.int32)
    want = ref.softmax_i32(pre, params(1, 128, 7))
    assert np.array_equal(got, want)


def test_signed_output_saturates_128_and_post_requant():
    p = params(0, 16, 0, post=ref.Dyadic(1, 0, 0, 0, 127), out_is_signed=1)
    got = ref.softmax_i32(np.array([[9, -9000]], np.int32), p)
    assert got.dtype == np.int8 and got[0].tolist() == [127, 0]
    # post requantization: multiply by 3/2 (m=3, s=1), add 10, clip
    p = params(0, 16, 0, post=ref.Dyadic(3, 1, 10, 0, 255))
    got = ref.softmax_i32(np.array([[3, -2, -17, -34, -97, 3]], np.int32), p)
    assert got[0].tolist() == [70, 55, 28, 13, 10, 70]   # from 40 30 12 2 0 40


def test_out_bits():
    for b in (2, 4, 6, 8):
        p = params(0, 16, 0, out_bits=b)
        got = ref.softmax_i32(np.array([[5, 5], [9, -900]], np.int32), p)
        assert got.tolist() == [[2 ** (b - 2)] * 2, [2 ** (b - 1), 0]]


def test_rejects_bad_params():
    row = np.zeros((1, 4), np.int32)
    bad = [params(3, 16, 0), params(0, 15, 0), params(0, 2 ** 24, 0), params(0, 2 ** 20, 4),
           params(0, 16, 0, out_bits=9), params(0, 16, 0, m_bits=32),
           params(0, 2 ** 15, 8, m_bits=24), params(0, 16, 0, pre_m=0),
           params(0, 16, 0, post=ref.Dyadic(1, 0, 0, -1, 255))]
    for p in bad:
        with pytest.raises(ref.OracleError):
            ref.softmax_i32(row, p)


# ----------------------------------------------------------------- brute force cross-check
def brute_softmax_row(row, variant, i0, n, m_bits=30, b=8):
    """Eq. 6-15 with Python integers (// and >> floor on any sign)."""
    live = [v for v in row if v != INT32_MIN]
    if not live:
        return [0] * len(row)
    mx = max(live)
    qexp = []
    for v in row:
        if v == INT32_MIN:
            qexp.append(0)
            continue
        d = max(v - mx, -(2 ** 30))
        qp = d + (d >> 1) - (d >> 4)
        q, r = divmod(-qp, i0)
        frac = ((-r) >> 1) if variant == 0 else ((-r) >> 1) + ((-r) >> 3) + ((-r) >> 4)
        qexp.append(((frac + i0) << n) >> q)
    f = (1 << m_bits) // sum(qexp)
    return [min((f * e) >> (m_bits - b + 1), 255) for e in qexp]


def test_all_short_rows_over_a_small_value_range():
    vals = [0, -1, -5, -16, -17, -100, -700]
    for variant in (0, 1):
        for i0, n in ((16, 0), (29, 3)):
            p = params(variant, i0, n)
            rows = np.array([[a, b, c] for a in vals for b in vals for c in vals], np.int32)
            got = ref.softmax_i32(rows, p)
            for r, g in zip(rows.tolist(), got.tolist()):
                assert g == brute_softmax_row(r, variant, i0, n)


# ----------------------------------------------------------------- second-degree form (variant 2)
def real_bit_exp_d2(delta, i0):
    """Eq. 11 with D = 2 over the reals, on top of the base change and the split of Eq. 7-9:
    2^-x ~ 1 - c x + (c x)^2 / 2 with c = (0.1011)b."""
    y = 1.4375 * (-delta) / i0
    q = math.floor(y)
    x = y - q
    return 2.0 ** (-q) * (1.0 - 0.6875 * x + (0.6875 * x) ** 2 / 2.0)


@pytest.mark.parametrize("i0,n", PARAM_SETS)
def test_second_degree_tracks_real_valued_series(i0, n):
    p = params(2, i0, n)
    one = i0 << n
    assert ref.bit_exp(0, p) == one
    # floors: Qp < 1, Phi three floors < 2.4, the squared term moves by < 0.6875 * 2.4 / ... < 2, its
    # own floor < 1, the final shift < 1
    tol = (1.4375 + 2.4 + 2.0 + 1.0) / i0 + 1.0 / one
    for delta in range(0, -40 * i0, -max(1, i0 // 37)):
        got = ref.bit_exp(delta, p) / one
        cands = [real_bit_exp_d2(delta + e, i0) for e in (-1.0, 0.0, 1.0)]
        assert min(abs(got - c) for c in cands) <= tol, (delta, got, cands)


def test_second_degree_error_against_exp_is_its_analytic_worst_case():
    # on x in [0, 1): 1 - c x + (c x)^2 / 2 - 2^-x with c = 0.6875 peaks at x -> 1:
    # 1 - 0.6875 + 0.236328 - 0.5 = 0.048828 (the exact-ln2 series gives 0.0471 there);
    # the first-degree form has 0.1875 at the same point
    worst_real = max(abs(1 - 0.6875 * x + (0.6875 * x) ** 2 / 2 - 2.0 ** (-x))
                     for x in np.linspace(0.0, 1.0, 20001)[:-1])
    assert abs(worst_real - 0.048828) < 2e-4
    i0, n = 4096, 3
    p2, p1 = params(2, i0, n), params(1, i0, n)
    worst2 = worst1 = 0.0
    for delta in range(0, -12 * i0, -7):
        t = math.exp(delta / i0)
        worst2 = max(worst2, abs(ref.bit_exp(delta, p2) / (i0 << n) - t))
        worst1 = max(worst1, abs(ref.bit_exp(delta, p1) / (i0 << n) - t))
    assert worst2 <= 0.048828 + 0.0014 + 6.0 / i0
    assert worst2 >= 0.048828 * 0.8
    assert worst2 < worst1 / 3


def test_second_degree_term_is_the_floored_square():
    # the only difference from variant 1 is + floor(Phi^2 / (2 i0)) before the shifts
    for i0, n in PARAM_SETS:
        p1, p2 = params(1, i0, 0), params(2, i0, 0)
        for r in range(0, i0, max(1, i0 // 50)):
            # find a delta whose split has q = 0 and this r: n = r means Qp = -r; scan near
            delta = -math.ceil(r / 1.4375)
            for d in (delta - 1, delta, delta + 1):
                if d > 0:
                    continue
                nn = -(d + (d >> 1) - (d >> 4))
                if nn >= i0:
                    continue
                phi = ((-nn) >> 1) + ((-nn) >> 3) + ((-nn) >> 4)
                assert ref.bit_exp(d, p1) == i0 + phi
                assert ref.bit_exp(d, p2) == i0 + phi + (phi * phi) // (2 * i0)


def test_second_degree_domain():
    with pytest.raises(ref.OracleError):
        ref.softmax_i32(np.zeros((1, 4), np.int32), params(2, 1 << 16, 0))
    ref.softmax_i32(np.zeros((1, 4), np.int32), params(2, (1 << 16) - 1, 0))


# ----------------------------------------------------------------- additive tables and minus infinity
def test_table_entry_int32_min_masks_whatever_the_score():
    p = params(1, 16, 0)
    # hand-worked: keys 0 and 2 live with equal scores -> 64 each (row C of the golden file);
    # key 1 is masked by the table although its score is positive and the largest
    scores = np.array([[5, 1000, 5]], np.int32)
    bias = np.array([[0, INT32_MIN, 0]], np.int32)
    assert ref.softmax_i32(scores, p, bias, 1)[0].tolist() == [64, 0, 64]
    # every key masked by the table, scores positive: the all-masked row, i.e. the zero-point
    bias = np.full((1, 3), INT32_MIN, np.int32)
    pz = params(1, 16, 0, post=ref.Dyadic(1, 0, 3, 0, 255))
    assert ref.softmax_i32(np.array([[7, 1, 9]], np.int32), pz, bias, 1)[0].tolist() == [3, 3, 3]
    # any other table value is an ordinary saturating addend: INT32_MIN + 1 leaves the key live
    bias = np.array([[INT32_MIN + 1, INT32_MIN + 1, INT32_MIN + 1]], np.int32)
    assert ref.softmax_i32(np.array([[7, 7, 7]], np.int32), p, bias, 1)[0].tolist() == [42, 42, 42]


def test_saturated_pre_requantized_scores():
    # hand-worked: 4 * (2^31 - 1) and 4 * 2^30 both exceed int32 and saturate at 2^31 - 1, so the
    # two keys tie: 64, 64 (row C).  Without the saturation the second would be 2^32 below the
    # first and get 0.
    p = params(1, 16, 0, pre_m=4, pre_s=0)
    row = np.array([[2 ** 31 - 1, 2 ** 30]], np.int32)
    assert ref.softmax_i32(row, p)[0].tolist() == [64, 64]
    # one step below the saturation point the order is kept: 4 * (2^29 - 8) = 2^31 - 32, delta -31:
    # Qp = -31 - 16 + 2 = -45, q = 2, r = 13, Phi(-13) = -7 - 2 - 1 = -10, base 6, Qexp = 6 >> 2 = 1
    # sum 17, f = floor(2^30 / 17) = 63161283, p = (16 f) >> 23 = 120, (1 f) >> 23 = 7
    row = np.array([[2 ** 30, 2 ** 29 - 8]], np.int32)
    assert ref.softmax_i32(row, p)[0].tolist() == [120, 7]
