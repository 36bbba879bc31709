"""Pins for the oracle's Unified Metric (Section 4.5, Eq. 16-20): the worked SQNR example the
section prints, Softplus identities, the harmonic form on equal terms, monotonicity in each
factor and a hand-built two-candidate selection."""
import math

import numpy as np
import pytest

from oracle import metric


def test_worked_sqnr_example_of_section_4_5():
    # signal power 10^4; error powers 100 and 60 -> 20 dB and 22.21 dB
    x = np.full(1000, 100.0)
    assert metric.sqnr_db(x, x - 10.0) == pytest.approx(20.0, abs=1e-12)
    got = metric.sqnr_db(x, x - math.sqrt(60.0))
    assert got == pytest.approx(22.2185, abs=1e-4)
    assert int(got * 100) / 100 == 22.21                       # as printed (truncated)
    # the literal "20 log" of the power ratio would have given 40 dB and 44.4 dB
    assert 20.0 * math.log10(1e4 / 100.0) == pytest.approx(40.0)


def test_sqnr_is_scale_free_and_perturbation_is_not():
    rng = np.random.default_rng(0)
    x = rng.standard_normal(5000)
    xh = x + 0.01 * rng.standard_normal(5000)
    assert metric.sqnr_db(7.0 * x, 7.0 * xh) == pytest.approx(metric.sqnr_db(x, xh), rel=1e-12)
    assert metric.perturbation(7.0 * x, 7.0 * xh) == pytest.approx(49.0 * metric.perturbation(x, xh), rel=1e-12)
    # ||.||_2^2 is the sum of squares, by hand: errors 1, -2, 2 -> 9
    assert metric.perturbation(np.array([1.0, 2.0, 3.0]), np.array([0.0, 4.0, 1.0])) == 9.0
    assert metric.sqnr_db(x, x) == math.inf


def test_softplus_identities():
    assert metric.softplus(0.0) == pytest.approx(math.log(2.0), abs=1e-15)
    for x in (-30.0, -2.5, -1e-9, 0.3, 4.0, 35.0, 700.0):
        assert metric.softplus(x) - metric.softplus(-x) == pytest.approx(x, rel=1e-12, abs=1e-12)
        if abs(x) < 30:
            assert metric.softplus(x) == pytest.approx(math.log(1.0 + math.exp(x)), rel=1e-13)
    assert metric.softplus(1e6) == 1e6                         # no overflow, asymptote x
    assert metric.softplus(-1e6) == 0.0
    assert 0.0 < metric.softplus(-40.0) < 1e-17


def test_harmonic_form_on_equal_terms():
    # 1 / N(Q) = N(P) = N(C) = t  ->  3 / (3 t) = 1 / t.  Build it: P = C, Q from N(Q) = 1 / N(P)
    p = 0.8
    t = metric.softplus(p)
    q = math.log(math.expm1(1.0 / t))                          # softplus^-1(1 / t)
    n = 4000
    rng = np.random.default_rng(3)
    x = rng.standard_normal(n)
    x *= math.sqrt(n * 1.0 / np.sum(x * x))                    # mean square exactly 1
    e = rng.standard_normal(n)
    e *= math.sqrt(p / np.sum(e * e))                          # ||e||^2 = p
    # choose the signal scale so that the SQNR is q: 10 log10(s^2 / (p / n)) = q
    s = math.sqrt((p / n) * 10.0 ** (q / 10.0))
    terms = metric.unified_metric(s * x, s * x - e, op_count=p)
    assert terms.p == pytest.approx(p, rel=1e-12)
    assert terms.q_db == pytest.approx(q, abs=1e-9)
    assert terms.score == pytest.approx(1.0 / t, rel=1e-9)


def test_monotone_in_each_factor():
    rng = np.random.default_rng(4)
    x = rng.standard_normal(2000)
    e = rng.standard_normal(2000)
    base = metric.unified_metric(x, x - 0.05 * e, 20.0 * 2000, "per_element")
    worse_err = metric.unified_metric(x, x - 0.10 * e, 20.0 * 2000, "per_element")
    dearer = metric.unified_metric(x, x - 0.05 * e, 25.0 * 2000, "per_element")
    assert worse_err.q_db < base.q_db and worse_err.p > base.p and worse_err.score < base.score
    assert dearer.score < base.score and dearer.q_db == base.q_db
    assert base.c == 20.0 and base.p == pytest.approx(np.sum((0.05 * e) ** 2) / 2000)


def test_hand_built_selection_and_omega():
    # two candidates on a 4-element layer, per-element mode, numbers small enough to do by hand:
    # x = [2, 2, 2, 2] (power 4).  A: error 0.2 everywhere (power 0.04, Q = 20 dB), 3 ops/element.
    # B: error 0.02 everywhere (power 0.0004, Q = 40 dB), 4 ops/element.
    x = np.full(4, 2.0)
    a = metric.unified_metric(x, x - 0.2, 12.0, "per_element")
    b = metric.unified_metric(x, x - 0.02, 16.0, "per_element")
    assert a.q_db == pytest.approx(20.0) and b.q_db == pytest.approx(40.0)
    sp = lambda v: math.log(1.0 + math.exp(v))
    want_a = 3.0 / (1.0 / sp(20.0) + sp(0.04) + sp(3.0))
    want_b = 3.0 / (1.0 / sp(40.0) + sp(0.0004) + sp(4.0))
    assert a.score == pytest.approx(want_a, rel=1e-12) and b.score == pytest.approx(want_b, rel=1e-12)
    # A: 3 / (0.05 + 0.7133 + 3.0486) = 0.7871 ; B: 3 / (0.025 + 0.6933 + 4.0181) = 0.6334 -> A
    assert a.score == pytest.approx(0.7871, abs=2e-4) and b.score == pytest.approx(0.6334, abs=2e-4)
    assert metric.select([a, b]) == 0 and metric.select([b, a]) == 1
    assert metric.select([a, a]) == 0                          # first among equals
    # with the cost equal, the more accurate candidate wins
    b2 = metric.unified_metric(x, x - 0.02, 12.0, "per_element")
    assert metric.select([a, b2]) == 1
    assert metric.omega([a.score, b2.score]) == pytest.approx(a.score + b2.score)


def test_literal_mode_is_dominated_by_cost():
    # the observation recorded as a reading: with whole-layer P and C the cheapest candidate wins
    rng = np.random.default_rng(5)
    x = rng.standard_normal(100000)
    good = metric.unified_metric(x, x + 1e-3 * rng.standard_normal(x.size), 22.0 * x.size)
    cheap = metric.unified_metric(x, x + 1e-1 * rng.standard_normal(x.size), 18.0 * x.size)
    assert metric.select([good, cheap]) == 1
    assert good.score == pytest.approx(3.0 / (good.c + good.p), rel=1e-6)


def test_operation_counts():
    assert metric.softmax_op_count(0, 10, 49) == 10 * 49 * 18 + 10
    assert metric.softmax_op_count(1, 10, 49) == 10 * 49 * 22 + 10
    assert metric.softmax_op_count(2, 1, 1) == 26
    assert metric.gelu_op_count(0, 100) == 1700 and metric.gelu_op_count(1, 100) == 1800
