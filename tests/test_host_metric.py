"""The library's host-only Unified Metric (Section 4.5, Eq. 16-20) against the oracle's, on random
tensors and on the oracle's own pins; operation counts and selection as well.  No GPU needed."""
import math

import numpy as np
import pytest

import paper_2511_15369_amd as ip
from oracle import metric


def _same(a: ip.Metric, b: metric.Terms):
    assert a.q_db == pytest.approx(b.q_db, rel=1e-12, abs=1e-12)
    assert a.p == pytest.approx(b.p, rel=1e-12)
    assert a.c == pytest.approx(b.c, rel=1e-15)
    assert a.score == pytest.approx(b.score, rel=1e-12)


def test_worked_example_through_the_library():
    x = np.full(1000, 100.0)
    assert ip.unified_metric(x, x - 10.0, 1.0).q_db == pytest.approx(20.0, abs=1e-12)
    assert ip.unified_metric(x, x - math.sqrt(60.0), 1.0).q_db == pytest.approx(22.2185, abs=1e-4)


@pytest.mark.parametrize("mode", [ip.METRIC_LITERAL, ip.METRIC_PER_ELEMENT])
def test_random_tensors_match_the_oracle(mode):
    rng = np.random.default_rng(mode)
    name = "literal" if mode == ip.METRIC_LITERAL else "per_element"
    for _ in range(30):
        n = int(rng.integers(1, 20000))
        x = rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 3)
        xh = x + rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 1)
        ops = float(rng.integers(1, 40)) * n
        _same(ip.unified_metric(x, xh, ops, mode), metric.unified_metric(x, xh, ops, name))
    x = rng.standard_normal(100)
    m = ip.unified_metric(x, x.copy(), 5.0, mode)
    assert m.q_db == math.inf and m.p == 0.0
    _same(m, metric.unified_metric(x, x.copy(), 5.0, name))


def test_softplus_terms_are_reported():
    x = np.full(4, 2.0)
    m = ip.unified_metric(x, x - 0.2, 12.0, ip.METRIC_PER_ELEMENT)
    assert m.n_q == pytest.approx(metric.softplus(20.0)) and m.n_p == pytest.approx(metric.softplus(0.04))
    assert m.n_c == pytest.approx(metric.softplus(3.0))
    assert m.score == pytest.approx(3.0 / (1.0 / m.n_q + m.n_p + m.n_c), rel=1e-15)
    assert m.score == pytest.approx(0.7871, abs=2e-4)          # the oracle's hand-built case


def test_selection_and_operation_counts():
    x = np.full(4, 2.0)
    a = ip.unified_metric(x, x - 0.2, 12.0, ip.METRIC_PER_ELEMENT)
    b = ip.unified_metric(x, x - 0.02, 16.0, ip.METRIC_PER_ELEMENT)
    b2 = ip.unified_metric(x, x - 0.02, 12.0, ip.METRIC_PER_ELEMENT)
    assert ip.unified_select([a, b]) == 0 and ip.unified_select([b, a]) == 1
    assert ip.unified_select([a, a]) == 0 and ip.unified_select([a, b2]) == 1
    for v in (0, 1, 2):
        for rows, cols in ((1, 1), (10, 49), (302592, 197)):
            assert ip.softmax_op_count(v, rows, cols) == metric.softmax_op_count(v, rows, cols)
    for v in (0, 1):
        assert ip.gelu_op_count(v, 12345) == metric.gelu_op_count(v, 12345)
    assert ip.softmax_op_count(3, 1, 1) == -1 and ip.gelu_op_count(2, 1) == -1


def test_argument_checks():
    import ctypes
    lib = ip.load()
    x = np.zeros(4)
    out = ip.Metric()
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert lib.iptq_unified_metric(None, vp(x), 4, 1.0, 0, ctypes.byref(out)) == -1
    assert lib.iptq_unified_metric(vp(x), vp(x), 0, 1.0, 0, ctypes.byref(out)) == -2
    assert lib.iptq_unified_metric(vp(x), vp(x), 4, 1.0, 7, ctypes.byref(out)) == -3
    assert lib.iptq_unified_metric(vp(x), vp(x), 4, -1.0, 0, ctypes.byref(out)) == -3
    best = ctypes.c_int32()
    assert lib.iptq_unified_select(None, 1, ctypes.byref(best)) == -1
    assert lib.iptq_unified_select(ctypes.byref(out), 0, ctypes.byref(best)) == -2
