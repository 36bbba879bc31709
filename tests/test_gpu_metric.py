"""The Unified Metric (Section 4.5) closed over the HIP path: synthetic real-valued attention
scores and MLP activations per layer, every candidate variant run through the kernels and
through the oracle, the library's metric on the kernels' dequantized outputs against the
oracle's metric on the oracle's: identical terms, identical choice per layer, identical Omega."""
import numpy as np
import pytest
from scipy.special import erf

import paper_2511_15369_amd as ip
from oracle import metric, prepare, ref
from tests.helpers import gpu_gelu_i8, gpu_softmax

pytestmark = pytest.mark.gpu


def _softmax_layer(rng, rows, cols, s_delta):
    z = rng.standard_normal((rows, cols)) * rng.uniform(0.5, 3.0)          # real-valued scores
    scores = np.rint(z / s_delta).astype(np.int32)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return scores, e / e.sum(axis=1, keepdims=True)                        # the real-valued layer output


@pytest.mark.parametrize("mode", ["literal", "per_element"])
def test_assignment_over_layers(mode):
    rng = np.random.default_rng(17)
    lib_mode = ip.METRIC_LITERAL if mode == "literal" else ip.METRIC_PER_ELEMENT
    omega_lib = omega_ref = 0.0
    picks = []
    for layer in range(6):
        cols = (197, 49)[layer % 2]
        rows = 300 + 17 * layer
        s_delta = 2.0 ** rng.uniform(-9, -4)
        scores, x = _softmax_layer(rng, rows, cols, s_delta)
        lib_c, ref_c = [], []
        for variant in (0, 1, 2):
            p = prepare.softmax_prepare(s_delta, cols, variant)
            got = gpu_softmax(scores, p)
            want = ref.softmax_i32(scores, p)
            assert np.array_equal(got, want)
            ops = ip.softmax_op_count(variant, rows, cols)
            assert ops == metric.softmax_op_count(variant, rows, cols)
            lib_c.append(ip.unified_metric(np.ascontiguousarray(x), got.astype(np.float64) / 128.0, ops, lib_mode))
            ref_c.append(metric.unified_metric(x, want.astype(np.float64) / 128.0, ops, mode))
        for a, b in zip(lib_c, ref_c):
            assert a.q_db == pytest.approx(b.q_db, rel=1e-12) and a.p == pytest.approx(b.p, rel=1e-12)
            assert a.score == pytest.approx(b.score, rel=1e-12)
        best = ip.unified_select(lib_c)
        assert best == metric.select(ref_c)
        picks.append(best)
        omega_lib += lib_c[best].score
        omega_ref += ref_c[best].score
    for layer in range(6):                                                  # GELU layers
        n = 5000 + 13 * layer
        s_in = 2.0 ** rng.uniform(-7, -4)
        q = np.clip(np.rint(rng.standard_normal(n) * 1.5 / s_in), -127, 127).astype(np.int8)
        xr = q.astype(np.float64) * s_in
        x = 0.5 * xr * (1.0 + erf(xr / np.sqrt(2.0)))                       # Eq. 1
        s_out = max(np.abs(x).max(), 1e-6) / 127.0
        lib_c, ref_c = [], []
        for variant in (0, 1):
            gp = prepare.gelu_prepare(s_in, s_out, 0, 0, variant)
            got = gpu_gelu_i8(q, gp)
            want = ref.gelu_i8(q, gp)
            assert np.array_equal(got, want)
            ops = ip.gelu_op_count(variant, n)
            lib_c.append(ip.unified_metric(x, got.astype(np.float64) * s_out, ops, lib_mode))
            ref_c.append(metric.unified_metric(x, want.astype(np.float64) * s_out, ops, mode))
        best = ip.unified_select(lib_c)
        assert best == metric.select(ref_c)
        picks.append(best)
        omega_lib += lib_c[best].score
        omega_ref += ref_c[best].score
    assert omega_lib == pytest.approx(omega_ref, rel=1e-12)
    if mode == "literal":
        # whole-layer perturbation and operation count swamp the SQNR term: always the cheapest
        assert picks == [0] * 12
