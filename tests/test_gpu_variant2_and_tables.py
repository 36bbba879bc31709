"""GPU parity for the second-degree Bit-exp (variant 2) and for additive-table entries equal to
INT32_MIN (masked whatever the score), on every kernel family, against the oracle."""
import numpy as np
import pytest

import workloads
from oracle import prepare, ref
from tests.helpers import gpu_softmax

pytestmark = pytest.mark.gpu
INT32_MIN = -(2 ** 31)


@pytest.mark.parametrize("name,unit,batch", [("deit_t", 0, 1), ("vit_b", 5, 1), ("swin_b", 0, 1),
                                             ("swin_b", 2, 3), ("swin_s_det", 0, 1)])
def test_variant2_configs(name, unit, batch):
    case = workloads.softmax_case(name, unit, batch=batch)
    scores = case.scores[:case.scores.shape[0] - 3]
    for signed in (0, 1):
        p = prepare.softmax_prepare(case.s_delta, scores.shape[1], 2, signed)
        want = ref.softmax_i32(scores, p, case.bias, case.bias_period_rows)
        for algo in (0, 1, 2, 3):
            got = gpu_softmax(scores, p, case.bias, case.bias_period_rows, algo=algo)
            assert np.array_equal(got, want), (name, unit, signed, algo)


@pytest.mark.parametrize("cols", [49, 197, 144, 64, 700])
def test_variant2_soft_rows_and_parameter_range(cols):
    rng = np.random.default_rng(cols)
    for i0, n in ((16, 0), (16, 10), (181, 7), (1000, 5), (4095, 3), (65535, 0), (65535, 2)):
        m_bits = 30
        if cols * (i0 << n) > (1 << m_bits):
            continue
        rows = int(rng.integers(40, 200))
        scores = np.rint(rng.standard_normal((rows, cols)) * 1.5 * i0).astype(np.int32)
        scores[rng.random(scores.shape) < 0.02] = INT32_MIN
        for out_bits in (8, 6):
            p = ref.SoftmaxParams(variant=2, i0=i0, n_shift=n, m_bits=m_bits, out_bits=out_bits,
                                  post=ref.Dyadic(1, 0, 0, 0, 255))
            want = ref.softmax_i32(scores, p)
            assert want.any()
            assert np.array_equal(gpu_softmax(scores, p), want), (i0, n, out_bits)
    with pytest.raises(Exception):
        gpu_softmax(np.zeros((4, cols), np.int32), ref.SoftmaxParams(variant=2, i0=65536, n_shift=0))


@pytest.mark.parametrize("cols,period", [(49, 196), (49, 147), (197, 197), (64, 256), (800, 8), (5000, 4)])
def test_table_entry_int32_min_masks_positive_scores(cols, period):
    """An entry INT32_MIN of the additive table masks the key whatever its score; a row whose
    every key is masked that way is the all-masked row although its scores are positive."""
    rng = np.random.default_rng(cols + period)
    rows = period * 3 + 7
    scores = np.abs(np.rint(rng.standard_normal((rows, cols)) * 500)).astype(np.int32) + 1
    scores[1, :] = 2 ** 31 - 1
    bias = np.rint(rng.standard_normal((period, cols)) * 30).astype(np.int32)
    bias[rng.random(bias.shape) < 0.2] = INT32_MIN
    bias[2 % period, :] = INT32_MIN
    bias[3 % period, :] = INT32_MIN + 1                     # finite: a live row
    for variant in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -6, cols, variant)
        p.post = ref.Dyadic(1, 0, 5, 0, 255)
        want = ref.softmax_i32(scores, p, bias, period)
        assert want[2 % period].tolist() == [5] * cols
        assert want[3 % period].max() > 5
        for algo in (0, 1, 2, 3):
            assert np.array_equal(gpu_softmax(scores, p, bias, period, algo=algo), want), (variant, algo)


@pytest.mark.parametrize("heads", [4, 3])
def test_bias_with_rare_minus_infinity_operands(heads):
    """Most slabs hold no INT32_MIN at all and a few do (the kernel adds the table with the plain
    saturating sum and repeats a slab with the minus-infinity rule when one of its operands is
    INT32_MIN): masked scores under positive table entries, masked table entries under positive
    scores, sums that saturate at both ends, in a tensor of several thousand slabs."""
    rng = np.random.default_rng(40 + heads)
    cols, period = 49, heads * 49
    rows = 5000 * 32 + 11
    scores = np.rint(rng.standard_normal((rows, cols)) * 600).astype(np.int32)
    bias = np.rint(rng.standard_normal((period, cols)) * 30).astype(np.int32)
    bias[5, 7] = INT32_MIN                                   # one masked table entry: every 32-row slab that holds table row 5
    bias[6, 3] = 2 ** 31 - 1
    bias[7, 3] = INT32_MIN + 1
    hit = rng.random(scores.shape) < 2e-5
    scores[hit] = INT32_MIN
    scores[rng.random(scores.shape) < 1e-5] = 2 ** 31 - 1
    scores[rng.random(scores.shape) < 1e-5] = INT32_MIN + 1
    scores[6, 3] = 2 ** 31 - 5                                # saturates upward with bias[6, 3]
    scores[7, 3] = -9                                         # with bias[7, 3] the sum clamps at INT32_MIN, which then counts as minus infinity
    for variant in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -7, cols, variant)
        want = ref.softmax_i32(scores, p, bias, period)
        assert np.array_equal(gpu_softmax(scores, p, bias, period, algo=4), want), (heads, variant)
