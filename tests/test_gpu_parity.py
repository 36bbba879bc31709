"""GPU parity: the HIP path against the CPU oracle, bit for bit, through the C ABI.

Every comparison is exact equality (integer work).  Inputs come from the seeded
generators; sizes here are what the oracle finishes in seconds, chosen to span several
wavefront slabs plus a ragged tail.  Full benchmark sizes are in test_gpu_fullsize.py.
"""
import numpy as np
import pytest

import workloads
from oracle import prepare, ref
from tests.helpers import (gpu_gelu_i8, gpu_gelu_i32, gpu_requant, gpu_softmax, lib_dyadic, lib_gelu,
                           lib_softmax)

pytestmark = pytest.mark.gpu
INT32_MIN = -(2 ** 31)

# (config, unit, reduced batch): a few thousand rows each, never a multiple of the slab
SOFTMAX_CASES = [("deit_t", 0, 1), ("vit_s", 3, 3), ("vit_b", 7, 2), ("swin_b", 0, 1),
                 ("swin_b", 1, 2), ("swin_b", 3, 5), ("swin_s_det", 0, 1)]


def _trim(case, drop):
    """Drop a few rows so that the row count is ragged with respect to every slab size."""
    rows = case.scores.shape[0] - drop
    return case.scores[:rows]


@pytest.mark.parametrize("name,unit,batch", SOFTMAX_CASES)
@pytest.mark.parametrize("variant", [0, 1])
def test_softmax_configs(name, unit, batch, variant):
    case = workloads.softmax_case(name, unit, batch=batch)
    scores = _trim(case, 5)
    for signed in (0, 1):
        p = prepare.softmax_prepare(case.s_delta, scores.shape[1], variant, signed)
        want = ref.softmax_i32(scores, p, case.bias, case.bias_period_rows)
        got = gpu_softmax(scores, p, case.bias, case.bias_period_rows)
        assert got.dtype == want.dtype
        assert np.array_equal(got, want), (name, unit, variant, signed)
    # the generic kernel family gives the same bytes
    p = prepare.softmax_prepare(case.s_delta, scores.shape[1], variant, 0)
    want = ref.softmax_i32(scores, p, case.bias, case.bias_period_rows)
    got = gpu_softmax(scores, p, case.bias, case.bias_period_rows, algo=1)
    assert np.array_equal(got, want)
    # and so does the run-time-row-length slab kernel
    got = gpu_softmax(scores, p, case.bias, case.bias_period_rows, algo=2)
    assert np.array_equal(got, want)
    got = gpu_softmax(scores, p, case.bias, case.bias_period_rows, algo=3)
    assert np.array_equal(got, want)


@pytest.mark.parametrize("cols", [197, 49])
@pytest.mark.parametrize("variant", [0, 1])
def test_softmax_soft_rows_all_scales(cols, variant):
    # scores scaled so that S_delta * sigma is about 0.5 .. 4: many non-zero probabilities
    rng = np.random.default_rng(100 + cols + variant)
    for log2s in (-4, -5.3, -7, -8.6, -10):
        s_delta = 2.0 ** log2s
        spread = float(rng.choice([0.5, 1.5, 4.0])) / s_delta
        rows = int(rng.integers(130, 400))
        scores = np.rint(rng.standard_normal((rows, cols)) * spread).astype(np.int32)
        p = prepare.softmax_prepare(s_delta, cols, variant)
        want = ref.softmax_i32(scores, p)
        assert want.any()
        assert np.array_equal(gpu_softmax(scores, p), want), (log2s, rows)


@pytest.mark.parametrize("cols", [197, 49])
def test_softmax_mask_and_extreme_rows(cols):
    rng = np.random.default_rng(7)
    rows = 150
    scores = np.rint(rng.standard_normal((rows, cols)) * 600).astype(np.int32)
    scores[3, :] = INT32_MIN                               # fully masked row
    scores[4, ::2] = INT32_MIN                             # half masked
    scores[5, :] = INT32_MIN
    scores[5, 7] = INT32_MIN + 1                           # one live entry next to the sentinel
    scores[6, :] = INT32_MIN + 1 + rng.integers(0, 50, cols)   # whole row near INT32_MIN
    scores[6, 1::3] = INT32_MIN
    scores[7, :] = 2 ** 31 - 1 - rng.integers(0, 50, cols)     # whole row near INT32_MAX
    scores[8, :] = rng.integers(INT32_MIN, 2 ** 31, cols)      # full-range garbage
    scores[9, :] = 0
    scores[9, 0] = 2 ** 31 - 1
    scores[9, 1] = INT32_MIN + 1
    scores[70, :] = INT32_MIN                              # a masked row in a later slab
    scores[71, 5:] = INT32_MIN
    big = [(2 ** 20, 3, 31), (2 ** 23 - 1, 0, 31)] if cols == 197 else [(2 ** 20, 3, 30), (2 ** 24 - 1, 0, 30)]
    for variant in (0, 1):
        for i0, n, m_bits in [(16, 0, 30), (128, 7, 30), (1000, 5, 30)] + big:
            p = ref.SoftmaxParams(variant=variant, i0=i0, n_shift=n, m_bits=m_bits)
            want = ref.softmax_i32(scores, p)
            assert np.array_equal(gpu_softmax(scores, p), want), (variant, i0, n)
            assert np.array_equal(gpu_softmax(scores, p, algo=1), want), (variant, i0, n)
            assert np.array_equal(gpu_softmax(scores, p, algo=2), want), (variant, i0, n)
            assert np.array_equal(gpu_softmax(scores, p, algo=3), want), (variant, i0, n)


@pytest.mark.parametrize("cols", [1, 2, 3, 4, 5, 6, 7, 16, 50, 63, 64, 65, 128, 144, 145, 196, 198, 199,
                                  257, 401, 415, 416, 417, 577, 785, 800, 1017, 1018, 1019, 1025, 1270,
                                  1274, 1275, 1280, 2045, 2046, 2048, 3325, 3326, 4096, 4097, 4099, 5117,
                                  5118, 8192, 13309, 13310, 20477, 20478, 26618, 26619, 32765, 32766, 40957, 40958, 65536])
def test_softmax_any_row_length(cols):
    rng = np.random.default_rng(cols)
    rows = 137 if cols < 300 else (37 if cols < 6000 else 9)
    scores = np.rint(rng.standard_normal((rows, cols)) * 300).astype(np.int32)
    scores[2, : max(1, cols // 3)] = INT32_MIN
    for variant in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -7.3, cols, variant)
        want = ref.softmax_i32(scores, p)
        for algo in (0, 1, 2, 3):                   # every kernel family (each falls back if it cannot serve)
            assert np.array_equal(gpu_softmax(scores, p, algo=algo), want), algo


@pytest.mark.parametrize("cols", [197, 49, 198, 144, 257, 577, 50, 64, 145, 800, 1025])
def test_softmax_partial_last_slab(cols):
    """Row counts that leave a partial slab (compiled and run-time row lengths): every row is
    right and nothing is written past the last one."""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(7000 + cols)
    max_rows = 75
    scores = np.rint(rng.standard_normal((max_rows, cols)) * 700).astype(np.int32)
    scores[::5, 1] = INT32_MIN
    bias = np.rint(rng.standard_normal((64, cols)) * 30).astype(np.int32)
    d_scores = torch.from_numpy(scores).cuda()
    d_bias = torch.from_numpy(bias).cuda()
    cases = [(prepare.softmax_prepare(2.0 ** -7.2, cols, 1), False),
             (prepare.softmax_prepare(2.0 ** -6.1, cols, 0, out_is_signed=1), True),
             (ref.SoftmaxParams(variant=1, i0=300, n_shift=6, post=ref.Dyadic(3, 1, 10, 0, 255)), True)]
    for rows in (1, 2, 3, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 65, 75):
        for p, with_bias in cases:
            dt = torch.int8 if p.out_is_signed else torch.uint8
            d_out = torch.full((rows * cols + 64,), 0x5A, dtype=dt, device="cuda")
            want = ref.softmax_i32(scores[:rows], p, bias if with_bias else None, 64 if with_bias else 0)
            for algo in (4, 0):                           # the slab kernels, then the default choice
                d_out.fill_(0x5A)
                ip.softmax_i32(d_scores, d_bias if with_bias else None, 64 if with_bias else 0, d_out, rows,
                               cols, lib_softmax(p, algo))
                torch.cuda.synchronize()
                got = d_out.cpu().numpy()
                assert np.array_equal(got[:rows * cols].reshape(rows, cols), want), (rows, with_bias, algo)
                assert (got[rows * cols:] == 0x5A).all(), (rows, with_bias, algo)


@pytest.mark.parametrize("cols", [49, 197, 64, 600, 1025, 4097])
def test_softmax_signed_output_around_zero_point_minus_128(cols):
    """post = (1, 0, -128, -128, 127): probabilities as int8 codes p - 128, the operand form of a
    signed 8-bit matrix instruction.  One exclusive-or on the packed bytes in the kernels; the
    oracle evaluates the general step.  One-hot rows (p = 128 -> 0) and fully masked rows
    (p = 0 -> -128) included; a narrower clip must still take the general route."""
    rng = np.random.default_rng(4300 + cols)
    rows = 150 if cols < 1000 else 9
    scores = np.rint(rng.standard_normal((rows, cols)) * 500).astype(np.int32)
    scores[0, :] = -1000000
    scores[0, cols // 2] = 1000000                    # one-hot
    scores[1, :] = INT32_MIN                          # fully masked
    bias = np.rint(rng.standard_normal((4, cols)) * 30).astype(np.int32)
    for variant, out_bits in ((0, 8), (1, 8), (1, 6)):
        p = prepare.softmax_prepare(2.0 ** -7.0, cols, variant, out_is_signed=1)
        p.out_bits = out_bits
        for qmax in (127, 0, -1):
            p.post = ref.Dyadic(1, 0, -128, -128, qmax)
            for b, period in ((None, 0), (bias, 4)):
                want = ref.softmax_i32(scores, p, b, period)
                assert want[0, cols // 2] == min(2 ** (out_bits - 1) - 128, qmax) and (want[1] == -128).all()
                for algo in (0, 1, 2, 3):
                    assert np.array_equal(gpu_softmax(scores, p, b, period, algo=algo), want), (variant, qmax, algo)


@pytest.mark.parametrize("cols,period", [(49, 196), (49, 392), (49, 12544), (49, 147), (49, 294), (49, 33), (197, 197), (197, 2364), (64, 256), (5, 65), (9, 100), (333, 17),
                                         (64, 200), (100, 96), (100, 45), (256, 1024), (576, 2304), (33, 7)])
def test_softmax_additive_table_with_workgroups_that_share_its_rows(cols, period):
    """With an additive table the wavefronts of a workgroup take slabs that start at congruent
    rows modulo the table's period (so that they read the same table rows): every slab must
    still be served exactly once, for periods that divide the slab, share a factor with it or
    are coprime to it, with a row count that leaves the last group of slabs incomplete.  Tables
    whose size is not a multiple of four scores (Swin with 3 or 6 heads: 147 x 49, 294 x 49)
    are read in chunks of four that can straddle the table's end."""
    rng = np.random.default_rng(cols * 100003 + period)
    for rows in (period * 9 + 5, 4111, 257):
        scores = np.rint(rng.standard_normal((rows, cols)) * 400).astype(np.int32)
        scores[rng.random((rows, cols)) < 0.01] = INT32_MIN
        bias = np.rint(rng.standard_normal((period, cols)) * 60).astype(np.int32)
        bias[rng.random((period, cols)) < 0.01] = INT32_MIN
        p = prepare.softmax_prepare(2.0 ** -6.7, cols, 1)
        want = ref.softmax_i32(scores, p, bias, period)
        for algo in (0, 2):
            assert np.array_equal(gpu_softmax(scores, p, bias, period, algo=algo), want), (rows, algo)


@pytest.mark.parametrize("cols", [49, 197, 256, 768, 800, 1025, 4096, 5117, 13312])
def test_softmax_views_off_the_16_byte_grid(cols):
    """Score and output tensors that are views into larger buffers, cut at the same element (so
    the scores start off the 16-byte grid and the output at the matching byte), and views cut
    at different elements: every row is right and no byte outside the view is written.  (256,
    768, 4096 and 13312 columns: off the grid a row touches one block more than on it, which
    takes one pass more.)"""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(8100 + cols)
    rows = 21 if cols < 2000 else 6
    scores = np.rint(rng.standard_normal((rows, cols)) * 500).astype(np.int32)
    scores[1, ::3] = INT32_MIN
    bias = np.rint(rng.standard_normal((4, cols)) * 40).astype(np.int32)
    d_bias = torch.from_numpy(bias).cuda()
    n = rows * cols
    p = prepare.softmax_prepare(2.0 ** -7.1, cols, 1)
    for in_off, out_off, with_bias in ((1, 1, False), (2, 2, False), (3, 3, False), (3, 7, False),
                                       (1, 2, False), (0, 3, False), (2, 2, True), (5, 1, False)):
        d_in = torch.zeros(n + 16, dtype=torch.int32, device="cuda")
        d_in[in_off:in_off + n] = torch.from_numpy(scores.reshape(-1)).cuda()
        d_out = torch.full((n + 32,), 0x5A, dtype=torch.uint8, device="cuda")
        want = ref.softmax_i32(scores, p, bias if with_bias else None, 4 if with_bias else 0)
        for algo in (0, 3, 4):
            d_out.fill_(0x5A)
            lp = lib_softmax(p)
            lp.algo = algo
            ip.softmax_i32(d_in[in_off:in_off + n], d_bias if with_bias else None, 4 if with_bias else 0,
                           d_out[out_off:out_off + n], rows, cols, lp)
            torch.cuda.synchronize()
            got = d_out.cpu().numpy()
            assert np.array_equal(got[out_off:out_off + n].reshape(rows, cols), want), (in_off, out_off, algo)
            assert (got[:out_off] == 0x5A).all() and (got[out_off + n:] == 0x5A).all(), (in_off, out_off, algo)


@pytest.mark.parametrize("cols", [197, 49, 144])
def test_softmax_fused_pre_requant_shifts(cols):
    """The requantization in front of the softmax at every shift class: below 16 (general
    form), 16..32 and above 32 (folded into one multiply-add in the slab kernel)."""
    rng = np.random.default_rng(900 + cols)
    rows = 70
    wide = rng.integers(INT32_MIN, 2 ** 31, size=(rows, cols)).astype(np.int32)
    wide[3, :5] = [INT32_MIN, 2 ** 31 - 1, INT32_MIN + 1, 0, -1]
    bias = np.rint(rng.standard_normal((64, cols)) * 1e6).astype(np.int32)
    for pre_s in (1, 15, 16, 17, 24, 31, 32, 33, 40, 45, 62):
        for pre_m in (1, 2, 20000, 32767):
            # scale the scores so that the requantized values span a few hundred codes
            want_span = 300.0
            scale = min(1.0, want_span * 2.0 ** pre_s / pre_m / 2.0 ** 31)
            scores = np.where(wide == INT32_MIN, INT32_MIN, np.rint(wide * scale)).astype(np.int32)
            for variant, signed in ((0, 0), (1, 1)):
                p = prepare.softmax_prepare(2.0 ** -5.3, cols, variant, out_is_signed=signed)
                p.pre_m, p.pre_s = pre_m, pre_s
                want = ref.softmax_i32(scores, p, bias, 64)
                assert np.array_equal(gpu_softmax(scores, p, bias, 64), want), (pre_s, pre_m, variant)
                assert np.array_equal(gpu_softmax(scores, p), ref.softmax_i32(scores, p)), (pre_s, pre_m)


def test_softmax_max_cols():
    cols = 65536
    rng = np.random.default_rng(3)
    scores = np.rint(rng.standard_normal((3, cols)) * 50).astype(np.int32)
    p = prepare.softmax_prepare(2.0 ** -5, cols, 1)
    assert p.n_shift < 15 - p.i0.bit_length() + 1
    assert np.array_equal(gpu_softmax(scores, p), ref.softmax_i32(scores, p))


@pytest.mark.parametrize("cols,rows", [(197, 16), (197, 15), (197, 33), (49, 64), (49, 63), (49, 130)])
def test_softmax_pre_post_outbits_bias(cols, rows):
    rng = np.random.default_rng(rows * cols)
    scores = np.rint(rng.standard_normal((rows, cols)) * 9000).astype(np.int32)
    scores[1, 3] = INT32_MIN
    bias = np.rint(rng.standard_normal((7, cols)) * 500).astype(np.int32)
    bias[0, 0] = 2 ** 31 - 1
    bias[1, 1] = INT32_MIN
    big_bias = np.rint(rng.standard_normal((96, cols)) * 500).astype(np.int32)   # 96 * cols % 4 == 0
    variants = [
        ref.SoftmaxParams(variant=1, i0=128, n_shift=7, pre_m=20000, pre_s=18),
        ref.SoftmaxParams(variant=0, i0=64, n_shift=8, pre_m=3, pre_s=0),
        ref.SoftmaxParams(variant=1, i0=300, n_shift=6, post=ref.Dyadic(3, 1, 10, 0, 255)),
        ref.SoftmaxParams(variant=0, i0=300, n_shift=6, post=ref.Dyadic(-255, 7, 100, -128, 127),
                          out_is_signed=1),
        ref.SoftmaxParams(variant=1, i0=300, n_shift=6, post=ref.Dyadic(1, 0, 0, 0, 100)),
        ref.SoftmaxParams(variant=1, i0=300, n_shift=6, post=ref.Dyadic(32767, 62, -3, -128, 127),
                          out_is_signed=1),
        ref.SoftmaxParams(variant=0, i0=50, n_shift=3, out_bits=4, m_bits=20),
        ref.SoftmaxParams(variant=1, i0=50, n_shift=3, out_bits=2, m_bits=31),
    ]
    for p in variants:
        for b, period in ((None, 0), (bias, 7), (big_bias, 96), (bias[:1], 1)):
            want = ref.softmax_i32(scores, p, b, period)
            assert np.array_equal(gpu_softmax(scores, p, b, period), want)
            assert np.array_equal(gpu_softmax(scores, p, b, period, algo=2), want)
            assert np.array_equal(gpu_softmax(scores, p, b, period, algo=3), want)


def test_swin_shifted_window_mask_as_a_combined_table():
    """Relative-position bias [heads*49, 49] plus a per-window additive mask [windows, 49, 49]
    (0 or 'minus infinity'), folded into one table of period windows*heads*49 rows."""
    rng = np.random.default_rng(31)
    images, windows, heads, t = 3, 4, 4, 49
    rows = images * windows * heads * t
    scores = np.rint(rng.standard_normal((rows, t)) * 900).astype(np.int32)
    rel = np.rint(rng.standard_normal((heads, t, t)) * 8).astype(np.int32)
    region = rng.integers(0, 3, size=(windows, t))                       # shifted-window regions
    mask = np.where(region[:, :, None] == region[:, None, :], 0, INT32_MIN).astype(np.int64)
    mask[0] = 0                                                           # an unshifted window
    table = np.clip(rel[None].astype(np.int64) + mask[:, None], INT32_MIN, 2 ** 31 - 1)
    table = table.astype(np.int32).reshape(windows * heads * t, t)
    period = windows * heads * t
    for variant in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -7.5, t, variant)
        want = ref.softmax_i32(scores, p, table, period)
        # the masked keys get probability 0, and every row keeps some mass
        blocked = np.tile(mask[:, None] == INT32_MIN, (images, heads, 1, 1)).reshape(rows, t)
        assert not want[blocked].any() and want.sum(axis=1).min() > 100
        assert np.array_equal(gpu_softmax(scores, p, table, period), want)
        assert np.array_equal(gpu_softmax(scores, p, table, period, algo=2), want)
        assert np.array_equal(gpu_softmax(scores, p, table, period, algo=3), want)


def test_softmax_empty_and_layers_entry():
    import torch
    import paper_2511_15369_amd as ip
    p = lib_softmax(prepare.softmax_prepare(2.0 ** -7, 197, 1))
    d_in = torch.zeros(16, dtype=torch.int32, device="cuda")
    d_out = torch.full((16,), 7, dtype=torch.uint8, device="cuda")
    ip.softmax_i32(d_in, None, 0, d_out, 0, 197, p)
    torch.cuda.synchronize()
    assert (d_out == 7).all()
    # three layers with different scales and variants in one call
    rng = np.random.default_rng(4)
    rows, cols, layers = 50, 197, 3
    x = np.rint(rng.standard_normal((layers, rows, cols)) * 2000).astype(np.int32)
    ps = [prepare.softmax_prepare(2.0 ** -(5 + l), cols, l % 2) for l in range(layers)]
    d_x = torch.from_numpy(x).cuda()
    d_y = torch.zeros((layers, rows, cols), dtype=torch.uint8, device="cuda")
    ip.softmax_i32_layers(d_x, rows * cols, d_y, rows * cols, rows, cols, layers,
                          [lib_softmax(q) for q in ps])
    torch.cuda.synchronize()
    y = d_y.cpu().numpy()
    for l in range(layers):
        assert np.array_equal(y[l], ref.softmax_i32(x[l], ps[l]))


def test_softmax_is_deterministic():
    case = workloads.softmax_case("vit_s", 0, batch=2)
    p = prepare.softmax_prepare(2.0 ** -9, 197, 1)
    a = gpu_softmax(case.scores, p)
    b = gpu_softmax(case.scores, p)
    assert np.array_equal(a, b)


# --------------------------------------------------------------------------------- GELU
GELU_CASES = [("deit_t", 0, 1), ("vit_s", 5, 1), ("vit_b", 2, 1), ("swin_b", 0, 1),
              ("swin_b", 3, 2), ("swin_s_det", 0, 1)]


@pytest.mark.parametrize("name,unit,batch", GELU_CASES)
@pytest.mark.parametrize("variant", [0, 1])
def test_gelu_i8_configs(name, unit, batch, variant):
    case = workloads.gelu_case(name, unit, batch=batch)
    x = case.x.reshape(-1)[: min(case.x.size, 3_000_000) - 5]
    p = prepare.gelu_prepare(case.s_in, case.s_out, case.zp_in, case.zp_out, variant)
    want = ref.gelu_i8(x, p)
    assert np.array_equal(gpu_gelu_i8(x, p), want)
    assert np.array_equal(gpu_gelu_i8(x, p, algo=1), want)
    assert np.array_equal(gpu_gelu_i8(x, p, inplace=True), want)


@pytest.mark.parametrize("variant", [0, 1])
def test_gelu_all_codes_all_scales(variant):
    allx = np.tile(np.arange(-128, 128, dtype=np.int8), 5)[:-3]
    rng = np.random.default_rng(variant)
    for _ in range(25):
        s_in = float(2.0 ** rng.uniform(-12, -3))
        s_out = float(2.0 ** rng.uniform(-12, -3))
        zi, zo = int(rng.integers(-128, 129)), int(rng.integers(-128, 128))
        p = prepare.gelu_prepare(s_in, s_out, zi, zo, variant)
        want = ref.gelu_i8(allx, p)
        assert np.array_equal(gpu_gelu_i8(allx, p), want), (s_in, s_out, zi, zo)
        assert np.array_equal(gpu_gelu_i8(allx, p, algo=1), want), (s_in, s_out, zi, zo)
    # a requantization with a small shift (wide path) and a positive multiplier
    p = prepare.gelu_prepare(2.0 ** -4, 2.0 ** -5, 0, 0, variant, 128)
    p.post = ref.Dyadic(-3, 18, 5, -100, 90)
    assert np.array_equal(gpu_gelu_i8(allx, p), ref.gelu_i8(allx, p))
    p.post = ref.Dyadic(-1, 3, 0, -128, 127)
    assert np.array_equal(gpu_gelu_i8(allx, p, algo=1), ref.gelu_i8(allx, p))


@pytest.mark.parametrize("n", [0, 1, 15, 16, 17, 255, 4097, 100003])
def test_gelu_i8_sizes_and_unaligned(n):
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(n)
    p = prepare.gelu_prepare(2.0 ** -5.5, 2.0 ** -6, 3, -11, 1)
    x = rng.integers(-128, 128, size=n + 8, dtype=np.int8)
    d_x = torch.from_numpy(x).cuda()
    for off in (0, 1, 5):
        d_out = torch.full((n + 8,), 0x5A, dtype=torch.int8, device="cuda")
        ip.gelu_i8(d_x[off:], d_out[off:], n, lib_gelu(p))
        torch.cuda.synchronize()
        got = d_out.cpu().numpy()
        assert np.array_equal(got[off:off + n], ref.gelu_i8(x[off:off + n], p))
        assert (got[:off] == 0x5A).all() and (got[off + n:] == 0x5A).all()


@pytest.mark.parametrize("variant", [0, 1])
def test_gelu_i32(variant):
    rng = np.random.default_rng(50 + variant)
    n = 70001
    x = np.rint(rng.standard_normal(n) * 40000).astype(np.int32)
    x[:6] = [INT32_MIN, 2 ** 31 - 1, 0, -1, 1, 123456789]
    p = prepare.gelu_prepare(2.0 ** -7, 2.0 ** -4, 5, -20, variant, max_abs_q=2000)
    assert np.array_equal(gpu_gelu_i32(x, p), ref.gelu_i32(x, p))
    p.pre_m, p.pre_s = 23000, 21
    assert np.array_equal(gpu_gelu_i32(x, p), ref.gelu_i32(x, p))
    p.pre_m, p.pre_s = 32767, 0                            # saturating pre-requantization
    assert np.array_equal(gpu_gelu_i32(x, p), ref.gelu_i32(x, p))
    p.zp_in = 2 ** 31 - 1
    assert np.array_equal(gpu_gelu_i32(x, p), ref.gelu_i32(x, p))
    # a second-order case with a large |q_b| (square does not fit 32 bits)
    if variant == 0:
        p2 = prepare.gelu_prepare(2.0 ** -22, 2.0 ** -15, 0, 0, 0, max_abs_q=200000)
        assert -p2.q_b > 2 ** 17
        x2 = np.rint(rng.standard_normal(n) * 300000).astype(np.int32)
        assert np.array_equal(gpu_gelu_i32(x2, p2), ref.gelu_i32(x2, p2))


@pytest.mark.parametrize("variant", [0, 1])
@pytest.mark.parametrize("max_abs_q", [1, 127, 255, 511, 512])
def test_gelu_i32_small_range(variant, max_abs_q):
    """Input ranges up to 511 are served by the per-workgroup table, 512 by the per-element
    kernel; both agree with the oracle and with the per-element kernel forced by `algo`."""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(500 + 10 * max_abs_q + variant)
    n = 40003
    x = np.rint(rng.standard_normal(n + 8) * 60000).astype(np.int32)
    x[:6] = [INT32_MIN, 2 ** 31 - 1, 0, -1, 1, 123456789]
    x[6:6 + 2 * max_abs_q + 3] = np.arange(-max_abs_q - 1, max_abs_q + 2) * 256    # every q and one beyond
    for pre, zp in (((1, 0), 0), ((16384, 22), -7), ((32767, 3), 100), ((1, 0), INT32_MIN), ((5, 1), 2 ** 31 - 1)):
        p = prepare.gelu_prepare(2.0 ** -5, 2.0 ** -5, zp, -11, variant, max_abs_q=max_abs_q)
        p.pre_m, p.pre_s = pre
        xs = x if pre != (1, 0) else (x // 256).astype(np.int32)
        want = ref.gelu_i32(xs, p)
        assert np.array_equal(gpu_gelu_i32(xs, p), want), (pre, zp)
        assert np.array_equal(gpu_gelu_i32(xs, p, algo=1), want), (pre, zp)
    # unaligned input and output, guard bytes untouched
    p = prepare.gelu_prepare(2.0 ** -5, 2.0 ** -5, 3, 4, variant, max_abs_q=max_abs_q)
    p.pre_m, p.pre_s = 20000, 22
    d_x = torch.from_numpy(x).cuda()
    for off in (1, 2, 3):
        d_out = torch.full((n + 8,), 0x5A, dtype=torch.int8, device="cuda")
        ip.gelu_i32(d_x[off:], d_out[off:], n, lib_gelu(p))
        torch.cuda.synchronize()
        got = d_out.cpu().numpy()
        assert np.array_equal(got[off:off + n], ref.gelu_i32(x[off:off + n], p))
        assert (got[:off] == 0x5A).all() and (got[off + n:] == 0x5A).all()


def test_gelu_layers_entry():
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(9)
    n, layers = 5000, 4
    x = rng.integers(-128, 128, size=(layers, n), dtype=np.int8)
    ps = [prepare.gelu_prepare(2.0 ** -(4 + l), 2.0 ** -(5 + l), 0, l, l % 2) for l in range(layers)]
    d_x = torch.from_numpy(x).cuda()
    d_y = torch.zeros_like(d_x)
    ip.gelu_i8_layers(d_x, n, d_y, n, n, layers, [lib_gelu(q) for q in ps])
    torch.cuda.synchronize()
    y = d_y.cpu().numpy()
    for l in range(layers):
        assert np.array_equal(y[l], ref.gelu_i8(x[l], ps[l]))


# --------------------------------------------------------------------------------- requant
@pytest.mark.parametrize("seed", range(3))
def test_requant(seed):
    rng = np.random.default_rng(seed)
    n = 100003
    x = rng.integers(INT32_MIN, 2 ** 31, size=n).astype(np.int32)
    x[:4] = [INT32_MIN, 2 ** 31 - 1, 0, -1]
    small = np.rint(rng.standard_normal(n) * 3000).astype(np.int32)
    for _ in range(12):
        m = int(rng.integers(-32767, 32768))
        s = int(rng.integers(0, 63))
        zp = int(rng.integers(-300, 300))
        signed = int(rng.integers(0, 2))
        lo, hi = (-128, 127) if signed else (0, 255)
        d = ref.Dyadic(m, s, zp, lo, hi)
        for data in (x, small):
            assert np.array_equal(gpu_requant(data, d, signed), ref.requant(data, d, signed)), (m, s)
    d = ref.Dyadic(*prepare.make_dyadic(0.0123), 3, -128, 127)
    assert np.array_equal(gpu_requant(small, d, 1), ref.requant(small, d, 1))


# --------------------------------------------------------------------------------- batched forms
def test_softmax_batch_mixed_problems():
    """One call, problems that differ in size, scale, variant, bias, output type and kernel
    family (packed, 32-bit, generic, ragged tails): each must equal its single-call result."""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(21)
    for cols in (49, 197, 33):
        specs = []
        for i in range(11):
            rows = int(rng.integers(1, 400))
            x = np.rint(rng.standard_normal((rows, cols)) * float(rng.choice([200, 3000]))).astype(np.int32)
            if i % 4 == 1:
                x[0, :] = INT32_MIN
            p = prepare.softmax_prepare(float(2.0 ** rng.uniform(-10, -4)), cols, i % 2, int(i % 3 == 0))
            if i == 5:
                p = ref.SoftmaxParams(variant=1, i0=2 ** 16, n_shift=2, out_is_signed=0)      # 32-bit arithmetic
            if i == 6:
                p.post = ref.Dyadic(3, 1, 7, 0, 255) if not p.out_is_signed else ref.Dyadic(3, 1, 7, -128, 127)
            if i == 7:
                p.pre_m, p.pre_s = 5, 1
            bias, period = None, 0
            if i % 5 == 2:
                period = 96
                bias = np.rint(rng.standard_normal((period, cols)) * 50).astype(np.int32)
            specs.append((x, p, bias, period))
        probs, keep = [], []
        for x, p, bias, period in specs:
            d_x = torch.from_numpy(x).cuda()
            d_b = None if bias is None else torch.from_numpy(bias).cuda()
            d_y = torch.full(x.shape, 0x5A, dtype=torch.int8 if p.out_is_signed else torch.uint8, device="cuda")
            keep.append((d_x, d_b, d_y))
            probs.append(ip.softmax_problem(d_x, d_b, period, d_y, x.shape[0], cols, lib_softmax(p)))
        ip.softmax_i32_batch(probs, len(probs), cols)
        torch.cuda.synchronize()
        for (x, p, bias, period), (_, _, d_y) in zip(specs, keep):
            assert np.array_equal(d_y.cpu().numpy(), ref.softmax_i32(x, p, bias, period))


def test_gelu_batch_mixed_problems():
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(22)
    specs, probs, keep = [], [], []
    for i in range(16):
        n = int(rng.choice([1, 15, 16, 4099, 70000, 300001]))
        x = rng.integers(-128, 128, size=n, dtype=np.int8)
        p = prepare.gelu_prepare(float(2.0 ** rng.uniform(-10, -4)), float(2.0 ** rng.uniform(-9, -4)),
                                 int(rng.integers(-20, 20)), int(rng.integers(-100, 100)), i % 2)
        d_x = torch.from_numpy(x).cuda()
        d_y = torch.full((n,), 0x5A, dtype=torch.int8, device="cuda")
        specs.append((x, p))
        keep.append((d_x, d_y))
        probs.append(ip.gelu_problem(d_x, d_y, n, lib_gelu(p, algo=int(i == 9))))
    ip.gelu_i8_batch(probs, len(probs))
    torch.cuda.synchronize()
    for (x, p), (_, d_y) in zip(specs, keep):
        assert np.array_equal(d_y.cpu().numpy(), ref.gelu_i8(x, p))


def test_layers_entry_more_than_one_batch():
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(23)
    rows, cols, layers = 70, 49, 19
    x = np.rint(rng.standard_normal((layers, rows, cols)) * 700).astype(np.int32)
    ps = [prepare.softmax_prepare(float(2.0 ** rng.uniform(-10, -4)), cols, l % 2) for l in range(layers)]
    d_x = torch.from_numpy(x).cuda()
    d_y = torch.zeros((layers, rows, cols), dtype=torch.uint8, device="cuda")
    ip.softmax_i32_layers(d_x, rows * cols, d_y, rows * cols, rows, cols, layers, [lib_softmax(q) for q in ps])
    torch.cuda.synchronize()
    y = d_y.cpu().numpy()
    for l in range(layers):
        assert np.array_equal(y[l], ref.softmax_i32(x[l], ps[l])), l


def test_calls_can_be_captured_in_a_hip_graph():
    """The entry points only enqueue kernels on the caller's stream (no allocation, no memset,
    no synchronisation), so a whole DeiT-Tiny block can be captured once and replayed; every
    replay, with fresh inputs copied into the captured buffers, must match the oracle."""
    import torch
    import paper_2511_15369_amd as ip
    sc = workloads.softmax_case("deit_t")
    gc = workloads.gelu_case("deit_t")
    rows, cols = sc.scores.shape
    sp = prepare.softmax_prepare(sc.s_delta, cols, 1)
    gp = prepare.gelu_prepare(gc.s_in, gc.s_out, gc.zp_in, gc.zp_out, 1)
    d_s = torch.from_numpy(sc.scores).cuda()
    d_p = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
    d_x = torch.from_numpy(gc.x.reshape(-1)).cuda()
    d_y = torch.zeros_like(d_x)
    lsp, lgp = lib_softmax(sp), lib_gelu(gp)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        ip.softmax_i32(d_s, None, 0, d_p, rows, cols, lsp)
        ip.gelu_i8(d_x, d_y, d_x.numel(), lgp)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        ip.softmax_i32(d_s, None, 0, d_p, rows, cols, lsp)
        ip.gelu_i8(d_x, d_y, d_x.numel(), lgp)
    rng = np.random.default_rng(77)
    for rep in range(4):
        s_new = np.rint(rng.standard_normal((rows, cols)) * (300 + 900 * rep)).astype(np.int32)
        x_new = rng.integers(-128, 128, size=d_x.numel(), dtype=np.int8)
        d_s.copy_(torch.from_numpy(s_new))
        d_x.copy_(torch.from_numpy(x_new))
        d_p.zero_()
        d_y.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(d_p.cpu().numpy(), ref.softmax_i32(s_new, sp)), rep
        assert np.array_equal(d_y.cpu().numpy(), ref.gelu_i8(x_new, gp)), rep


def test_concurrent_calls_from_several_host_threads_and_streams():
    """The library keeps no state: host threads that call it at the same time, each on a stream
    of its own, get the same results as one thread would."""
    import threading
    import torch
    import paper_2511_15369_amd as ip
    n_threads, rounds = 4, 25
    rng = np.random.default_rng(31)
    jobs = []
    for t in range(n_threads):
        cols = (197, 49, 64, 1025)[t]
        rows = 300 if cols < 1000 else 40
        x = np.rint(rng.standard_normal((rows, cols)) * 600).astype(np.int32)
        sp = prepare.softmax_prepare(2.0 ** -(6.0 + t), cols, t % 2)
        g = rng.integers(-128, 128, size=50000 + 13 * t, dtype=np.int8)
        gp = prepare.gelu_prepare(2.0 ** -(4.0 + t), 2.0 ** -5.0, t, -t, t % 2)
        jobs.append((x, sp, ref.softmax_i32(x, sp), g, gp, ref.gelu_i8(g, gp)))
    errors = []

    def worker(t):
        try:
            x, sp, want_s, g, gp, want_g = jobs[t]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                d_x = torch.from_numpy(x).cuda()
                d_g = torch.from_numpy(g).cuda()
                lsp, lgp = lib_softmax(sp), lib_gelu(gp)
                for _ in range(rounds):
                    d_p = torch.zeros(x.shape, dtype=torch.uint8, device="cuda")
                    d_y = torch.zeros_like(d_g)
                    ip.softmax_i32(d_x, None, 0, d_p, x.shape[0], x.shape[1], lsp)
                    ip.gelu_i8(d_g, d_y, d_g.numel(), lgp)
                    stream.synchronize()
                    if not (np.array_equal(d_p.cpu().numpy(), want_s) and np.array_equal(d_y.cpu().numpy(), want_g)):
                        errors.append((t, "mismatch"))
                        return
        except Exception as exc:                      # surfaces in the main thread below
            errors.append((t, repr(exc)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(n_threads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
    assert not any(th.is_alive() for th in threads)
    assert not errors, errors


def test_elementwise_views_at_every_offset():
    """Requantization, GELU on int32 accumulators and GELU on int8 codes on views that start at
    every offset of the input's and the output's 16-byte grids (the kernels peel the output's
    head up to its vector boundary and load the input wherever that leaves it): exact results,
    no byte outside the view written, sizes around the peel / vector / tail boundaries."""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(909)
    dy = ref.Dyadic(-23170, 21, 5, -128, 127)
    gp32 = prepare.gelu_prepare(2.0 ** -4.7, 2.0 ** -5.2, 2, -3, 1, max_abs_q=127)
    gp32.pre_m, gp32.pre_s = 20000, 26
    gp8 = prepare.gelu_prepare(2.0 ** -4.7, 2.0 ** -5.2, 2, -3, 1)
    for n in (63, 64, 65, 67, 100, 4099, 70001):
        x32 = rng.integers(-(2 ** 31), 2 ** 31, size=n).astype(np.int32)
        x8 = rng.integers(-128, 128, size=n, dtype=np.int8)
        want_rq = ref.requant(x32, dy, 1)
        want_g32 = ref.gelu_i32(x32, gp32)
        want_g8 = ref.gelu_i8(x8, gp8)
        for in_off in (0, 1, 2, 3, 5):
            d_x32 = torch.zeros(n + 8, dtype=torch.int32, device="cuda")
            d_x32[in_off:in_off + n] = torch.from_numpy(x32).cuda()
            for out_off in (0, 1, 2, 3, 4, 7, 15):
                for what, want in (("requant", want_rq), ("gelu_i32", want_g32), ("gelu_i32 direct", want_g32)):
                    d_y = torch.full((n + 32,), 0x5A, dtype=torch.int8, device="cuda")
                    if what == "requant":
                        ip.requant(d_x32[in_off:in_off + n], d_y[out_off:out_off + n], n, 1, lib_dyadic(dy))
                    else:
                        ip.gelu_i32(d_x32[in_off:in_off + n], d_y[out_off:out_off + n], n,
                                    lib_gelu(gp32, algo=int(what.endswith("direct"))))
                    torch.cuda.synchronize()
                    got = d_y.cpu().numpy()
                    assert np.array_equal(got[out_off:out_off + n], want), (what, n, in_off, out_off)
                    assert (got[:out_off] == 0x5A).all() and (got[out_off + n:] == 0x5A).all(), (what, n, in_off, out_off)
        for in_off in (0, 1, 3, 4, 9, 15, 16, 17):
            d_x8 = torch.zeros(n + 32, dtype=torch.int8, device="cuda")
            d_x8[in_off:in_off + n] = torch.from_numpy(x8).cuda()
            for out_off in (0, 1, 3, 4, 9, 15, 16, 17):
                d_y = torch.full((n + 48,), 0x5A, dtype=torch.int8, device="cuda")
                ip.gelu_i8(d_x8[in_off:in_off + n], d_y[out_off:out_off + n], n, lib_gelu(gp8))
                torch.cuda.synchronize()
                got = d_y.cpu().numpy()
                assert np.array_equal(got[out_off:out_off + n], want_g8), ("gelu_i8", n, in_off, out_off)
                assert (got[:out_off] == 0x5A).all() and (got[out_off + n:] == 0x5A).all(), ("gelu_i8", n, in_off, out_off)
        # in place on an unaligned view
        d_io = torch.zeros(n + 32, dtype=torch.int8, device="cuda")
        d_io[5:5 + n] = torch.from_numpy(x8).cuda()
        ip.gelu_i8(d_io[5:5 + n], d_io[5:5 + n], n, lib_gelu(gp8))
        torch.cuda.synchronize()
        assert np.array_equal(d_io.cpu().numpy()[5:5 + n], want_g8), ("in place", n)


def test_library_loaded_before_torch_binds_to_torchs_hip_runtime():
    """A process that loads the library first and imports torch afterwards must still launch on
    the runtime torch's buffers belong to (torch ships its own copy of the HIP runtime)."""
    import os
    import subprocess
    import sys
    code = (
        "import paper_2511_15369_amd as ip\n"
        "ip.load()\n"
        "import torch\n"
        "x = torch.arange(-4000, 3880, dtype=torch.int32, device='cuda').reshape(40, 197)\n"
        "o = torch.zeros((40, 197), dtype=torch.uint8, device='cuda')\n"
        "ip.softmax_i32(x, None, 0, o, 40, 197, ip.softmax_prepare(2.0 ** -6, 197, 1, 0))\n"
        "torch.cuda.synchronize()\n"
        "print('sum', int(o.sum()))\n")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", code], cwd=root, capture_output=True, text=True, timeout=240)
    assert r.returncode == 0, r.stderr[-2000:]
    x = np.arange(-4000, 3880, dtype=np.int32).reshape(40, 197)
    want = ref.softmax_i32(x, prepare.softmax_prepare(2.0 ** -6, 197, 1))
    assert "sum %d" % int(want.sum()) in r.stdout
