"""Pins for the oracle's softmax with a per-window additive mask beside the relative-position
bias (shifted-window attention of the Swin-shaped benchmark configurations; Section 4.1 keeps
every operation of the block in integer arithmetic).  What fixes it: a hand-worked two-window
case, and the composition of both tables into one (built here, row by row, in plain Python)
fed to the plain-table entry point, which has its own pins."""
import numpy as np

from oracle import ref

INT32_MIN = -(2 ** 31)


def compose(bias, mask, heads, cols):
    """table[(w * heads + h) * cols + q] = bias[h * cols + q] (+) mask[w, q]; (+) is the
    saturating sum with INT32_MIN absorbing."""
    n_w = mask.shape[0]
    out = np.empty((n_w * heads * cols, cols), np.int64)
    for w in range(n_w):
        for h in range(heads):
            for q in range(cols):
                b = bias[h * cols + q].astype(np.int64)
                m = mask[w, q].astype(np.int64)
                s = np.clip(b + m, INT32_MIN, 2 ** 31 - 1)
                s[(b == INT32_MIN) | (m == INT32_MIN)] = INT32_MIN
                out[(w * heads + h) * cols + q] = s
    return out.astype(np.int32)


def test_hand_worked_two_windows():
    # cols = 2, one head, two windows, two images: rows [image, window, head, query].
    # window 0 masks nothing; window 1 masks key 1 for query 0 and key 0 for query 1.
    p = ref.SoftmaxParams(variant=1, i0=16, n_shift=0)
    mask = np.array([[[0, 0], [0, 0]], [[0, INT32_MIN], [INT32_MIN, 0]]], np.int32)
    scores = np.array([[5, 5], [5, 5], [5, 9], [9, 5]] * 2, np.int32)
    got = ref.softmax_i32_windowed(scores, p, None, 0, mask, 1)
    # unmasked equal pair -> 64, 64; a single live key -> 128 (rows B and C of the golden file)
    want = [[64, 64], [64, 64], [128, 0], [0, 128]] * 2
    assert got.tolist() == want


def test_windowed_equals_the_composed_table():
    rng = np.random.default_rng(21)
    for cols, heads, n_w, images in ((5, 2, 3, 2), (7, 3, 4, 3), (4, 1, 2, 5)):
        p = ref.SoftmaxParams(variant=int(rng.integers(0, 3)), i0=64, n_shift=8)
        rows = images * n_w * heads * cols
        scores = np.rint(rng.standard_normal((rows, cols)) * 150).astype(np.int32)
        scores[rng.random((rows, cols)) < 0.03] = INT32_MIN
        bias = np.rint(rng.standard_normal((heads * cols, cols)) * 20).astype(np.int32)
        mask = np.where(rng.random((n_w, cols, cols)) < 0.3, INT32_MIN, 0).astype(np.int32)
        mask[0] = 0
        mask[-1, 1, :] = INT32_MIN                       # a fully masked query in the last window
        table = compose(bias, mask, heads, cols)
        want = ref.softmax_i32(scores, p, table, n_w * heads * cols)
        got = ref.softmax_i32_windowed(scores, p, bias, heads * cols, mask, heads)
        assert np.array_equal(got, want)
        # the fully masked query yields the zero-point (0) in every image and head
        for img in range(images):
            for h in range(heads):
                r = ((img * n_w + (n_w - 1)) * heads + h) * cols + 1
                assert got[r].tolist() == [0] * cols
        # mask without bias, bias without mask
        assert np.array_equal(ref.softmax_i32_windowed(scores, p, None, 0, mask, heads),
                              ref.softmax_i32(scores, p, compose(np.zeros_like(bias), mask, heads, cols),
                                              n_w * heads * cols))
        assert np.array_equal(ref.softmax_i32_windowed(scores, p, bias, heads * cols, None, heads),
                              ref.softmax_i32(scores, p, bias, heads * cols))


def test_general_additive_mask_values():
    # a finite negative mask value is an ordinary addend (the -100-style mask of the float model)
    p = ref.SoftmaxParams(variant=0, i0=16, n_shift=0)
    mask = np.array([[[0, -20], [0, 0]]], np.int32)
    scores = np.array([[3, 3], [3, 3]], np.int32)
    got = ref.softmax_i32_windowed(scores, p, None, 0, mask, 1)
    # row 0: deltas 0, -20 -> variant 0 of row A in the golden file: Qexp 16 and 5, sum 21,
    # f = floor(2^30 / 21) = 51130563, p = (16 f) >> 23 = 97, (5 f) >> 23 = 30
    assert got.tolist() == [[97, 30], [64, 64]]


def test_packed_mask_by_hand_and_round_trip():
    # 2 windows of 3 tokens: window 0 unmasked; window 1: query 0 masks key 2, query 2 masks keys 0, 1
    mask = np.zeros((2, 3, 3), np.int32)
    mask[1, 0, 2] = INT32_MIN
    mask[1, 2, 0] = mask[1, 2, 1] = INT32_MIN
    mask[0, 1, 1] = -7                                   # a finite addend is "not masked"
    bits = ref.pack_window_mask(mask)
    assert bits.shape == (2, 3, 1) and bits.dtype == np.uint64
    assert bits[:, :, 0].tolist() == [[0, 0, 0], [4, 0, 3]]
    back = ref.unpack_window_mask(bits, 3)
    want = mask.copy()
    want[0, 1, 1] = 0
    assert np.array_equal(back, want)
    # more than 64 keys: two words per row, bit 64 is bit 0 of the second word
    big = np.zeros((1, 70, 70), np.int32)
    big[0, 5, 63] = big[0, 5, 64] = big[0, 5, 69] = INT32_MIN
    b = ref.pack_window_mask(big)
    assert b.shape == (1, 70, 2)
    assert int(b[0, 5, 0]) == 1 << 63 and int(b[0, 5, 1]) == (1 << 0) | (1 << 5)
    assert np.array_equal(ref.unpack_window_mask(b, 70), big)
    rng = np.random.default_rng(3)
    m = np.where(rng.random((3, 49, 49)) < 0.3, INT32_MIN, 0).astype(np.int32)
    assert np.array_equal(ref.unpack_window_mask(ref.pack_window_mask(m), 49), m)


def test_softmax_with_packed_mask_equals_the_int32_mask():
    rng = np.random.default_rng(4)
    cols, heads, n_w = 6, 2, 3
    rows = 2 * n_w * heads * cols
    scores = np.rint(rng.standard_normal((rows, cols)) * 100).astype(np.int32)
    bias = np.rint(rng.standard_normal((heads * cols, cols)) * 10).astype(np.int32)
    mask = np.where(rng.random((n_w, cols, cols)) < 0.3, INT32_MIN, 0).astype(np.int32)
    p = ref.SoftmaxParams(variant=1, i0=64, n_shift=8)
    a = ref.softmax_i32_windowed(scores, p, bias, heads * cols, mask, heads)
    b = ref.softmax_i32_windowed_bits(scores, p, bias, heads * cols, ref.pack_window_mask(mask), heads)
    assert np.array_equal(a, b)
