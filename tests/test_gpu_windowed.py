"""GPU parity of the softmax with a per-window mask beside the relative-position bias
(shifted-window attention; iptq_softmax_i32_windowed) against the oracle, bit for bit, through
the C ABI: small ragged cases on every route, every discontinuity of the mask rows inside a
slab, and the Swin-B stages at full size in the launch configuration the benchmark times."""
import numpy as np
import pytest

import workloads
from oracle import prepare, ref
from tests.helpers import (gpu_pack_window_mask, gpu_softmax, gpu_softmax_windowed, gpu_softmax_windowed_bits,
                           lib_softmax)

pytestmark = pytest.mark.gpu
INT32_MIN = -(2 ** 31)


def _case(rng, images, side, heads, win=7, shift=3, drop=0, spread=600.0):
    t = win * win
    mask = workloads.shifted_window_mask(side, side, win, shift)
    n_w = mask.shape[0]
    rows = images * n_w * heads * t - drop
    scores = np.rint(rng.standard_normal((rows, t)) * spread).astype(np.int32)
    bias = np.rint(rng.standard_normal((heads * t, t)) * 8).astype(np.int32)
    return scores, bias, mask


@pytest.mark.parametrize("heads,side", [(4, 14), (3, 14), (8, 21), (1, 14), (6, 28)])
@pytest.mark.parametrize("variant", [0, 1, 2])
def test_windowed_small(heads, side, variant):
    """Row counts that leave a partial slab; 3 and 6 heads give a bias table whose size is not a
    multiple of four (its own straddling chunk beside the mask's)."""
    rng = np.random.default_rng(heads * 1000 + side * 10 + variant)
    scores, bias, mask = _case(rng, 3, side, heads, drop=int(rng.integers(0, 40)))
    scores[rng.random(scores.shape) < 0.01] = INT32_MIN
    for signed in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -6.5, 49, variant, signed)
        want = ref.softmax_i32_windowed(scores, p, bias, heads * 49, mask, heads)
        for algo in (0, 1):
            got = gpu_softmax_windowed(scores, p, bias, heads * 49, mask, heads, algo=algo)
            assert np.array_equal(got, want), (heads, side, variant, signed, algo)
    # masked keys get probability 0 and every row keeps mass
    blocked = np.tile(mask[:, None] == INT32_MIN, (3, heads, 1, 1)).reshape(-1, 49)[:scores.shape[0]]
    assert not want[blocked].any()


def test_windowed_equals_a_combined_table_on_the_gpu():
    rng = np.random.default_rng(5)
    heads, side = 4, 14
    scores, bias, mask = _case(rng, 5, side, heads)
    n_w = mask.shape[0]
    table = np.empty((n_w, heads, 49, 49), np.int64)
    table[:] = bias.reshape(1, heads, 49, 49).astype(np.int64) + mask[:, None].astype(np.int64)
    table = np.clip(table, INT32_MIN, 2 ** 31 - 1)
    table[np.broadcast_to(mask[:, None] == INT32_MIN, table.shape)] = INT32_MIN
    table = table.astype(np.int32).reshape(n_w * heads * 49, 49)
    p = prepare.softmax_prepare(2.0 ** -7.5, 49, 1)
    got = gpu_softmax_windowed(scores, p, bias, heads * 49, mask, heads)
    assert np.array_equal(got, gpu_softmax(scores, p, table, n_w * heads * 49))
    assert np.array_equal(got, ref.softmax_i32_windowed(scores, p, bias, heads * 49, mask, heads))


def test_windowed_general_values_full_mask_rows_and_no_bias():
    """Finite mask values are ordinary addends; a query whose every key is masked yields the
    zero-point although its scores are positive; a mask without a bias is served too."""
    rng = np.random.default_rng(6)
    heads, t, n_w, images = 2, 49, 5, 4
    rows = images * n_w * heads * t
    scores = np.abs(np.rint(rng.standard_normal((rows, t)) * 300)).astype(np.int32) + 1
    bias = np.rint(rng.standard_normal((heads * t, t)) * 8).astype(np.int32)
    bias[rng.random(bias.shape) < 0.02] = INT32_MIN
    mask = np.where(rng.random((n_w, t, t)) < 0.3, INT32_MIN, 0).astype(np.int32)
    mask[1] = np.rint(rng.standard_normal((t, t)) * 200).astype(np.int32)       # additive, finite
    mask[2, 5, :] = INT32_MIN                                                    # fully masked query
    mask[4, :, :] = INT32_MIN + 1                                                # huge but finite
    p = prepare.softmax_prepare(2.0 ** -6, t, 1)
    p.post = ref.Dyadic(1, 0, 3, 0, 255)
    want = ref.softmax_i32_windowed(scores, p, bias, heads * t, mask, heads)
    r = ((0 * n_w + 2) * heads + 1) * t + 5
    assert want[r].tolist() == [3] * t
    for algo in (0, 1):
        assert np.array_equal(gpu_softmax_windowed(scores, p, bias, heads * t, mask, heads, algo=algo), want)
    want = ref.softmax_i32_windowed(scores, p, None, 0, mask, heads)
    assert np.array_equal(gpu_softmax_windowed(scores, p, None, 0, mask, heads), want)
    # bias only through the same entry point
    want = ref.softmax_i32_windowed(scores, p, bias, heads * t, None, heads)
    assert np.array_equal(gpu_softmax_windowed(scores, p, bias, heads * t, None, heads), want)


def test_windowed_12x12_windows():
    rng = np.random.default_rng(8)
    heads = 3
    scores, bias, mask = _case(rng, 2, 48, heads, win=12, shift=6, drop=7, spread=300.0)
    assert mask.shape == (16, 144, 144)
    p = prepare.softmax_prepare(2.0 ** -6, 144, 1)
    want = ref.softmax_i32_windowed(scores, p, bias, heads * 144, mask, heads)
    assert np.array_equal(gpu_softmax_windowed(scores, p, bias, heads * 144, mask, heads), want)
    # the same mask one bit per key: three words per query, in the slab kernel and the three-pass one
    bits = ref.pack_window_mask(mask)
    assert bits.shape == (16, 144, 3)
    for algo in (0, 1):
        assert np.array_equal(gpu_softmax_windowed_bits(scores, p, bias, heads * 144, bits, heads, algo=algo), want), algo


@pytest.mark.parametrize("heads", [4, 3])
def test_windowed_bits_12x12_dense_masks(heads):
    """144-token windows with random masks (bits in all three words at every lane offset), masked
    scores, a fully masked query, both variants and output types, a ragged row count."""
    rng = np.random.default_rng(80 + heads)
    t, n_w = 144, 3
    rows = 3 * n_w * heads * t - 5
    scores = np.rint(rng.standard_normal((rows, t)) * 300).astype(np.int32)
    scores[rng.random(scores.shape) < 0.01] = INT32_MIN
    bias = np.rint(rng.standard_normal((heads * t, t)) * 8).astype(np.int32)
    mask = np.where(rng.random((n_w, t, t)) < 0.4, INT32_MIN, 0).astype(np.int32)
    mask[1, 7, :] = INT32_MIN
    mask[2, :, :] = 0
    mask[2, np.arange(t), (np.arange(t) * 5) % t] = INT32_MIN
    bits = ref.pack_window_mask(mask)
    dirty = bits.copy()
    dirty[:, :, 2] |= np.uint64(0xFFFFFFFFFFFF0000)          # bits 144..191: no such keys
    for variant, signed in ((1, 0), (0, 1), (2, 0)):
        p = prepare.softmax_prepare(2.0 ** -6.5, t, variant, signed)
        want = ref.softmax_i32_windowed(scores, p, bias, heads * t, mask, heads)
        for b in (bits, dirty):
            assert np.array_equal(gpu_softmax_windowed_bits(scores, p, bias, heads * t, b, heads), want), (variant, signed)


def test_windowed_other_row_length_takes_the_three_pass_kernel():
    rng = np.random.default_rng(9)
    t, heads, n_w = 16, 2, 3
    rows = 4 * n_w * heads * t
    scores = np.rint(rng.standard_normal((rows, t)) * 300).astype(np.int32)
    bias = np.rint(rng.standard_normal((heads * t, t)) * 8).astype(np.int32)
    mask = np.where(rng.random((n_w, t, t)) < 0.3, INT32_MIN, 0).astype(np.int32)
    p = prepare.softmax_prepare(2.0 ** -6, t, 0)
    want = ref.softmax_i32_windowed(scores, p, bias, heads * t, mask, heads)
    assert np.array_equal(gpu_softmax_windowed(scores, p, bias, heads * t, mask, heads), want)


@pytest.mark.parametrize("stage", [0, 1, 2])
def test_windowed_swin_b_full_size(stage):
    """Swin-B at batch 64, shifted-window blocks of stages 1-3 (64, 16 and 4 windows per image),
    the benchmark's score generator, one launch."""
    import torch
    import paper_2511_15369_amd as ip
    case = workloads.softmax_case("swin_b", stage)
    heads = workloads.CONFIGS["swin_b"]["heads"][stage]
    side = workloads.SWIN_B_MAP_SIDE[stage]
    mask = workloads.shifted_window_mask(side, side)
    assert mask.shape[0] == workloads.CONFIGS["swin_b"]["windows"][stage]
    rows, cols = case.scores.shape
    for variant in (1, 0):
        p = prepare.softmax_prepare(case.s_delta, cols, variant)
        want = ref.softmax_i32_windowed(case.scores, p, case.bias, case.bias_period_rows, mask, heads)
        got = gpu_softmax_windowed(case.scores, p, case.bias, case.bias_period_rows, mask, heads)
        assert np.array_equal(got, want), (stage, variant)
    # the batched entry point carries the mask too
    d_s = torch.from_numpy(case.scores).cuda()
    d_b = torch.from_numpy(case.bias).cuda()
    d_m = torch.from_numpy(mask).cuda()
    d_o = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
    prob = ip.softmax_problem(d_s, d_b, case.bias_period_rows, d_o, rows, cols, lib_softmax(p), d_m, mask.shape[0], heads)
    ip.softmax_i32_batch([prob], 1, cols)
    torch.cuda.synchronize()
    assert np.array_equal(d_o.cpu().numpy(), want)


@pytest.mark.parametrize("n_w,cols", [(4, 49), (3, 7), (2, 64), (2, 65), (1, 144), (5, 130), (1, 1)])
def test_pack_window_mask_matches_the_oracle(n_w, cols):
    """The packing kernel against the oracle's plain loops: one, two and three words per query,
    finite entries and INT32_MIN + 1 count as "not masked", the buffer's other bytes stay."""
    rng = np.random.default_rng(n_w * 1000 + cols)
    mask = np.where(rng.random((n_w, cols, cols)) < 0.4, INT32_MIN, 0).astype(np.int32)
    mask[rng.random(mask.shape) < 0.05] = INT32_MIN + 1
    mask[rng.random(mask.shape) < 0.05] = -5
    _, got = gpu_pack_window_mask(mask)
    assert np.array_equal(got, ref.pack_window_mask(mask))


@pytest.mark.parametrize("heads,side", [(4, 14), (3, 14), (8, 21), (1, 14), (6, 28)])
@pytest.mark.parametrize("variant", [0, 1, 2])
def test_windowed_bits_small(heads, side, variant):
    """The mask one bit per key on the slab route (49 keys, with a bias) and the three-pass route:
    ragged row counts, masked scores, both output types; bits beyond the row length are ignored."""
    rng = np.random.default_rng(heads * 1000 + side * 10 + variant + 7)
    scores, bias, mask = _case(rng, 3, side, heads, drop=int(rng.integers(0, 40)))
    scores[rng.random(scores.shape) < 0.01] = INT32_MIN
    bits = ref.pack_window_mask(mask)
    dirty = bits | np.uint64(0xFFFE000000000000)            # bits 49..63 set: no such keys
    for signed in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -6.5, 49, variant, signed)
        want = ref.softmax_i32_windowed_bits(scores, p, bias, heads * 49, bits, heads)
        for algo in (0, 1):
            for b in (bits, dirty):
                got = gpu_softmax_windowed_bits(scores, p, bias, heads * 49, b, heads, algo=algo)
                assert np.array_equal(got, want), (heads, side, variant, signed, algo)


def test_windowed_bits_dense_random_masks_full_rows_and_no_bias():
    """Random masks (every bit position used, at every lane offset), a query whose every key is
    masked although its scores are positive, a mask without a bias, other row lengths with one
    and with three words per query (three-pass kernel)."""
    rng = np.random.default_rng(16)
    heads, t, n_w, images = 2, 49, 5, 4
    rows = images * n_w * heads * t - 13
    scores = np.abs(np.rint(rng.standard_normal((rows, t)) * 300)).astype(np.int32) + 1
    bias = np.rint(rng.standard_normal((heads * t, t)) * 8).astype(np.int32)
    bias[rng.random(bias.shape) < 0.02] = INT32_MIN
    mask = np.where(rng.random((n_w, t, t)) < 0.5, INT32_MIN, 0).astype(np.int32)
    mask[2, 5, :] = INT32_MIN
    mask[3, :, :] = 0
    mask[3, np.arange(t), np.arange(t)] = INT32_MIN         # one key per query, a different one each
    bits = ref.pack_window_mask(mask)
    for variant in (0, 1):
        p = prepare.softmax_prepare(2.0 ** -6, t, variant)
        p.post = ref.Dyadic(1, 0, 3, 0, 255)
        want = ref.softmax_i32_windowed(scores, p, bias, heads * t, mask, heads)
        r = ((0 * n_w + 2) * heads + 1) * t + 5
        assert want[r].tolist() == [3] * t
        for algo in (0, 1):
            assert np.array_equal(gpu_softmax_windowed_bits(scores, p, bias, heads * t, bits, heads, algo=algo), want)
        want = ref.softmax_i32_windowed(scores, p, None, 0, mask, heads)
        assert np.array_equal(gpu_softmax_windowed_bits(scores, p, None, 0, bits, heads), want)
    for t2 in (16, 144, 130):
        rows2 = 2 * 3 * heads * t2 - 5
        sc = np.rint(rng.standard_normal((rows2, t2)) * 300).astype(np.int32)
        bi = np.rint(rng.standard_normal((heads * t2, t2)) * 8).astype(np.int32)
        mk = np.where(rng.random((3, t2, t2)) < 0.3, INT32_MIN, 0).astype(np.int32)
        p = prepare.softmax_prepare(2.0 ** -6, t2, 1)
        want = ref.softmax_i32_windowed(sc, p, bi, heads * t2, mk, heads)
        assert np.array_equal(gpu_softmax_windowed_bits(sc, p, bi, heads * t2, ref.pack_window_mask(mk), heads), want), t2


@pytest.mark.parametrize("stage", [0, 1, 2])
def test_windowed_bits_swin_b_full_size(stage):
    """Swin-B at batch 64, shifted-window blocks of stages 1-3, the mask packed by the library:
    the launch the benchmark times, and the batched entry point."""
    import torch
    import paper_2511_15369_amd as ip
    case = workloads.softmax_case("swin_b", stage)
    heads = workloads.CONFIGS["swin_b"]["heads"][stage]
    side = workloads.SWIN_B_MAP_SIDE[stage]
    mask = workloads.shifted_window_mask(side, side)
    rows, cols = case.scores.shape
    d_bits, host_bits = gpu_pack_window_mask(mask)
    assert np.array_equal(host_bits, ref.pack_window_mask(mask))
    d_s = torch.from_numpy(case.scores).cuda()
    d_b = torch.from_numpy(case.bias).cuda()
    for variant in (1, 0):
        p = prepare.softmax_prepare(case.s_delta, cols, variant)
        want = ref.softmax_i32_windowed(case.scores, p, case.bias, case.bias_period_rows, mask, heads)
        d_o = torch.full((rows, cols), 0x5A, dtype=torch.uint8, device="cuda")
        ip.softmax_i32_windowed_bits(d_s, d_b, case.bias_period_rows, d_bits, mask.shape[0], heads, d_o, rows, cols,
                                     lib_softmax(p))
        torch.cuda.synchronize()
        assert np.array_equal(d_o.cpu().numpy(), want), (stage, variant)
    d_o = torch.full((rows, cols), 0x5A, dtype=torch.uint8, device="cuda")
    prob = ip.softmax_problem(d_s, d_b, case.bias_period_rows, d_o, rows, cols, lib_softmax(p), None, mask.shape[0],
                              heads, d_bits)
    ip.softmax_i32_batch([prob], 1, cols)
    torch.cuda.synchronize()
    assert np.array_equal(d_o.cpu().numpy(), want)


def test_windowed_bits_argument_checks():
    import ctypes
    import torch
    import paper_2511_15369_amd as ip
    t = 49
    d_s = torch.zeros((98, t), dtype=torch.int32, device="cuda")
    d_o = torch.zeros((98, t), dtype=torch.uint8, device="cuda")
    d_m = torch.zeros((2, t, t), dtype=torch.int32, device="cuda")
    d_w = torch.zeros((2, t, 1), dtype=torch.int64, device="cuda")
    p = lib_softmax(prepare.softmax_prepare(2.0 ** -6, t, 1))
    lib = ip.load()
    fn = lib.iptq_softmax_i32_windowed_bits
    for n_w, heads in ((0, 1), (1, 0), (-1, 1), (2 ** 30, 4)):
        rc = fn(d_s.data_ptr(), None, 0, d_w.data_ptr(), n_w, heads, d_o.data_ptr(), 98, t, ctypes.byref(p), None)
        assert rc == -2, (n_w, heads)
    rc = fn(d_s.data_ptr(), None, 0, d_w.data_ptr() + 4, 2, 1, d_o.data_ptr(), 98, t, ctypes.byref(p), None)
    assert rc == -6                                          # words are 8-byte aligned
    # both forms of the mask in one problem of a batch: refused
    prob = ip.softmax_problem(d_s, None, 0, d_o, 98, t, p, d_m, 2, 1, d_w)
    arr = (ip.SoftmaxProblem * 1)(prob)
    assert lib.iptq_softmax_i32_batch(arr, 1, t, None) == -3
    pk = lib.iptq_pack_window_mask
    assert pk(d_m.data_ptr(), -1, t, d_w.data_ptr(), None) == -2
    assert pk(d_m.data_ptr(), 2, 0, d_w.data_ptr(), None) == -2
    assert pk(None, 2, t, d_w.data_ptr(), None) == -1
    assert pk(d_m.data_ptr(), 2, t, d_m.data_ptr(), None) == -3           # overlap
    assert pk(d_m.data_ptr(), 0, t, None, None) == 0
    torch.cuda.synchronize()
    assert not d_o.any() and not d_w.any()                   # nothing was launched


def test_windowed_argument_checks():
    import ctypes
    import torch
    import paper_2511_15369_amd as ip
    t = 49
    d_s = torch.zeros((98, t), dtype=torch.int32, device="cuda")
    d_o = torch.zeros((98, t), dtype=torch.uint8, device="cuda")
    d_m = torch.zeros((2, t, t), dtype=torch.int32, device="cuda")
    p = lib_softmax(prepare.softmax_prepare(2.0 ** -6, t, 1))
    fn = ip.load().iptq_softmax_i32_windowed
    for n_w, heads in ((0, 1), (1, 0), (-1, 1), (2 ** 30, 4)):
        rc = fn(d_s.data_ptr(), None, 0, d_m.data_ptr(), n_w, heads, d_o.data_ptr(), 98, t, ctypes.byref(p), None)
        assert rc == -2, (n_w, heads)
    torch.cuda.synchronize()
    assert not d_o.any()                                     # nothing was launched


def test_windowed_calls_in_a_hip_graph_and_on_views_off_the_16_byte_grid():
    """The packing call and both windowed softmax forms captured once in a HIP graph and replayed
    with fresh scores and a fresh mask each time (eager copies and synchronisations between the
    replays); the score and output tensors are views that start one element off the 16-byte grid."""
    import torch
    import paper_2511_15369_amd as ip
    rng = np.random.default_rng(21)
    heads, t, side = 4, 49, 14
    mask0 = workloads.shifted_window_mask(side, side)
    n_w = mask0.shape[0]
    rows = 6 * n_w * heads * t - 9
    bias = np.rint(rng.standard_normal((heads * t, t)) * 8).astype(np.int32)
    p = prepare.softmax_prepare(2.0 ** -6.5, t, 1)
    lp = lib_softmax(p)
    buf_s = torch.zeros(rows * t + 8, dtype=torch.int32, device="cuda")
    d_s = buf_s[1:1 + rows * t].view(rows, t)              # 4 bytes off the 16-byte grid
    d_b = torch.from_numpy(bias).cuda()
    d_m = torch.from_numpy(mask0.copy()).cuda()
    d_w = torch.zeros((n_w, t, 1), dtype=torch.int64, device="cuda")
    buf_a = torch.zeros(rows * t + 32, dtype=torch.uint8, device="cuda")
    buf_b = torch.zeros(rows * t + 32, dtype=torch.uint8, device="cuda")
    d_a = buf_a[1:1 + rows * t].view(rows, t)               # one byte off
    d_o = buf_b[3:3 + rows * t].view(rows, t)

    def work():
        ip.pack_window_mask(d_m, n_w, t, d_w)
        ip.softmax_i32_windowed_bits(d_s, d_b, heads * t, d_w, n_w, heads, d_a, rows, t, lp)
        ip.softmax_i32_windowed(d_s, d_b, heads * t, d_m, n_w, heads, d_o, rows, t, lp)

    side_stream = torch.cuda.Stream()
    side_stream.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side_stream):
        work()
    torch.cuda.current_stream().wait_stream(side_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        work()
    for rep in range(4):
        scores = np.rint(rng.standard_normal((rows, t)) * (200 + 400 * rep)).astype(np.int32)
        mask = np.where(rng.random((n_w, t, t)) < 0.1 * (rep + 1), INT32_MIN, 0).astype(np.int32)
        d_s.copy_(torch.from_numpy(scores))
        d_m.copy_(torch.from_numpy(mask))
        buf_a.fill_(0x5A)
        buf_b.fill_(0x5A)
        d_w.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = ref.softmax_i32_windowed(scores, p, bias, heads * t, mask, heads)
        assert np.array_equal(d_w.cpu().numpy().view(np.uint64), ref.pack_window_mask(mask)), rep
        assert np.array_equal(d_a.cpu().numpy(), want), rep
        assert np.array_equal(d_o.cpu().numpy(), want), rep
        for buf, off in ((buf_a, 1), (buf_b, 3)):          # nothing written around the views
            host = buf.cpu().numpy()
            assert (host[:off] == 0x5A).all() and (host[off + rows * t:] == 0x5A).all(), rep
