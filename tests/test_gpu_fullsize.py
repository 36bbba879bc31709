"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The oracle processes about 35 M softmax elements and 110 M GELU elements per second on one
core, so whole layers are compared element by element rather than sampled: one layer of
each ViT-shaped config, every Swin-B stage and the detection-scale Swin-S stage.
"""
import numpy as np
import pytest

import bench
import workloads
from oracle import prepare, ref
from tests.helpers import gelu_fields, softmax_fields

pytestmark = pytest.mark.gpu

FULL_UNITS = [("deit_t", 0), ("vit_s", 4), ("vit_b", 0), ("vit_b", 11), ("swin_b", 0), ("swin_b", 1),
              ("swin_b", 2), ("swin_b", 3), ("swin_s_det", 0)]


@pytest.mark.parametrize("name,unit", FULL_UNITS)
def test_full_size_unit_matches_oracle(name, unit):
    import torch
    print("full-size parity", name, unit, flush=True)
    u = bench.Unit(name, unit)
    u.softmax()
    u.gelu()
    torch.cuda.synchronize()
    probs = u.d_probs.cpu().numpy()
    y = u.d_y.cpu().numpy()

    sc = workloads.softmax_case(name, unit)
    assert sc.scores.shape == (u.rows, u.cols)
    assert np.array_equal(u.d_scores.cpu().numpy(), sc.scores)      # same input on both sides
    p = prepare.softmax_prepare(sc.s_delta, u.cols, sc.variant)
    assert softmax_fields(p) == softmax_fields(u.sp)
    want = ref.softmax_i32(sc.scores, p, sc.bias, sc.bias_period_rows)
    assert np.array_equal(probs, want)

    gc = workloads.gelu_case(name, unit)
    gp = prepare.gelu_prepare(gc.s_in, gc.s_out, gc.zp_in, gc.zp_out, gc.variant)
    assert gelu_fields(gp) == gelu_fields(u.gp)
    assert np.array_equal(y, ref.gelu_i8(gc.x.reshape(-1), gp))


def test_other_variant_at_full_size():
    """The variant the seeded draw did not pick, on the two target shapes."""
    import torch
    for name, unit in (("vit_b", 0), ("swin_b", 0)):
        sc = workloads.softmax_case(name, unit)
        other = 1 - sc.variant
        u = bench.Unit(name, unit, variant_override=other)
        u.softmax()
        u.gelu()
        torch.cuda.synchronize()
        p = prepare.softmax_prepare(sc.s_delta, u.cols, other)
        assert np.array_equal(u.d_probs.cpu().numpy(),
                              ref.softmax_i32(sc.scores, p, sc.bias, sc.bias_period_rows))
        gc = workloads.gelu_case(name, unit)
        gp = prepare.gelu_prepare(gc.s_in, gc.s_out, gc.zp_in, gc.zp_out, other)
        assert np.array_equal(u.d_y.cpu().numpy(), ref.gelu_i8(gc.x.reshape(-1), gp))


@pytest.mark.parametrize("name,unit", [("vit_b", 3), ("swin_b", 0)])
def test_six_bit_and_second_degree_forms_at_full_size(name, unit):
    """The softmax forms the benchmark times beside the default one, on the two target shapes at
    full size: 6-bit probabilities (b = 6 of Eq. 15), the int8 output that clips 128 to 127, the
    signed codes p - 128, and the second-degree Bit-exp."""
    from tests.helpers import gpu_softmax
    sc = workloads.softmax_case(name, unit)
    cols = sc.scores.shape[1]
    forms = []
    p6 = prepare.softmax_prepare(sc.s_delta, cols, sc.variant)
    p6.out_bits = 6
    p6.post = ref.Dyadic(1, 0, 0, 0, 63)
    forms.append(("out_bits 6", p6))
    p6b = prepare.softmax_prepare(sc.s_delta, cols, sc.variant)
    p6b.out_bits, p6b.m_bits = 6, 29                       # the form the benchmark times: M - (b - 1) = 24
    p6b.post = ref.Dyadic(1, 0, 0, 0, 63)
    forms.append(("out_bits 6, M 29", p6b))
    forms.append(("int8 clip", prepare.softmax_prepare(sc.s_delta, cols, sc.variant, 1)))
    ps = prepare.softmax_prepare(sc.s_delta, cols, sc.variant, 1)
    ps.post = ref.Dyadic(1, 0, -128, -128, 127)
    forms.append(("p - 128", ps))
    forms.append(("second degree", prepare.softmax_prepare(sc.s_delta, cols, 2)))
    for what, p in forms:
        print("full-size parity", name, unit, what, flush=True)
        want = ref.softmax_i32(sc.scores, p, sc.bias, sc.bias_period_rows)
        got = gpu_softmax(sc.scores, p, sc.bias, sc.bias_period_rows, algo=4)
        assert np.array_equal(got, want), (name, unit, what)


def test_batched_launch_configuration_at_full_size():
    """bench.py's batched form: the four Swin-B stages through one softmax and one GELU call."""
    import torch
    import paper_2511_15369_amd as ip
    units = bench.build_units("swin_b")
    probs = [ip.softmax_problem(u.d_scores, u.d_bias, u.period, u.d_probs, u.rows, u.cols, u.sp) for u in units]
    gelus = [ip.gelu_problem(u.d_x, u.d_y, u.gelu_n, u.gp) for u in units]
    ip.softmax_i32_batch(probs, len(units), units[0].cols)
    ip.gelu_i8_batch(gelus, len(units))
    torch.cuda.synchronize()
    for i, u in enumerate(units):
        sc = workloads.softmax_case("swin_b", i)
        p = prepare.softmax_prepare(sc.s_delta, u.cols, sc.variant)
        assert np.array_equal(u.d_probs.cpu().numpy(),
                              ref.softmax_i32(sc.scores, p, sc.bias, sc.bias_period_rows)), i
        gc = workloads.gelu_case("swin_b", i)
        gp = prepare.gelu_prepare(gc.s_in, gc.s_out, gc.zp_in, gc.zp_out, gc.variant)
        assert np.array_equal(u.d_y.cpu().numpy(), ref.gelu_i8(gc.x.reshape(-1), gp)), i


def test_batched_vit_b_layers_at_full_size():
    """Two ViT-B layers and a 21-row problem in one call: a launch long enough for the
    steady-state lane layout (the single-layer calls above use the short-launch one), with
    a partial last slab."""
    import torch
    import paper_2511_15369_amd as ip
    units = [bench.Unit("vit_b", 0), bench.Unit("vit_b", 11)]
    small_rows = 21
    d_small = torch.full((small_rows * units[0].cols + 32,), 0x5A, dtype=torch.uint8, device="cuda")
    probs = [ip.softmax_problem(u.d_scores, None, 0, u.d_probs, u.rows, u.cols, u.sp) for u in units]
    probs.append(ip.softmax_problem(units[0].d_scores, None, 0, d_small, small_rows, units[0].cols, units[1].sp))
    ip.softmax_i32_batch(probs, len(probs), units[0].cols)
    torch.cuda.synchronize()
    cases = [workloads.softmax_case("vit_b", 0), workloads.softmax_case("vit_b", 11)]
    for u, sc in zip(units, cases):
        p = prepare.softmax_prepare(sc.s_delta, u.cols, sc.variant)
        assert np.array_equal(u.d_probs.cpu().numpy(), ref.softmax_i32(sc.scores, p))
    p = prepare.softmax_prepare(cases[1].s_delta, units[0].cols, cases[1].variant)
    got = d_small.cpu().numpy()
    n = small_rows * units[0].cols
    assert np.array_equal(got[:n].reshape(small_rows, -1), ref.softmax_i32(cases[0].scores[:small_rows], p))
    assert (got[n:] == 0x5A).all()


@pytest.mark.parametrize("cols", [197, 64, 1025])
def test_softmax_of_more_than_2_31_scores(cols):
    """One call over more than 2^31 scores (64-bit element offsets in every kernel family:
    compiled row length, run-time-length slab, wavefront per row).  The tensor repeats a block
    of 1009 rows (a prime, so slabs meet it at every phase); the whole output is compared on
    the GPU with the oracle's result for that block, repeated."""
    import torch
    import paper_2511_15369_amd as ip
    from tests.helpers import lib_softmax
    block_rows = 1009
    reps = (2 ** 31) // (block_rows * cols) + 1
    rows = block_rows * reps
    assert rows * cols > 2 ** 31
    print("softmax of", rows, "x", cols, flush=True)
    rng = np.random.default_rng(cols)
    base = np.rint(rng.standard_normal((block_rows, cols)) * 900).astype(np.int32)
    base[5, : cols // 2] = -(2 ** 31)
    p = prepare.softmax_prepare(2.0 ** -7.4, cols, 1)
    want = torch.from_numpy(ref.softmax_i32(base, p).reshape(-1)).cuda()
    d_in = torch.from_numpy(base).cuda().repeat(reps, 1)
    d_out = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
    ip.softmax_i32(d_in, None, 0, d_out, rows, cols, lib_softmax(p))
    torch.cuda.synchronize()
    del d_in
    tiles = d_out.view(reps, block_rows * cols)
    for lo in range(0, reps, 512):                   # in pieces: the comparison's temporaries stay small
        assert bool((tiles[lo:lo + 512] == want.view(1, -1)).all()), lo


def test_elementwise_calls_of_more_than_2_31_elements():
    """GELU over more than 2^32 int8 codes and requantization over more than 2^31 int32
    values: periodic inputs (period 1021), the whole output compared with the oracle's period."""
    import torch
    import paper_2511_15369_amd as ip
    from tests.helpers import lib_dyadic, lib_gelu
    period = 1021
    rng = np.random.default_rng(77)

    n = 2 ** 32 + 4099
    pat = rng.integers(-128, 128, size=period, dtype=np.int8)
    gp = prepare.gelu_prepare(2.0 ** -4.6, 2.0 ** -5.1, 3, -4, 1)
    want = torch.from_numpy(ref.gelu_i8(pat, gp)).cuda()
    reps = n // period + 1
    d_x = torch.from_numpy(pat).cuda().repeat(reps)[:n].contiguous()
    d_y = torch.zeros(n, dtype=torch.int8, device="cuda")
    print("gelu of", n, flush=True)
    ip.gelu_i8(d_x, d_y, n, lib_gelu(gp))
    torch.cuda.synchronize()
    del d_x
    full = (n // period) * period
    tiles = d_y[:full].view(-1, period)
    for lo in range(0, tiles.shape[0], 1 << 18):
        assert bool((tiles[lo:lo + (1 << 18)] == want.view(1, -1)).all()), lo
    assert bool((d_y[full:] == want[: n - full]).all())
    del d_y, tiles

    n = 2 ** 31 + 1031
    pat32 = rng.integers(-(2 ** 31), 2 ** 31, size=period).astype(np.int32)
    dy = ref.Dyadic(23170, 38, -3, -128, 127)
    want = torch.from_numpy(ref.requant(pat32, dy, 1)).cuda()
    reps = n // period + 1
    d_x = torch.from_numpy(pat32).cuda().repeat(reps)[:n].contiguous()
    d_y = torch.zeros(n, dtype=torch.int8, device="cuda")
    print("requant of", n, flush=True)
    ip.requant(d_x, d_y, n, 1, lib_dyadic(dy))
    torch.cuda.synchronize()
    del d_x
    full = (n // period) * period
    tiles = d_y[:full].view(-1, period)
    for lo in range(0, tiles.shape[0], 1 << 18):
        assert bool((tiles[lo:lo + (1 << 18)] == want.view(1, -1)).all()), lo
    assert bool((d_y[full:] == want[: n - full]).all())
