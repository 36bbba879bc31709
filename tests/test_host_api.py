"""CPU-side checks of the HIP library: it loads, exports what the header declares, rejects
bad arguments before touching the GPU, derives the same constants as the oracle, and its
integer helpers (compiled for the host from the kernels' own source) are exact."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2511_15369_amd as ip
from oracle import prepare, ref
from tests.helpers import gelu_fields, lib_gelu, lib_softmax, softmax_fields

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    lib = ip.load()
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):      # iptq.h and the test hooks' header
        header = open(os.path.join(ROOT, "include", h)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        names |= set(re.findall(r"\b(iptq_[a-z0-9_]+)\s*\(", header))
    assert any(n.startswith("iptq_debug_") for n in names)
    assert {"iptq_softmax_i32", "iptq_gelu_i8", "iptq_gelu_i32", "iptq_requant",
            "iptq_softmax_i32_layers", "iptq_gelu_i8_layers", "iptq_make_dyadic",
            "iptq_softmax_prepare", "iptq_gelu_prepare", "iptq_strerror",
            "iptq_version"} <= names
    for n in names:
        assert hasattr(lib, n), n
    assert ip.version() >= 100
    assert "NULL" in ip.strerror(-1) and ip.strerror(0) == "ok"


def test_prepare_matches_the_oracles_derivation():
    rng = np.random.default_rng(0)
    for _ in range(300):
        s = float(2.0 ** rng.uniform(-12, -4))
        cols = int(rng.integers(1, 2000))
        variant = int(rng.integers(0, 2))
        signed = int(rng.integers(0, 2))
        assert softmax_fields(ip.softmax_prepare(s, cols, variant, signed)) == \
            softmax_fields(prepare.softmax_prepare(s, cols, variant, signed))
        s_in = float(2.0 ** rng.uniform(-12, -3))
        s_out = float(2.0 ** rng.uniform(-12, -3))
        zi, zo = int(rng.integers(-128, 128)), int(rng.integers(-128, 128))
        maxq = int(rng.choice([128, 255, 1000, 70000]))
        a = ip.gelu_prepare(s_in, s_out, zi, zo, variant, maxq)
        b = prepare.gelu_prepare(s_in, s_out, zi, zo, variant, maxq)
        assert gelu_fields(a) == gelu_fields(b)
    for r in [1.0, -1.0, 0.3, 2.0 ** -40, 3e4, -7.7e-7, 2.0 ** -70]:
        assert ip.make_dyadic(r) == prepare.make_dyadic(r)
    with pytest.raises(ip.IptqError):
        ip.make_dyadic(1e6)
    with pytest.raises(ip.IptqError):
        ip.make_dyadic(0.0)


def test_floor_pow2_div_is_exact():
    f = ip.load().iptq_debug_floor_pow2_div
    f.restype = ctypes.c_uint32
    f.argtypes = [ctypes.c_int32, ctypes.c_uint32]
    rng = np.random.default_rng(1)
    for m in (7, 8, 15, 24, 30, 31):
        top = 1 << m
        sig = set(range(1, min(top, 5000) + 1))
        sig |= {top, top - 1, top // 2, top // 2 + 1, top // 3, top // 3 + 1}
        sig |= {1 << k for k in range(m + 1)} | {(1 << k) - 1 for k in range(1, m + 1)}
        sig |= {(1 << k) + 1 for k in range(m)}
        sig |= set(int(v) for v in rng.integers(1, top + 1, size=20000))
        for s in sig:
            if 1 <= s <= top:
                assert f(m, s) == top // s, (m, s)
    assert f(30, 0) == 0


def _plan(p, rows, cols, has_bias=0, period=0):
    fn = ip.load().iptq_debug_softmax_plan
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.POINTER(ip.SoftmaxParams), ctypes.c_int64, ctypes.c_int32, ctypes.c_int32,
                   ctypes.c_int64, ctypes.POINTER(ctypes.c_int64)]
    out = (ctypes.c_int64 * 12)()
    rc = fn(ctypes.byref(p), rows, cols, has_bias, period, out)
    return rc, list(out)


@pytest.mark.parametrize("i0,n", [(16, 0), (17, 3), (64, 8), (128, 7), (181, 7), (255, 7), (257, 6),
                                  (1000, 5), (4097, 2), (65535, 0), (2 ** 24 - 1, 0), (2 ** 20, 3)])
def test_softmax_plan_divider_and_clamp(i0, n):
    p = lib_softmax(ref.SoftmaxParams(variant=1, i0=i0, n_shift=n))
    rc, o = _plan(p, 10, 3)
    assert rc == 0
    magic, sh, D, i0n, p_shift, _, _, n_max = o[:8]
    assert i0n == i0 << n and p_shift == 23
    # the divider is exact on the whole reachable range (sampled densely for large i0)
    step = max(1, n_max // 200000)
    ns = np.arange(0, n_max + 1, step, dtype=np.uint64)
    edge = np.array([k * i0 + d for k in range(0, n_max // i0 + 2) for d in (-1, 0, 1)], np.int64)
    ns = np.concatenate([ns, edge[(edge >= 0) & (edge <= n_max)].astype(np.uint64)])
    got = ((ns * np.uint64(magic)) >> np.uint64(32)) >> np.uint64(sh)
    assert np.array_equal(got, ns // np.uint64(i0))
    # at and beyond the clamp the oracle's exponential is zero; just inside it may not be
    for variant in (0, 1):
        op = ref.SoftmaxParams(variant=variant, i0=i0, n_shift=n)
        assert ref.bit_exp(-D, op) == 0 and ref.bit_exp(-D - 1, op) == 0
        assert ref.bit_exp(-(2 ** 30), op) == 0
    assert n_max // i0 <= 31


def test_packed_path_divider_is_exact_wherever_it_is_enabled():
    """Every i0 of the usual scale range: when the plan enables the packed 16-bit path, its
    24-bit divider must give n div i0 for every reachable n, and all values must fit."""
    enabled = 0
    for i0 in list(range(16, 3400)) + [4000, 5000, 2 ** 14, 2 ** 15 - 1]:
        for n_shift in {max(0, 15 - i0.bit_length()), 0}:
            p = lib_softmax(ref.SoftmaxParams(variant=1, i0=i0, n_shift=n_shift))
            rc, o = _plan(p, 10, 49)
            assert rc == 0
            D, n_max, mode, mg24, t16 = o[2], o[7], o[8], o[9], o[10]
            if mode == 0:
                continue
            enabled += 1
            assert mode == (1 if t16 == 0 else 2)
            assert D <= 32767 and (n_max << t16) <= 65535 and mg24 < 2 ** 24 and (i0 << n_shift) < 2 ** 15
            n = np.arange(0, n_max + 1, dtype=np.uint64)
            q = ((n << np.uint64(t16)) * np.uint64(mg24)) >> np.uint64(32)
            assert np.array_equal(q, n // np.uint64(i0)), i0
            assert int(q.max()) <= 15
    assert enabled > 3000
    # default parameters of the whole benchmark scale range take the packed path
    for log2s in np.linspace(-10, -4, 25):
        p = ip.softmax_prepare(float(2.0 ** log2s), 197, 1, 0)
        rc, o = _plan(p, 10, 197)
        assert rc == 0 and o[8] in (1, 2)


def test_bias_period_divider():
    p = lib_softmax(ref.SoftmaxParams())
    for period in (2, 3, 49, 196, 392, 1568, 1000003, 2 ** 31 - 1):
        rc, o = _plan(p, 100, 49, 1, period)
        assert rc == 0
        magic, sh = o[5], o[6]
        rows = np.concatenate([np.arange(0, 5000), np.array([2 ** 31 - 1, 2 ** 31 - 2, period - 1,
                               period, period + 1, 7 * period - 1, 7 * period])]).astype(np.uint64)
        rows = rows[rows < 2 ** 31]
        got = ((rows * np.uint64(magic)) >> np.uint64(32)) >> np.uint64(sh)
        assert np.array_equal(got, rows // np.uint64(period))


def _softmax_rc(p, rows=0, cols=4, scores=None, out=None, bias=None, period=0):
    return ip.load().iptq_softmax_i32(scores, bias, period, out, rows, cols, ctypes.byref(p), None)


def test_softmax_argument_errors_without_a_gpu():
    good = lib_softmax(ref.SoftmaxParams())
    assert _softmax_rc(good, rows=0) == 0                     # empty input is a no-op
    assert ip.load().iptq_softmax_i32(None, None, 0, None, 0, 4, None, None) == -1
    assert _softmax_rc(good, rows=5) == -1                    # data pointers missing
    assert _softmax_rc(good, rows=-1) == -2
    assert _softmax_rc(good, rows=2 ** 31) == -2
    assert _softmax_rc(good, cols=0) == -2
    assert _softmax_rc(good, cols=65537) == -2
    assert _softmax_rc(good, rows=0, bias=ctypes.c_void_p(16), period=0) == -2
    for field, val in (("variant", 3), ("variant", -1), ("i0", 15), ("i0", 2 ** 24), ("n_shift", -1), ("n_shift", 21),
                       ("out_bits", 1), ("out_bits", 9), ("m_bits", 32), ("m_bits", 6), ("pre_m", 0),
                       ("pre_m", 32768), ("pre_s", 63), ("out_is_signed", 2), ("algo", 7)):
        bad = lib_softmax(ref.SoftmaxParams())
        setattr(bad, field, val)
        assert _softmax_rc(bad) == -3, field
    bad = lib_softmax(ref.SoftmaxParams(i0=2 ** 20, n_shift=4))
    assert _softmax_rc(bad) == -3                             # i0 << N >= 2^24
    bad = lib_softmax(ref.SoftmaxParams(post=ref.Dyadic(1, 0, 0, -1, 255)))
    assert _softmax_rc(bad) == -3                             # qmin outside uint8
    bad = lib_softmax(ref.SoftmaxParams(variant=2, i0=2 ** 16, n_shift=0))
    assert _softmax_rc(bad) == -4                             # the second-degree form needs i0 < 2^16
    assert _softmax_rc(lib_softmax(ref.SoftmaxParams(variant=2, i0=2 ** 16 - 1, n_shift=0))) == 0
    wnd = ip.load().iptq_softmax_i32_windowed
    m = ctypes.c_void_p(64)
    assert wnd(None, None, 0, m, 4, 2, None, 0, 49, ctypes.byref(good), None) == 0      # no rows: a no-op
    assert wnd(None, None, 0, m, 0, 2, None, 0, 49, ctypes.byref(good), None) == -2
    assert wnd(None, None, 0, m, 4, 0, None, 0, 49, ctypes.byref(good), None) == -2
    assert wnd(None, None, 0, m, 2 ** 20, 2 ** 10, None, 0, 49, ctypes.byref(good), None) == -2
    assert wnd(None, None, 0, ctypes.c_void_p(66), 4, 2, None, 0, 49, ctypes.byref(good), None) == -6
    assert wnd(None, None, 0, None, 0, 0, None, 0, 49, ctypes.byref(good), None) == 0    # no mask: plain call
    bad = lib_softmax(ref.SoftmaxParams(i0=2 ** 14, n_shift=9, m_bits=24))
    assert _softmax_rc(bad, cols=4) == -4                     # cols * (i0 << N) > 2^M
    assert _softmax_rc(good, rows=3, scores=ctypes.c_void_p(6), out=ctypes.c_void_p(64)) == -6
    assert _softmax_rc(good, rows=3, scores=ctypes.c_void_p(64), out=ctypes.c_void_p(80)) == -3  # overlap


def test_gelu_and_requant_argument_errors_without_a_gpu():
    lib = ip.load()
    good = lib_gelu(prepare.gelu_prepare(2.0 ** -5, 2.0 ** -5, 0, 0, 1))
    assert lib.iptq_gelu_i8(None, None, 0, ctypes.byref(good), None) == 0
    assert lib.iptq_gelu_i8(None, None, 4, ctypes.byref(good), None) == -1
    assert lib.iptq_gelu_i8(None, None, -4, ctypes.byref(good), None) == -2
    assert lib.iptq_gelu_i8(None, None, 0, None, None) == -1
    for field, val, code in (("variant", 3, -3), ("q_b", 0, -3), ("q_c", 0, -3), ("k", 63, -3),
                             ("k", -1, -3), ("max_abs_q", 0, -3), ("zp_in", 129, -3),
                             ("pre_m", 0, -3), ("algo", 2, -3), ("q_b", -40000, -4), ("k", 0, -4),
                             ("max_abs_q", 2 ** 30, -4)):
        bad = lib_gelu(prepare.gelu_prepare(2.0 ** -5, 2.0 ** -5, 0, 0, 1))
        assert bad.k > 0
        setattr(bad, field, val)
        assert lib.iptq_gelu_i8(None, None, 0, ctypes.byref(bad), None) == code, field
    assert lib.iptq_gelu_i32(ctypes.c_void_p(2), ctypes.c_void_p(64), 4, ctypes.byref(good), None) == -6
    # the range condition uses the ceiling of (|q_b|^p + 2|q_c|) / 2^k: here the floor bound
    # (2147 * 10^6 < 2^31) would pass while v reaches -2148
    edge = ref.GeluParams(1, -13, -140711946, 17, 100, 10 ** 6, 1, 0, ref.Dyadic(18658, 45, -104, -128, 127))
    assert lib.iptq_gelu_i32(None, None, 0, ctypes.byref(lib_gelu(edge)), None) == -4
    edge.k = 18
    assert lib.iptq_gelu_i32(None, None, 0, ctypes.byref(lib_gelu(edge)), None) == 0
    d = ip.Dyadic(1, 0, 0, 0, 255)
    assert lib.iptq_requant(None, None, 0, 0, ctypes.byref(d), None) == 0
    assert lib.iptq_requant(None, None, 3, 0, ctypes.byref(d), None) == -1
    assert lib.iptq_requant(None, None, -3, 0, ctypes.byref(d), None) == -2
    assert lib.iptq_requant(None, None, 0, 2, ctypes.byref(d), None) == -3
    for dd in (ip.Dyadic(32768, 0, 0, 0, 255), ip.Dyadic(1, 63, 0, 0, 255), ip.Dyadic(1, 0, 0, 9, 3),
               ip.Dyadic(1, 0, 0, 0, 256), ip.Dyadic(1, 0, 2 ** 25, 0, 255)):
        assert lib.iptq_requant(None, None, 0, 0, ctypes.byref(dd), None) == -3
    # layer-batched forms validate every layer before launching anything
    arr = (ip.SoftmaxParams * 2)(lib_softmax(ref.SoftmaxParams()), lib_softmax(ref.SoftmaxParams(i0=3)))
    assert lib.iptq_softmax_i32_layers(None, 0, None, 0, 0, 4, 2, arr, None) == -3
    assert lib.iptq_softmax_i32_layers(None, 0, None, 0, 0, 4, -1, arr, None) == -2
    garr = (ip.GeluParams * 1)(good)
    assert lib.iptq_gelu_i8_layers(None, 0, None, 0, 0, 1, garr, None) == 0


def test_batch_argument_errors_without_a_gpu():
    lib = ip.load()
    good = lib_softmax(ref.SoftmaxParams())
    bad = lib_softmax(ref.SoftmaxParams(i0=3))
    arr = (ip.SoftmaxProblem * 2)(ip.SoftmaxProblem(None, None, 0, None, 0, good),
                                  ip.SoftmaxProblem(None, None, 0, None, 0, bad))
    assert lib.iptq_softmax_i32_batch(arr, 1, 49, None) == 0          # empty problems: no-op
    assert lib.iptq_softmax_i32_batch(arr, 2, 49, None) == -3         # second problem is invalid
    assert lib.iptq_softmax_i32_batch(arr, -1, 49, None) == -2
    assert lib.iptq_softmax_i32_batch(arr, 17, 49, None) == -2
    assert lib.iptq_softmax_i32_batch(None, 2, 49, None) == -1
    assert lib.iptq_softmax_i32_batch(None, 0, 49, None) == 0
    arr = (ip.SoftmaxProblem * 1)(ip.SoftmaxProblem(None, None, 0, None, 5, good))
    assert lib.iptq_softmax_i32_batch(arr, 1, 49, None) == -1         # data pointers missing
    g = lib_gelu(prepare.gelu_prepare(2.0 ** -5, 2.0 ** -5, 0, 0, 1))
    garr = (ip.GeluProblem * 2)(ip.GeluProblem(None, None, 0, g), ip.GeluProblem(None, None, 3, g))
    assert lib.iptq_gelu_i8_batch(garr, 1, None) == 0
    assert lib.iptq_gelu_i8_batch(garr, 2, None) == -1
    assert lib.iptq_gelu_i8_batch(garr, 17, None) == -2


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2511_15369_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", os.path.join(ROOT, "no_such_dir", "libiptq.so"))
    with pytest.raises(ImportError):
        b.load()


def test_run_time_row_length_layouts_fit_what_the_kernels_assume():
    """For every row length: the lane layout the host picks for the run-time-row-length
    kernels satisfies what their indexing relies on (blocks per lane within the compiled
    slot count, chunk passes within the unrolled loop, LDS within a workgroup's 64 KB)."""
    import ctypes
    fn = ip.load().iptq_debug_softmax_layout
    fn.argtypes = [ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    fn.restype = ctypes.c_int
    out = (ctypes.c_int32 * 12)()
    served_by_registers = 0
    for cols in list(range(1, 6200)) + [8191, 8192, 13000, 13107, 13108, 20000, 65535, 65536]:
        assert fn(cols, out) == 0
        dyn_ok, k, slots, n_used, wide_ok, passes, wslots, _unused0, _unused1, wg_ok, waves, gslots = list(out)
        # blocks a row can touch at its worst alignment inside a 16-byte grid
        if cols % 4 == 0:
            nb_max = cols // 4
        elif cols % 2 == 0:
            nb_max = (cols + 2 + 3) // 4
        else:
            nb_max = (cols + 3 + 3) // 4
        assert nb_max >= max(((phi + cols + 3) >> 2) for phi in range(0, 4, 4 if cols % 4 == 0 else (2 if cols % 2 == 0 else 1)))
        if dyn_ok:
            assert k in (1, 2, 4, 8, 16) and 1 <= slots <= 10 and (slots <= 8 or k == 16)
            assert (k == 1 or slots >= 5) and n_used == slots    # the layouts that are instantiated
            assert slots == -(-nb_max // k)                  # exactly: the kernel's slot roles rely on it
            nb_min = min(((phi + cols + 3) >> 2) for phi in range(0, 4, 4 if cols % 4 == 0 else (2 if cols % 2 == 0 else 1)))
            assert nb_min >= k * (slots - 1)                 # slots 0 .. slots-2 exist in every row
            rpw = 64 // k
            assert (rpw * cols) % 4 == 0                     # a slab starts on a 16-byte boundary
            in_chunks = rpw * cols // 4
            assert 64 * (slots - 2) < in_chunks <= 64 * slots    # only the last two passes can be short
            wave_lds = ((rpw * cols * 4 + 15) & ~15) + 144
            assert wave_lds <= 65536
        else:
            assert nb_max > 16 * 10
        nb_lo = min(((phi + cols + 3) >> 2) for phi in range(4))     # a row may start anywhere in its block
        if wide_ok:
            assert wslots == passes == -(-nb_max // 64) and 1 <= passes <= 16     # exactly, as for the slab layouts
            assert nb_lo >= 64 * (passes - 1)                # passes 0 .. passes-2 exist in every row
        else:
            assert nb_max > 64 * 16
        if wg_ok:
            assert waves in (4, 8, 16) and gslots == -(-nb_max // (64 * waves))     # exactly
            assert {4: 5, 8: 7, 16: 7}[waves] <= gslots <= {4: 13, 8: 13, 16: 10}[waves] or wide_ok    # instantiated wherever one wavefront per row does not serve
            assert nb_lo >= 64 * waves * (gslots - 1)        # passes 0 .. gslots-2 exist in every row
        else:
            assert nb_max > 512 * 20
        served_by_registers += bool(dyn_ok or wide_ok or wg_ok)
    assert served_by_registers >= 6199
