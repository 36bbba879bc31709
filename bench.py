#!/usr/bin/env python3
"""Benchmark of the integer softmax + GELU hot path on one MI355X.

A step is one pass of the whole path over one batch of the chosen workload: for every
layer (ViT / DeiT) or stage (Swin), the integer softmax over the int32 attention scores
(with the Swin bias / detection mask where the workload has one) followed by the integer
GELU over the int8 MLP activations, each layer with its own buffers, scales and variant,
one kernel launch per layer and function.  Inputs are seeded synthetic tensors already
resident in HBM when the timed region starts; a workload whose step touches less than
512 MB rotates over several buffer sets, so that nothing is served from the 256 MB
last-level cache.

Prints one JSON line: whole-job elements/s (K steps between two events, with the median and
the minimum of the per-step times beside the mean), the roofline figures of the dominant
kernel (softmax; event timing on the launch stream), both approximation variants of each
function, the other benchmark configurations, and the CPU oracle timed on a bounded sample
of the same workload.
"""
import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# Kernel arguments in device memory (this ROCm's default, stated here so that the figures do not
# depend on the caller's environment; the output records the value in force).  With arguments in
# host memory every kernel starts with a read across the bus: about 3 us per launch, 65 % -> 57 %
# on the Swin-B-shaped step.  Read by the HIP runtime when it starts, so set before torch loads.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E peak
SOFTMAX_BYTES_PER_EL = 5       # int32 in, one byte out
GELU_BYTES_PER_EL = 2          # int8 in, int8 out
CACHE_FLUSH_BYTES = 512e6      # bytes that must be touched before a buffer is used again
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "softmax_gelu_hbm_traffic.md")
KERNEL_SOURCES = ("softmax_rows.h", "device_common.h", "softmax_kernels.hip", "elementwise_kernels.hip")


def kernel_source_hash():
    """Identifies the kernel sources a profile was taken with."""
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2511_15369_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per softmax launch from the tracked rocprofv3 counter summary (lines
    `traffic <workload> <bytes>` under a `kernel-sources <hash>` line), or None when there is no
    figure for this workload or the kernels have changed since it was taken."""
    try:
        text = open(TRAFFIC_PROFILE).read()
    except OSError:
        return None
    m = re.search(r"^\s*kernel-sources\s+([0-9a-f]+)\s*$", text, re.M)
    if not m or m.group(1) != kernel_source_hash():
        return None
    m = re.search(r"^\s*traffic\s+%s\s+([0-9.eE+]+)\s*$" % re.escape(workload), text, re.M)
    return float(m.group(1)) if m else None


class Unit:
    """Device buffers and parameters of one layer / stage (`sets` rotating copies of the buffers)."""

    def __init__(self, name, unit, batch=None, seed=0, variant_override=None, sets=1):
        import torch

        import paper_2511_15369_amd as ip
        import workloads

        cfg = workloads.CONFIGS[name]
        self.name, self.unit = name, unit
        b = cfg["batch"] if batch is None else batch
        heads, tokens, windows = cfg["heads"][unit], cfg["tokens"][unit], cfg["windows"][unit]
        self.heads, self.windows = heads, windows
        sc = workloads.layer_scales(name, unit, seed)
        self.scales = sc

        # scores = Q K^T formed on the GPU in float32 (exact: |sum| < 2^24), then cast
        q, k = workloads.softmax_qk(name, unit, batch, seed)
        dq = torch.from_numpy(q).cuda().float()
        dk = torch.from_numpy(k).cuda().float()
        s = torch.bmm(dq, dk.transpose(1, 2)).to(torch.int32)
        del dq, dk
        if cfg["mask"]:
            km = torch.from_numpy(workloads.detection_key_mask()).cuda()      # [windows, tokens]
            s = s.view(b, windows, heads, tokens, tokens)
            s = torch.where(km[None, :, None, None, :], torch.tensor(-2 ** 31, dtype=torch.int32,
                                                                     device="cuda"), s)
        self.rows, self.cols = b * windows * heads * tokens, tokens
        first = s.reshape(self.rows, self.cols).contiguous()
        self.scores_sets = [first] + [first.clone() for _ in range(sets - 1)]
        bias, period = workloads.softmax_bias(name, unit, seed)
        self.d_bias = None if bias is None else torch.from_numpy(bias).cuda()
        self.period = period
        self.probs_sets = [torch.empty((self.rows, self.cols), dtype=torch.uint8, device="cuda")
                           for _ in range(sets)]

        g = workloads.gelu_case(name, unit, batch, seed)
        self.gelu_case = g
        self.gelu_n = int(g.x.size)
        gx = torch.from_numpy(g.x).cuda().reshape(-1)
        self.x_sets = [gx] + [gx.clone() for _ in range(sets - 1)]
        self.y_sets = [torch.empty_like(gx) for _ in range(sets)]
        self.set_variants(variant_override)
        self.use_set(0)

    def set_variants(self, override=None, softmax_variant=None, gelu_variant=None):
        """Per-unit seeded variants, or `override` for both functions."""
        import paper_2511_15369_amd as ip
        sc, g = self.scales, self.gelu_case
        sv = sc["softmax_variant"] if override is None else override
        gv = sc["gelu_variant"] if override is None else override
        if softmax_variant is not None:
            sv = softmax_variant
        if gelu_variant is not None:
            gv = gelu_variant
        self.sp = ip.softmax_prepare(sc["s_delta"], self.cols, sv, 0)
        self.gp = ip.gelu_prepare(g.s_in, g.s_out, g.zp_in, g.zp_out, gv, 255)

    def use_set(self, i):
        i %= len(self.scores_sets)
        self.d_scores, self.d_probs = self.scores_sets[i], self.probs_sets[i]
        self.d_x, self.d_y = self.x_sets[i], self.y_sets[i]

    def softmax(self):
        import paper_2511_15369_amd as ip
        ip.softmax_i32(self.d_scores, self.d_bias, self.period, self.d_probs, self.rows, self.cols,
                       self.sp)

    def gelu(self):
        import paper_2511_15369_amd as ip
        ip.gelu_i8(self.d_x, self.d_y, self.gelu_n, self.gp)

    @property
    def softmax_elements(self):
        return self.rows * self.cols


def sets_needed(name):
    """Buffer sets so that at least CACHE_FLUSH_BYTES are touched between two uses of a buffer in
    every timed region (the whole step, the softmax launches alone, the GELU launches alone)."""
    import workloads
    cfg = workloads.CONFIGS[name]
    b = cfg["batch"]
    sm = sum(b * cfg["windows"][u] * cfg["heads"][u] * cfg["tokens"][u] ** 2 for u in range(cfg["units"]))
    ge = sum(b * cfg["mlp_tokens"][u] * cfg["mlp_width"][u] for u in range(cfg["units"]))
    least = min(SOFTMAX_BYTES_PER_EL * sm, GELU_BYTES_PER_EL * ge)
    return max(1, min(8, int(CACHE_FLUSH_BYTES // least) + 1))


def build_units(name, batch=None, seed=0, variant_override=None, sets=1):
    import workloads
    return [Unit(name, u, batch, seed, variant_override, sets) for u in range(workloads.CONFIGS[name]["units"])]


MARKERS = False      # --markers: a roctx range around every timed region, named by its leg


def time_steps(fn, reps, before_each=None, leg=None):
    """reps calls of fn() back to back on the launch stream, twice: once between two events (the
    mean: nothing but the calls' own launches sits in the timed region), once with an event after
    every call (median and minimum of the single calls; an event record is a packet of its own on
    the stream and costs a workload of one or two launches per call several per cent).
    Returns (mean ms per call, median ms, min ms).  With --markers both passes sit inside a roctx
    range called `leg`, so that a rocprofv3 run with --kernel-trace --marker-trace can tell which
    launches belong to which line of the output."""
    import torch
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    if MARKERS and leg:
        torch.cuda.nvtx.range_push(leg)
    first.record()
    for i in range(reps):
        if before_each is not None:
            before_each(i)
        fn()
    last.record()
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(reps):
        if before_each is not None:
            before_each(i)
        fn()
        ev[i + 1].record()
    torch.cuda.synchronize()
    if MARKERS and leg:
        torch.cuda.nvtx.range_pop()
    each = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
    return first.elapsed_time(last) / reps, each[len(each) // 2], each[0]


def warm(fn, seconds=0.2):
    """Runs fn() for a while, untimed: after host-side set-up the clocks need some tens of
    milliseconds of work to reach their steady state."""
    import torch
    t_end = time.perf_counter() + seconds
    i = 0
    while time.perf_counter() < t_end:
        fn()
        i += 1
        if i % 8 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()


def time_region(fn, reps, leg=None):
    return time_steps(fn, reps, leg=leg)[0]


def pct(gbps):
    return 100.0 * gbps / HBM_PEAK_GBS


def measure_fused(steps):
    """The requantization fused in front of both layers, on ViT-B-sized tensors: softmax with
    the scores requantized to about 8 bits first (dyadic 20000 / 2^24), and the GELU taking
    int32 accumulators requantized to int8 codes (dyadic 20000 / 2^26, |q| <= 127)."""
    import torch

    import paper_2511_15369_amd as ip
    units = [Unit("vit_b", u) for u in range(4)]
    sps, gps = [], []
    for u in units:
        sp = ip.softmax_prepare(2.0 ** -4, u.cols, u.sp.variant, 0)
        sp.pre_m, sp.pre_s = 20000, 24
        sps.append(sp)
        gp = ip.gelu_prepare(2.0 ** -5, 2.0 ** -5, 0, 0, u.gp.variant, 127)
        gp.pre_m, gp.pre_s = 20000, 26
        gps.append(gp)
    d_y32 = [torch.empty(u.softmax_elements, dtype=torch.int8, device="cuda") for u in units]

    def softmax_pre():
        for u, sp in zip(units, sps):
            ip.softmax_i32(u.d_scores, None, 0, u.d_probs, u.rows, u.cols, sp)

    def gelu_i32():
        for u, gp, y in zip(units, gps, d_y32):
            ip.gelu_i32(u.d_scores.view(-1), y, u.softmax_elements, gp)

    res = {}
    for name, fn in (("softmax_pre_requant", softmax_pre), ("gelu_i32", gelu_i32)):
        warm(fn)
        mean, med, mn = time_steps(fn, steps, leg="fused_requant/" + name)
        el = units[0].softmax_elements
        gb = SOFTMAX_BYTES_PER_EL * el / (mean / len(units) * 1e-3) / 1e9
        res[name] = {"elements": el, "avg_launch_us": mean / len(units) * 1e3,
                     "median_launch_us": med / len(units) * 1e3, "min_launch_us": mn / len(units) * 1e3,
                     "gbps": gb, "pct_of_hbm_peak": pct(gb)}
    del units, d_y32
    return res


def measure_softmax_forms(steps):
    """Other forms of the softmax on the ViT-B layer shape (302,592 x 197; four tensor sets,
    one launch each): int8 output saturating at 127, 6-bit probabilities (W6A6), the
    second-degree exponential, signed codes around the zero-point -128."""
    import torch

    import paper_2511_15369_amd as ip
    units = [Unit("vit_b", u) for u in range(4)]
    el = units[0].softmax_elements
    out_i8 = [torch.empty((u.rows, u.cols), dtype=torch.int8, device="cuda") for u in units]

    def form(kind, u):
        if kind == "int8_saturating":
            return ip.softmax_prepare(u.scales["s_delta"], u.cols, u.sp.variant, 1), True
        if kind == "out_bits_6":
            # b = 6 with M = 29, so that M - (b - 1) = 24 as with the 8-bit default (the packed
            # arithmetic needs the probability in the top byte of a 32-bit product)
            p = ip.softmax_prepare(u.scales["s_delta"], u.cols, u.sp.variant, 0)
            p.out_bits, p.m_bits = 6, 29
            return p, False
        if kind == "second_degree":
            return ip.softmax_prepare(u.scales["s_delta"], u.cols, 2, 0), False
        p = ip.softmax_prepare(u.scales["s_delta"], u.cols, u.sp.variant, 1)     # signed codes p - 128
        p.post = ip.Dyadic(1, 0, -128, -128, 127)
        return p, True

    res = {}
    for kind in ("int8_saturating", "out_bits_6", "second_degree", "signed_zero_point_minus_128"):
        params = [form(kind, u) for u in units]

        def fn():
            for u, (p, signed), o8 in zip(units, params, out_i8):
                ip.softmax_i32(u.d_scores, None, 0, o8 if signed else u.d_probs, u.rows, u.cols, p)

        warm(fn)
        mean, med, mn = time_steps(fn, steps, leg="softmax_forms/" + kind)
        gb = SOFTMAX_BYTES_PER_EL * el / (mean / len(units) * 1e-3) / 1e9
        res[kind] = {"avg_launch_us": mean / len(units) * 1e3, "median_launch_us": med / len(units) * 1e3,
                     "min_launch_us": mn / len(units) * 1e3, "gbps": gb, "pct_of_hbm_peak": pct(gb)}
    del units, out_i8
    return res


def measure_gelu_per_element(steps):
    """The GELU polynomial evaluated per element (IPTQ_ALGO_GENERIC: the arithmetic of Eq. 3 and
    Eq. 5 for every value, no table), ViT-B layer shape, both degrees."""
    import torch

    import paper_2511_15369_amd as ip
    units = [Unit("vit_b", u) for u in range(4)]
    res = {}
    for variant in (0, 1):
        gps = []
        for u in units:
            g = u.gelu_case
            gp = ip.gelu_prepare(g.s_in, g.s_out, g.zp_in, g.zp_out, variant, 255)
            gp.algo = ip.ALGO_GENERIC
            gps.append(gp)

        def fn():
            for u, gp in zip(units, gps):
                ip.gelu_i8(u.d_x, u.d_y, u.gelu_n, gp)

        warm(fn)
        mean, med, mn = time_steps(fn, steps, leg="gelu_per_element/degree_%d" % (2 if variant == 0 else 4))
        gb = GELU_BYTES_PER_EL * units[0].gelu_n / (mean / len(units) * 1e-3) / 1e9
        res["degree_%d" % (2 if variant == 0 else 4)] = {
            "avg_launch_us": mean / len(units) * 1e3, "median_launch_us": med / len(units) * 1e3,
            "min_launch_us": mn / len(units) * 1e3, "gbps": gb, "pct_of_hbm_peak": pct(gb)}
    del units
    return res


def measure_swin_shifted(steps):
    """Swin-B stages 1-3 with the shifted-window mask beside the bias (iptq_softmax_i32_windowed: the
    int32 mask; iptq_softmax_i32_windowed_bits: one bit per key), one launch per stage, four
    tensor sets."""
    import torch

    import paper_2511_15369_amd as ip
    import workloads
    units = [Unit("swin_b", u, sets=4) for u in range(3)]
    masks = [torch.from_numpy(workloads.shifted_window_mask(workloads.SWIN_B_MAP_SIDE[u],
                                                            workloads.SWIN_B_MAP_SIDE[u])).cuda() for u in range(3)]
    packed = []                                       # the same masks one bit per key, packed by the library
    for u, m in zip(units, masks):
        b = torch.empty((u.windows, u.cols, 1), dtype=torch.int64, device="cuda")
        ip.pack_window_mask(m, u.windows, u.cols, b)
        packed.append(b)
    res = {}
    for s, (u, m, mb) in enumerate(zip(units, masks, packed)):
        def fn():
            for k in range(4):
                u.use_set(k)
                ip.softmax_i32_windowed(u.d_scores, u.d_bias, u.period, m, u.windows, u.heads, u.d_probs,
                                        u.rows, u.cols, u.sp)

        def bits():
            for k in range(4):
                u.use_set(k)
                ip.softmax_i32_windowed_bits(u.d_scores, u.d_bias, u.period, mb, u.windows, u.heads, u.d_probs,
                                             u.rows, u.cols, u.sp)

        def plain():
            for k in range(4):
                u.use_set(k)
                u.softmax()

        out = {}
        for name, f in (("bias_and_mask", fn), ("bias_and_mask_bits", bits), ("bias_only", plain)):
            warm(f)
            mean, med, mn = (t / 4 for t in time_steps(f, steps, leg="swin_b_shifted_windows/stage_%d/%s" % (s + 1, name)))
            gb = SOFTMAX_BYTES_PER_EL * u.softmax_elements / (mean * 1e-3) / 1e9
            out[name] = {"avg_launch_us": mean * 1e3, "median_launch_us": med * 1e3, "min_launch_us": mn * 1e3,
                         "gbps": gb, "pct_of_hbm_peak": pct(gb)}
        res["stage_%d" % (s + 1)] = out
    del units, masks, packed
    return res


def measure_row_lengths(steps):
    """Row lengths outside the five benchmark configurations, about 60 M scores per launch
    (a ViT-B layer's worth), four rotating tensor sets: which kernel family serves each and at
    what fraction of the HBM roofline.  Scores round(N(0, 5000)), scale 2^-7, variant 1."""
    import torch

    import paper_2511_15369_amd as ip
    res = {}
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    for cols in (50, 64, 145, 196, 401, 600, 785, 1025, 2048, 4097, 8192, 16384):
        rows = 60_000_000 // cols
        ins = [(torch.randn((rows, cols), device="cuda", generator=gen) * 5000).round().to(torch.int32)
               for _ in range(4)]
        outs = [torch.empty((rows, cols), dtype=torch.uint8, device="cuda") for _ in range(4)]
        sp = ip.softmax_prepare(2.0 ** -7, cols, 1, 0)

        def fn():
            for x, y in zip(ins, outs):
                ip.softmax_i32(x, None, 0, y, rows, cols, sp)

        warm(fn, 0.1)
        ms = time_region(fn, max(1, steps // 2), leg="row_lengths/%d" % cols) / len(ins)
        el = rows * cols
        res[str(cols)] = {"rows": rows, "kernel": ip.softmax_kernel_family(cols),
                          "avg_launch_us": ms * 1e3,
                          "pct_of_hbm_peak": pct(SOFTMAX_BYTES_PER_EL * el / (ms * 1e-3) / 1e9)}
        del ins, outs
    return res


def cpu_baseline(name, budget_units=12):
    """The CPU oracle on the first layers of the same workload: once on one thread, then the
    same calls row-partitioned over every host core (threads; the C calls release the GIL)."""
    from concurrent.futures import ThreadPoolExecutor

    import numpy as np

    import workloads
    from oracle import prepare, ref

    n_units = min(budget_units, workloads.CONFIGS[name]["units"])
    cores = min(os.cpu_count() or 1, 16)          # the GPU machine grants 16 host cores per GPU
    elements, seconds, seconds_all = 0, 0.0, 0.0
    used = 0
    with ThreadPoolExecutor(max_workers=cores) as pool:
        for u in range(n_units):
            sc = workloads.softmax_case(name, u)
            p = prepare.softmax_prepare(sc.s_delta, sc.scores.shape[1], sc.variant)
            gc = workloads.gelu_case(name, u)
            gp = prepare.gelu_prepare(gc.s_in, gc.s_out, gc.zp_in, gc.zp_out, gc.variant)
            gx = gc.x.reshape(-1)
            t0 = time.perf_counter()
            ref.softmax_i32(sc.scores, p, sc.bias, sc.bias_period_rows)
            ref.gelu_i8(gx, gp)
            seconds += time.perf_counter() - t0
            # all cores: row blocks that start on a multiple of the bias period
            period = max(1, sc.bias_period_rows)
            rows = sc.scores.shape[0]
            step = -(-rows // cores)
            step = -(-step // period) * period
            row_jobs = [(r, min(rows, r + step)) for r in range(0, rows, step)]
            el_jobs = np.array_split(np.arange(gx.size), cores)
            t0 = time.perf_counter()
            futs = [pool.submit(ref.softmax_i32, sc.scores[a:b], p, sc.bias, sc.bias_period_rows)
                    for a, b in row_jobs]
            futs += [pool.submit(ref.gelu_i8, gx[j[0]:j[-1] + 1], gp) for j in el_jobs if j.size]
            for f in futs:
                f.result()
            seconds_all += time.perf_counter() - t0
            elements += sc.scores.size + gc.x.size
            used = u + 1
            if seconds + seconds_all > 25.0:
                break
    return {"value": elements / seconds, "unit": "elements/s", "cores": 1, "kind": "oracle",
            "sample": "softmax+GELU of the first %d of %d units of %s, full size, %.1f s"
                      % (used, workloads.CONFIGS[name]["units"], name, seconds),
            "all_cores": {"value": elements / seconds_all, "cores": cores, "seconds": seconds_all}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vit_b",
                    choices=["deit_t", "vit_s", "vit_b", "swin_b", "swin_s_det"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the other benchmark configurations")
    ap.add_argument("--markers", action="store_true",
                    help="a roctx range around every timed region (for rocprofv3 --marker-trace)")
    args = ap.parse_args()
    global MARKERS
    MARKERS = args.markers
    if args.gpus != 1:
        print("bench.py measures one GPU only: softmax rows and GELU elements are independent, so "
              "the path has no multi-GPU form to time (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2511_15369_amd as ip
    import workloads

    ip.load()
    torch.cuda.set_device(0)

    def measure(name, both_variants):
        sets = sets_needed(name)
        units = build_units(name, sets=sets)
        rotate = (lambda i: [u.use_set(i) for u in units]) if sets > 1 else None

        def step():
            for u in units:
                u.softmax()
                u.gelu()

        def softmax_only():
            for u in units:
                u.softmax()

        def gelu_only():
            for u in units:
                u.gelu()

        sm_el = sum(u.softmax_elements for u in units)
        ge_el = sum(u.gelu_n for u in units)
        alg_bytes = SOFTMAX_BYTES_PER_EL * sm_el + GELU_BYTES_PER_EL * ge_el

        def timed():
            # bring the clocks to their steady state first (a few dozen milliseconds of the same
            # work, untimed), then the W warm-up steps, then the K timed ones
            t_end = time.perf_counter() + 0.2
            i = 0
            while time.perf_counter() < t_end:
                if rotate:
                    rotate(i)
                step()
                i += 1
                if i % 8 == 0:
                    torch.cuda.synchronize()
            for i in range(args.warmup):
                if rotate:
                    rotate(i)
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ms, med, mn = time_steps(step, args.steps, rotate, leg=name + "/step")
            wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
            sm = time_steps(softmax_only, args.steps, rotate, leg=name + "/softmax")
            ge = time_steps(gelu_only, args.steps, rotate, leg=name + "/gelu")
            return ms, med, mn, wall_ms, sm, ge

        ms, med, mn, wall_ms, sm_t, ge_t = timed()
        n = len(units)

        def fam(t, el, bpe):
            return {"elements": el, "launches": n, "avg_launch_us": t[0] / n * 1e3,
                    "median_launch_us": t[1] / n * 1e3, "min_launch_us": t[2] / n * 1e3,
                    "gbps": bpe * el / n / (t[0] / n * 1e-3) / 1e9}

        res = {
            "ms_per_step": ms, "median_ms_per_step": med, "min_ms_per_step": mn, "wall_ms_per_step": wall_ms,
            "buffer_sets": sets, "elements_per_step": sm_el + ge_el,
            "softmax": dict(fam(sm_t, sm_el, SOFTMAX_BYTES_PER_EL), rows_per_launch=[u.rows for u in units]),
            "gelu": fam(ge_t, ge_el, GELU_BYTES_PER_EL),
        }
        res["value"] = (sm_el + ge_el) / (ms * 1e-3)
        res["algorithmic_gbps"] = alg_bytes / (ms * 1e-3) / 1e9
        res["median_pct_of_hbm_peak"] = pct(alg_bytes / (med * 1e-3) / 1e9)

        if both_variants:
            # every unit with variant 0 of both functions, then variant 1 (the headline uses the
            # seeded per-unit draw)
            res["variants"] = {}
            for v in (0, 1):
                for u in units:
                    u.set_variants(v)
                step()
                vms, vmed, vmn = time_steps(step, args.steps, rotate, leg="%s/variant_%d/step" % (name, v))
                vsm = time_steps(softmax_only, args.steps, rotate, leg="%s/variant_%d/softmax" % (name, v))
                vge = time_steps(gelu_only, args.steps, rotate, leg="%s/variant_%d/gelu" % (name, v))
                res["variants"]["softmax_%d_gelu_%d" % (v, v)] = {
                    "ms_per_step": vms, "median_ms_per_step": vmed, "min_ms_per_step": vmn,
                    "value": (sm_el + ge_el) / (vms * 1e-3),
                    "pct_of_hbm_peak": pct(alg_bytes / (vms * 1e-3) / 1e9),
                    "softmax_avg_launch_us": vsm[0] / n * 1e3, "softmax_median_launch_us": vsm[1] / n * 1e3,
                    "gelu_avg_launch_us": vge[0] / n * 1e3, "gelu_median_launch_us": vge[1] / n * 1e3}
            for u in units:
                u.set_variants(None)

        # the same work through the batched entry points: one launch per kernel family
        if n <= ip.BATCH_MAX:
            for u in units:
                u.use_set(0)
            sm_probs = (ip.SoftmaxProblem * n)(*[
                ip.softmax_problem(u.d_scores, u.d_bias, u.period, u.d_probs, u.rows, u.cols, u.sp)
                for u in units])
            ge_probs = (ip.GeluProblem * n)(*[ip.gelu_problem(u.d_x, u.d_y, u.gelu_n, u.gp) for u in units])
            cols = units[0].cols

            def step_batched():
                ip.softmax_i32_batch(sm_probs, n, cols)
                ip.gelu_i8_batch(ge_probs, n)

            for _ in range(3):
                step_batched()
            bms = time_region(step_batched, args.steps, leg=name + "/batched/step")
            bsm = time_region(lambda: ip.softmax_i32_batch(sm_probs, n, cols), args.steps, leg=name + "/batched/softmax")
            res["batched"] = {"what": "all units of the workload in one launch per function: a throughput "
                                      "figure, not an inference schedule (the units depend on each other)",
                              "ms_per_step": bms, "value": (sm_el + ge_el) / (bms * 1e-3),
                              "pct_of_hbm_peak": pct(alg_bytes / (bms * 1e-3) / 1e9),
                              "softmax_launch_us": bsm * 1e3,
                              "softmax_gbps": SOFTMAX_BYTES_PER_EL * sm_el / (bsm * 1e-3) / 1e9}
        # the per-unit launch sequence captured once in a HIP graph and replayed (no host work
        # between kernels)
        try:
            for u in units:
                u.use_set(0)
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                step()
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            graph.replay()
            gms = time_region(graph.replay, args.steps, leg=name + "/graph_replay")
            res["graph_replay"] = {"ms_per_step": gms, "value": (sm_el + ge_el) / (gms * 1e-3),
                                   "pct_of_hbm_peak": pct(alg_bytes / (gms * 1e-3) / 1e9)}
            del graph
        except Exception as exc:                      # graphs are an extra, never the headline
            res["graph_replay"] = {"error": str(exc)[:200]}

        # what a plain streaming kernel of the softmax's byte mix (4 B in, 1 B out per element)
        # reaches with the same launch pattern: the library's requantization kernel over every
        # unit's score tensor, one launch per unit
        dy = ip.Dyadic(1, 0, 0, 0, 255)

        def requant_all():
            for u in units:
                ip.requant(u.d_scores.view(-1), u.d_probs.view(-1), u.softmax_elements, 0, dy)

        warm(requant_all, 0.05)
        rq = time_steps(requant_all, max(1, args.steps // 2), rotate, leg=name + "/stream_ceiling")
        res["stream_ceiling"] = {"what": "iptq_requant (int32 -> uint8, the softmax's 5 B/element mix) over the "
                                         "same score tensors, one launch per unit",
                                 "gbps": SOFTMAX_BYTES_PER_EL * sm_el / (rq[0] * 1e-3) / 1e9,
                                 "avg_launch_us": rq[0] / n * 1e3, "median_launch_us": rq[1] / n * 1e3}
        del units
        return res

    main_res = measure(args.workload, both_variants=args.workload in ("vit_b", "swin_b", "swin_s_det"))
    sm = main_res["softmax"]
    cfg = workloads.CONFIGS[args.workload]
    out = {
        "metric": "int softmax+GELU elements/s and achieved HBM GB/s (% of peak), 1xMI355X",
        "value": main_res["value"],
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"],
        "median_ms_per_step": main_res["median_ms_per_step"],
        "min_ms_per_step": main_res["min_ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "%s: %d units x (softmax int32->uint8 + GELU int8->int8), batch %d, "
                               "one launch per unit and function, per-unit scales and variants, seed 0"
                               % (args.workload, cfg["units"], cfg["batch"]),
                   "softmax_elements_per_step": sm["elements"],
                   "gelu_elements_per_step": main_res["gelu"]["elements"],
                   "buffer_sets": main_res["buffer_sets"]},
        "algorithmic_gbps": main_res["algorithmic_gbps"],
        "pct_of_hbm_peak": pct(main_res["algorithmic_gbps"]),
        "median_pct_of_hbm_peak": main_res["median_pct_of_hbm_peak"],
        "roofline": {
            "bound": "hbm",
            # single calls of at most 3072 rows (DeiT-T at batch 1) run one wavefront per row
            "kernel": "softmax_rows_kernel" if min(sm["rows_per_launch"]) > 3072 else "softmax_wide_kernel",
            "achieved": sm["gbps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": sm["gbps"] / HBM_PEAK_GBS,
            "traffic": measured_traffic(args.workload),
            "timing": "events on the launch stream around back-to-back softmax launches (includes the gaps "
                      "between kernels); the rocprofv3 kernel-trace average is in profiles/",
            "avg_launch_us": sm["avg_launch_us"], "median_launch_us": sm["median_launch_us"],
            "min_launch_us": sm["min_launch_us"],
            "algorithmic_bytes_per_launch": SOFTMAX_BYTES_PER_EL * sm["elements"] // sm["launches"],
        },
        "kernel_sources": kernel_source_hash(),
        "hip_force_dev_kernarg": os.environ.get("HIP_FORCE_DEV_KERNARG"),
        "kernels": {"softmax": sm, "gelu": main_res["gelu"]},
        "variants": main_res.get("variants"),
        "stream_ceiling": main_res["stream_ceiling"],
        "batched": main_res.get("batched"),
        "graph_replay": main_res.get("graph_replay"),
    }
    if not args.no_extra:
        # the other benchmark configurations, same protocol, one compact entry each
        out["extra"] = {}
        for name in ("swin_b", "vit_s", "swin_s_det", "deit_t"):
            if name == args.workload:
                continue
            r = measure(name, both_variants=name in ("vit_b", "swin_b", "swin_s_det"))
            e = {k: r[k] for k in ("value", "ms_per_step", "median_ms_per_step", "min_ms_per_step",
                                   "buffer_sets", "algorithmic_gbps", "softmax", "gelu", "stream_ceiling")}
            e["pct_of_hbm_peak"] = pct(r["algorithmic_gbps"])
            e["median_pct_of_hbm_peak"] = r["median_pct_of_hbm_peak"]
            if "variants" in r:
                e["variants"] = r["variants"]
            if name == "swin_b":
                e["batched"] = r.get("batched")
                e["graph_replay"] = r.get("graph_replay")
            elif "batched" in r:
                e["batched_pct_of_hbm_peak"] = r["batched"]["pct_of_hbm_peak"]
            out["extra"][name] = e
        out["extra"]["fused_requant"] = measure_fused(args.steps)
        out["extra"]["softmax_forms"] = measure_softmax_forms(args.steps)
        out["extra"]["gelu_per_element"] = measure_gelu_per_element(args.steps)
        out["extra"]["swin_b_shifted_windows"] = measure_swin_shifted(args.steps)
        out["extra"]["row_lengths"] = measure_row_lengths(args.steps)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
