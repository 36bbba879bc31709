#!/usr/bin/env python3
"""Benchmark of the integer softmax + GELU hot path on one MI355X.

A step is one pass of the whole path over one batch of the chosen workload: for every
layer (ViT / DeiT) or stage (Swin), the integer softmax over the int32 attention scores
(with the Swin bias / detection mask where the workload has one) followed by the integer
GELU over the int8 MLP activations, each layer with its own buffers, scales and variant.
Inputs are seeded synthetic tensors already resident in HBM when the timed region starts.

Prints one JSON line: whole-job elements/s, the roofline figures of the dominant kernel
(softmax; measured live with events on the launch stream) and the CPU oracle timed on a
bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E peak
SOFTMAX_BYTES_PER_EL = 5       # int32 in, one byte out
GELU_BYTES_PER_EL = 2          # int8 in, int8 out
# HBM bytes per softmax launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, keyed by workload (per single-layer / stage-1 launch); None where not measured.
MEASURED_TRAFFIC = {"vit_b": 301.4e6, "swin_b": 197.2e6}


class Unit:
    """Device buffers and parameters of one layer / stage."""

    def __init__(self, name, unit, batch=None, seed=0, variant_override=None):
        import numpy as np
        import torch

        import paper_2511_15369_amd as ip
        import workloads

        cfg = workloads.CONFIGS[name]
        self.name, self.unit = name, unit
        b = cfg["batch"] if batch is None else batch
        heads, tokens, windows = cfg["heads"][unit], cfg["tokens"][unit], cfg["windows"][unit]
        sc = workloads.layer_scales(name, unit, seed)
        self.scales = sc
        sv = sc["softmax_variant"] if variant_override is None else variant_override
        gv = sc["gelu_variant"] if variant_override is None else variant_override

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
        self.d_scores = s.reshape(self.rows, self.cols).contiguous()
        bias, period = workloads.softmax_bias(name, unit, seed)
        self.d_bias = None if bias is None else torch.from_numpy(bias).cuda()
        self.period = period
        self.d_probs = torch.empty((self.rows, self.cols), dtype=torch.uint8, device="cuda")
        self.sp = ip.softmax_prepare(sc["s_delta"], self.cols, sv, 0)

        g = workloads.gelu_case(name, unit, batch, seed)
        self.gelu_n = int(g.x.size)
        self.d_x = torch.from_numpy(g.x).cuda().reshape(-1)
        self.d_y = torch.empty_like(self.d_x)
        self.gp = ip.gelu_prepare(g.s_in, g.s_out, g.zp_in, g.zp_out, gv, 255)
        del np

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


def build_units(name, batch=None, seed=0, variant_override=None):
    import workloads
    return [Unit(name, u, batch, seed, variant_override) for u in range(workloads.CONFIGS[name]["units"])]


def time_region(fn, reps):
    """Average milliseconds of fn() over reps calls, events on the launch stream."""
    import torch
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(reps):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / reps


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
        for _ in range(3):
            fn()
        ms = time_region(fn, steps) / len(units)
        el = units[0].softmax_elements
        res[name] = {"elements": el, "avg_launch_us": ms * 1e3,
                     "gbps": SOFTMAX_BYTES_PER_EL * el / (ms * 1e-3) / 1e9,
                     "pct_of_hbm_peak": 100.0 * SOFTMAX_BYTES_PER_EL * el / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
    del units, d_y32
    torch.cuda.empty_cache()
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
    for cols in (50, 64, 145, 196, 401, 600, 785, 1025, 2048, 4097, 8192, 16384, 32768):
        rows = 60_000_000 // cols
        ins = [(torch.randn((rows, cols), device="cuda", generator=gen) * 5000).round().to(torch.int32)
               for _ in range(4)]
        outs = [torch.empty((rows, cols), dtype=torch.uint8, device="cuda") for _ in range(4)]
        sp = ip.softmax_prepare(2.0 ** -7, cols, 1, 0)

        def fn():
            for x, y in zip(ins, outs):
                ip.softmax_i32(x, None, 0, y, rows, cols, sp)

        fn()
        ms = time_region(fn, max(1, steps // 2)) / len(ins)
        el = rows * cols
        res[str(cols)] = {"rows": rows, "kernel": ip.softmax_kernel_family(cols),
                          "avg_launch_us": ms * 1e3,
                          "pct_of_hbm_peak": 100.0 * SOFTMAX_BYTES_PER_EL * el / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS}
        del ins, outs
    torch.cuda.empty_cache()
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
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: softmax rows and GELU elements are independent, so "
              "the path has no multi-GPU form to time (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2511_15369_amd as ip
    import workloads

    ip.load()
    torch.cuda.set_device(0)

    def measure(name):
        units = build_units(name)

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

        # the same work through the batched entry points: one launch per kernel family
        sm_probs = (ip.SoftmaxProblem * len(units))(*[
            ip.softmax_problem(u.d_scores, u.d_bias, u.period, u.d_probs, u.rows, u.cols, u.sp)
            for u in units])
        ge_probs = (ip.GeluProblem * len(units))(*[
            ip.gelu_problem(u.d_x, u.d_y, u.gelu_n, u.gp) for u in units])
        cols = units[0].cols

        def step_batched():
            ip.softmax_i32_batch(sm_probs, len(units), cols)
            ip.gelu_i8_batch(ge_probs, len(units))

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ms = time_region(step, args.steps)
        wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        sm_ms = time_region(softmax_only, args.steps) / len(units)
        ge_ms = time_region(gelu_only, args.steps) / len(units)
        sm_el = sum(u.softmax_elements for u in units)
        ge_el = sum(u.gelu_n for u in units)
        res = {
            "ms_per_step": ms, "wall_ms_per_step": wall_ms,
            "elements_per_step": sm_el + ge_el,
            "softmax": {"elements": sm_el, "launches": len(units), "avg_launch_us": sm_ms * 1e3,
                        "rows_per_launch": [u.rows for u in units],
                        "gbps": SOFTMAX_BYTES_PER_EL * sm_el / len(units) / (sm_ms * 1e-3) / 1e9},
            "gelu": {"elements": ge_el, "launches": len(units), "avg_launch_us": ge_ms * 1e3,
                     "gbps": GELU_BYTES_PER_EL * ge_el / len(units) / (ge_ms * 1e-3) / 1e9},
        }
        res["value"] = (sm_el + ge_el) / (ms * 1e-3)
        alg_bytes = SOFTMAX_BYTES_PER_EL * sm_el + GELU_BYTES_PER_EL * ge_el
        res["algorithmic_gbps"] = alg_bytes / (ms * 1e-3) / 1e9
        if len(units) <= ip.BATCH_MAX:
            for _ in range(3):
                step_batched()
            bms = time_region(step_batched, args.steps)
            bsm = time_region(lambda: ip.softmax_i32_batch(sm_probs, len(units), cols), args.steps)
            res["batched"] = {"ms_per_step": bms, "value": (sm_el + ge_el) / (bms * 1e-3),
                              "algorithmic_gbps": alg_bytes / (bms * 1e-3) / 1e9,
                              "pct_of_hbm_peak": 100.0 * alg_bytes / (bms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                              "softmax_launch_us": bsm * 1e3,
                              "softmax_gbps": SOFTMAX_BYTES_PER_EL * sm_el / (bsm * 1e-3) / 1e9}
        # the per-unit launch sequence captured once in a HIP graph and replayed (no host work
        # between kernels)
        try:
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
            gms = time_region(graph.replay, args.steps)
            res["graph_replay"] = {"ms_per_step": gms, "value": (sm_el + ge_el) / (gms * 1e-3),
                                   "pct_of_hbm_peak": 100.0 * alg_bytes / (gms * 1e-3) / 1e9 / HBM_PEAK_GBS}
            del graph
        except Exception as exc:                      # graphs are an extra, never the headline
            res["graph_replay"] = {"error": str(exc)[:200]}

        # streaming ceiling of this machine for the softmax's byte mix (4 B in, 1 B out per element):
        # the library's plain requantization kernel over every unit's score tensor
        dy = ip.Dyadic(1, 0, 0, 0, 255)

        def requant_all():
            for u in units:
                ip.requant(u.d_scores.view(-1), u.d_probs.view(-1), u.softmax_elements, 0, dy)

        requant_all()
        rq_ms = time_region(requant_all, max(1, args.steps // 2))
        res["stream_ceiling_gbps"] = SOFTMAX_BYTES_PER_EL * sm_el / (rq_ms * 1e-3) / 1e9
        del units
        torch.cuda.empty_cache()
        return res

    main_res = measure(args.workload)
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
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int32",
        "data": "synthetic",
        "config": {"workload": "%s: %d units x (softmax int32->uint8 + GELU int8->int8), batch %d, "
                               "per-unit scales and variants, seed 0"
                               % (args.workload, cfg["units"], cfg["batch"]),
                   "softmax_elements_per_step": sm["elements"],
                   "gelu_elements_per_step": main_res["gelu"]["elements"]},
        "algorithmic_gbps": main_res["algorithmic_gbps"],
        "pct_of_hbm_peak": 100.0 * main_res["algorithmic_gbps"] / HBM_PEAK_GBS,
        "roofline": {
            "bound": "hbm",
            # single calls of at most 3072 rows (DeiT-T at batch 1) run one wavefront per row
            "kernel": "softmax_rows_kernel" if min(sm["rows_per_launch"]) > 3072 else "softmax_wide_kernel",
            "achieved": sm["gbps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": sm["gbps"] / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC.get(args.workload),
            "avg_launch_us": sm["avg_launch_us"],
            "algorithmic_bytes_per_launch": SOFTMAX_BYTES_PER_EL * sm["elements"] // sm["launches"],
        },
        "kernels": {"softmax": sm, "gelu": main_res["gelu"]},
        "stream_ceiling": {"what": "iptq_requant (int32 -> uint8, same 5 B/element mix) over the same tensors, "
                                   "one launch per unit", "gbps": main_res["stream_ceiling_gbps"]},
        "batched": main_res.get("batched"),
        "graph_replay": main_res.get("graph_replay"),
    }
    if not args.no_extra:
        # the other benchmark configurations, same protocol, one compact entry each
        out["extra"] = {}
        for name in ("swin_b", "vit_s", "swin_s_det", "deit_t"):
            if name == args.workload:
                continue
            r = measure(name)
            e = {k: r[k] for k in ("value", "ms_per_step", "algorithmic_gbps", "softmax", "gelu")}
            e["pct_of_hbm_peak"] = 100.0 * r["algorithmic_gbps"] / HBM_PEAK_GBS
            if name == "swin_b":
                e["batched"] = r.get("batched")
                e["graph_replay"] = r.get("graph_replay")
            elif "batched" in r:
                e["batched_pct_of_hbm_peak"] = r["batched"]["pct_of_hbm_peak"]
            out["extra"][name] = e
    if not args.no_extra:
        out["extra"]["fused_requant"] = measure_fused(args.steps)
        out["extra"]["row_lengths"] = measure_row_lengths(args.steps)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
