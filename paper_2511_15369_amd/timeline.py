"""Where the microseconds of one softmax launch go: per-wavefront phase times from the
instrumented build of the library.

    python -m paper_2511_15369_amd.build timeline      # builds libiptq_timeline.so (no GPU needed)
    python -m paper_2511_15369_amd.timeline             # on the GPU: the four Swin-B stages

Each wavefront of the compiled-row-length kernels records the device-wide 100 MHz clock at
entry, after its slab has landed in LDS (loads and the bias add done), after the arithmetic,
after its last store is issued and after that store is acknowledged.  Printed per launch: the
kernel's span (first entry to last acknowledged store), the distribution of each phase over the
wavefronts, and the cumulative fraction of wavefronts past each phase over time.  Inputs rotate
over enough tensor sets that nothing is served from the 256 MB last-level cache.
"""
import ctypes
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
TIMELINE_LIB = os.path.join(HERE, "libiptq_timeline.so")


def run(rows, cols, lanes_per_row, heads, reps=3, out=sys.stdout):
    import torch

    from . import binding as b
    p = b.softmax_prepare(2.0 ** -7, cols, 1, 0)
    nbuf = max(3, int(600e6 // (5 * rows * cols)) + 1)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(0)
    bufs = [((torch.randn((rows, cols), device="cuda", generator=gen) * 5000).round().to(torch.int32),
             torch.empty((rows, cols), dtype=torch.uint8, device="cuda")) for _ in range(nbuf)]
    bias, period = None, 0
    if heads:
        period = heads * cols
        bias = (torch.randn((period, cols), device="cuda", generator=gen) * 8).round().to(torch.int32)
    rpw = 64 // lanes_per_row
    n_slabs = min(-(-rows // rpw), 65536)
    reader = getattr(b.load(), "iptq_debug_timeline_%d_%d" % (cols, lanes_per_row))
    reader.argtypes = [ctypes.c_void_p, ctypes.c_int]
    reader.restype = ctypes.c_int
    for i in range(nbuf):
        b.softmax_i32(bufs[i][0], bias, period, bufs[i][1], rows, cols, p)
    for rep in range(reps):
        for i in range(nbuf - 1):
            b.softmax_i32(bufs[i][0], bias, period, bufs[i][1], rows, cols, p)
        torch.cuda.synchronize()
        b.softmax_i32(bufs[-1][0], bias, period, bufs[-1][1], rows, cols, p)
        torch.cuda.synchronize()
        tl = np.zeros((n_slabs, 5), dtype=np.uint64)
        assert reader(tl.ctypes.data_as(ctypes.c_void_p), tl.size) == 0
        t = (tl.astype(np.int64) - tl[:, 0].min().astype(np.int64)) / 100.0          # microseconds
        span = t[:, 4].max()

        def dist(a):
            return "min %5.2f  p10 %5.2f  median %5.2f  p90 %5.2f  max %5.2f" % (
                a.min(), np.percentile(a, 10), np.median(a), np.percentile(a, 90), a.max())

        print("rows %d x %d, %d bias heads, %d wavefronts (%.1f MB): span %.2f us" % (
            rows, cols, heads, n_slabs, 5e-6 * rows * cols, span), file=out)
        print("  entry after launch     ", dist(t[:, 0]), file=out)
        print("  slab landed in LDS     ", dist(t[:, 1] - t[:, 0]), file=out)
        print("  arithmetic             ", dist(t[:, 2] - t[:, 1]), file=out)
        print("  bytes to LDS, stores   ", dist(t[:, 3] - t[:, 2]), file=out)
        print("  stores acknowledged    ", dist(t[:, 4] - t[:, 3]), file=out)
        print("  wavefront lifetime     ", dist(t[:, 4] - t[:, 0]), file=out)
        if rep == reps - 1:
            step = 0.5 if span < 14 else 2.0
            print("  time us | entered  loaded  computed  stored   (fraction of wavefronts)", file=out)
            for x in np.arange(0.0, span + step, step):
                print("  %7.1f | %.3f    %.3f   %.3f     %.3f" % (
                    x, (t[:, 0] <= x).mean(), (t[:, 1] <= x).mean(), (t[:, 2] <= x).mean(), (t[:, 4] <= x).mean()), file=out)
        out.flush()
    del bufs
    torch.cuda.empty_cache()


def main():
    from . import binding as b
    if not os.path.exists(TIMELINE_LIB):
        raise SystemExit("libiptq_timeline.so is not built: run `python -m paper_2511_15369_amd.build timeline`")
    b._LIB_PATH = TIMELINE_LIB                         # this process only
    b._lib = None
    # the four Swin-B stages at batch 64 (49-column rows, 2 lanes per row, bias fused)
    for rows, heads in ((100352, 32), (200704, 16), (401408, 8), (802816, 4)):
        run(rows, 49, 2, heads)


if __name__ == "__main__":
    main()
