"""Build the HIP library in-tree: ``python -m paper_2511_15369_amd.build``.

hipcc cross-compiles for gfx950 without a GPU.  The shared object lands next to
this file so that it travels with the source tree.
"""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libiptq.so")
TIMELINE_LIB = os.path.join(HERE, "libiptq_timeline.so")
# the slowest translation units first (the pool takes them in this order)
SOURCES = ["softmax_wgrow_w4_hi.hip", "softmax_wgrow_w8_hi.hip", "softmax_wgrow_w16.hip", "softmax_wgrow_w4_lo.hip", "softmax_wgrow_w8_lo.hip",
           "softmax_wide_p14_16.hip", "softmax_wide_p11_13.hip", "softmax_wide_p7_10.hip", "softmax_wide_p1_6.hip", "softmax_rowsdyn_k16_long.hip",
           "softmax_rows_577.hip", "softmax_rows_257.hip", "softmax_rows_197.hip", "softmax_rows_198.hip",
           "softmax_rows_144.hip", "softmax_rows_49.hip", "softmax_rows_197_k8.hip", "softmax_rows_198_k8.hip",
           "softmax_rowsdyn_k2.hip", "softmax_rowsdyn_k1.hip", "softmax_rowsdyn_k4.hip", "softmax_rowsdyn_k8.hip",
           "softmax_rowsdyn_k16.hip", "softmax_kernels.hip", "elementwise_kernels.hip",
           "softmax_rowsdyn.hip", "softmax_wide.hip", "softmax_wgrow.hip", "api.hip", "debug_hooks.hip",
           "plan.cpp", "metric.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
         "-Wno-unused-parameter",
         # packed-FP32 instructions stay off: the kernels are integer-only anyway
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(extra_flags=(), verbose: bool = False, lib: str = LIB, obj_dir: str = OBJ) -> str:
    os.makedirs(obj_dir, exist_ok=True)

    def one(src):
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        subprocess.check_call(["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS
                              + list(extra_flags))
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(one, SOURCES))
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, lib)
    if verbose:
        print("built", lib)
    return lib


def build_timeline(verbose: bool = False) -> str:
    """The instrumented library for `python -m paper_2511_15369_amd.timeline` (per-wavefront phase
    timestamps in the compiled-row-length softmax kernels); never loaded by the product path."""
    return build(["-DIPTQ_TIMELINE"], verbose, TIMELINE_LIB, OBJ + "_timeline")


if __name__ == "__main__":
    if sys.argv[1:] == ["timeline"]:
        build_timeline(verbose=True)
    else:
        build(sys.argv[1:], verbose=True)
