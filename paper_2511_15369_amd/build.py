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


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS + list(extra)
    subprocess.check_call(cmd)
    return obj


def build(extra_flags=(), verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(lambda s: _compile(s, extra_flags), SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs)
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(sys.argv[1:], verbose=True)
