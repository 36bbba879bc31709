"""The kernels must be integer-only: compile the device code to gfx950 assembly (hipcc
cross-compiles without a GPU) and fail on any floating-point, conversion, reciprocal or
matrix-core instruction."""
import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_15369_amd", "csrc")
# v_cvt_pk_i16_i32 / v_cvt_pk_u16_u32 are integer-to-integer saturating packs and are allowed
FORBIDDEN = re.compile(r"^\s+(v_[a-z0-9_]*_(f16|f32|f64|bf16)\b|v_cvt_(?!pk_[iu]16_[iu]32)|v_rcp|v_rsq|v_sqrt|v_mfma|v_smfmac|"
                       r"v_exp|v_log|v_pk_[a-z]+_f|v_dot[0-9]*_f|v_fma|v_mad_f|v_mac_f|v_div_)", re.M)


SOURCES = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src, out_dir):
    out = os.path.join(out_dir, src + ".s")
    subprocess.check_call(["hipcc", "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17",
                           "--cuda-device-only", "-S", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", os.path.join(CSRC, src), "-o", out],
                          stderr=subprocess.DEVNULL)
    with open(out) as f:
        return f.read()


@pytest.fixture(scope="session")
def assembly(tmp_path_factory):
    """src -> assembly text.  In a single process every translation unit is compiled up front on
    all cores (one after the other they take minutes); a pytest-xdist worker compiles only the
    files of the tests it was given."""
    out_dir = str(tmp_path_factory.mktemp("isa"))
    if os.environ.get("PYTEST_XDIST_WORKER"):
        return lambda src: _compile(src, out_dir)
    pool = ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1))
    futures = {src: pool.submit(_compile, src, out_dir) for src in SOURCES}
    return lambda src: futures[src].result()


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not installed")
@pytest.mark.parametrize("src", SOURCES)
def test_no_floating_point_instructions(src, assembly):
    text = assembly(src)
    if ".amdhsa_kernel" not in text:                   # a host-only translation unit
        assert "__global__" not in open(os.path.join(CSRC, src)).read()
        return
    assert "s_endpgm" in text
    hits = FORBIDDEN.findall(text)
    assert not hits, hits[:5]
    # no kernel may fall back to per-lane scratch memory (register spills, or a by-value
    # argument struct the compiler had to copy to private memory to index it)
    scratch = re.findall(r"\.amdhsa_private_segment_fixed_size (\d+)", text)
    assert scratch and all(int(b) == 0 for b in scratch), scratch
