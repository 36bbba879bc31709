"""The boundary is a C ABI: a C99 program that includes only include/iptq.h, links libiptq.so
and calls the host-side entry points (no GPU work) must compile without warnings and run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2511_15369_amd")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not installed")
def test_c99_program_links_and_runs(tmp_path):
    lib = os.path.join(PKG, "libiptq.so")
    if not os.path.exists(lib):
        pytest.skip("libiptq.so not built")
    exe = str(tmp_path / "host_only")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                           "-I", os.path.join(ROOT, "include"),
                           os.path.join(ROOT, "tests", "c_consumer", "host_only.c"), "-o", exe,
                           "-L", PKG, "-liptq", "-Wl,-rpath," + PKG])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, (out.returncode, out.stdout, out.stderr)
    assert out.stdout.startswith("ok ")


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not installed")
def test_header_is_plain_c99():
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                           "-x", "c", os.path.join(ROOT, "include", "iptq.h")])
