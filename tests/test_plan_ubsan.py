"""The library's host-side validation and constant derivation (plan.cpp, plain C++) under
UndefinedBehaviorSanitizer, on random and extreme parameters: every call must return a
documented code without tripping the sanitizer."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2511_15369_amd", "csrc")
DRIVER = r"""
#include <stdint.h>
#include <math.h>
#include <stdio.h>
#include "plan.h"
using namespace iptq;
static uint64_t s = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }
static int32_t pick(int32_t lo, int32_t hi) { return lo + (int32_t)(rnd() % (uint64_t)((int64_t)hi - lo + 1)); }
static int32_t wild() { const int32_t v[] = {INT32_MIN, INT32_MAX, -1, 0, 1, 15, 16, 1 << 24, (1 << 24) - 1, 32767, 32768, -32768, 62, 63};
                        return (rnd() & 3) ? (int32_t)(rnd() >> 32) : v[rnd() % 14]; }
int main()
{
    long ok = 0, bad = 0;
    for (int t = 0; t < 300000; ++t) {
        iptq_softmax_params_t p;
        const bool sane = (rnd() & 3) != 0;
        p.variant = sane ? pick(0, 1) : wild();
        p.i0 = sane ? pick(16, (rnd() & 1) ? 4000 : (1 << 24) - 1) : wild();
        p.n_shift = sane ? pick(0, 12) : wild();
        p.m_bits = sane ? pick(20, 31) : wild();
        p.out_bits = sane ? pick(2, 8) : wild();
        p.pre_m = sane ? pick(1, 32767) : wild();
        p.pre_s = sane ? pick(0, 62) : wild();
        p.post.m = sane ? pick(-32767, 32767) : wild();
        p.post.s = sane ? pick(0, 62) : wild();
        p.post.zp = sane ? pick(-300, 300) : wild();
        p.post.qmin = sane ? 0 : wild();
        p.post.qmax = sane ? pick(1, 255) : wild();
        p.out_is_signed = sane ? 0 : wild();
        p.algo = sane ? pick(0, 2) : wild();
        SoftmaxDev dev;
        const int64_t rows = sane ? pick(0, 1 << 20) : (int64_t)wild() * 3;
        const int32_t cols = sane ? pick(1, 700) : wild();
        const int64_t period = sane ? pick(1, 5000) : (int64_t)wild();
        int rc = plan_softmax(&p, rows, cols, (int)(rnd() & 1), period, &dev);
        if (rc > 0 || rc < -6) { printf("bad code %d\n", rc); return 2; }
        (rc == 0 ? ok : bad)++;

        iptq_gelu_params_t g;
        g.variant = sane ? pick(0, 1) : wild();
        g.q_b = sane ? -pick(1, (rnd() & 1) ? 30000 : (1 << 30)) : wild();
        g.q_c = sane ? -(int64_t)(rnd() >> (4 + rnd() % 50)) - 1 : (int64_t)rnd();
        g.k = sane ? pick(0, 62) : wild();
        g.zp_in = sane ? pick(-128, 128) : wild();
        g.max_abs_q = sane ? pick(1, 70000) : wild();
        g.pre_m = sane ? pick(1, 32767) : wild();
        g.pre_s = sane ? pick(0, 62) : wild();
        g.post = p.post;
        g.post.qmin = sane ? -128 : wild();
        g.post.qmax = sane ? 127 : wild();
        g.algo = sane ? pick(0, 1) : wild();
        GeluDev gd;
        rc = plan_gelu(&g, (int)(rnd() & 1), &gd);
        if (rc > 0 || rc < -6) { printf("bad gelu code %d\n", rc); return 3; }
        (rc == 0 ? ok : bad)++;

        int32_t m, sh;
        const double ratios[] = {0.0, 1e-300, 1e300, -3.5, 0.3, 32767.9, 32768.0, 1.0 / 3.0, NAN, INFINITY, -INFINITY, 5e-324};
        iptq_make_dyadic(ratios[rnd() % 12] * (double)(1 + rnd() % 5), &m, &sh);
        iptq_softmax_params_t sp;
        iptq_softmax_prepare(ratios[rnd() % 12], wild(), wild(), wild(), &sp);
        iptq_softmax_prepare(1.0 / (double)(16 + rnd() % 100000), pick(1, 70000), pick(0, 1), pick(0, 1), &sp);
        iptq_gelu_params_t gq;
        iptq_gelu_prepare(ratios[rnd() % 12], ratios[rnd() % 12], wild(), wild(), wild(), wild(), &gq);
        iptq_gelu_prepare(1.0 / (double)(8 + rnd() % 5000000), 1.0 / (double)(8 + rnd() % 5000), pick(-128, 128),
                          pick(-128, 127), pick(0, 1), pick(1, 100000), &gq);
    }
    printf("ok %ld accepted %ld rejected\n", ok, bad);
    return (ok > 1000 && bad > 1000) ? 0 : 4;
}
"""


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not installed")
def test_host_plans_have_no_undefined_behaviour(tmp_path):
    src = tmp_path / "driver.cpp"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    subprocess.check_call(["g++", "-O1", "-g", "-std=c++17", "-fsanitize=undefined,float-cast-overflow",
                           "-fno-sanitize-recover=all", "-I", CSRC, str(src),
                           os.path.join(CSRC, "plan.cpp"), "-o", str(exe)])
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr[-2000:]
    assert res.stdout.startswith("ok")
