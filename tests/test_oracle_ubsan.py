"""The oracle under UndefinedBehaviorSanitizer: signed overflow, bad shift counts and
out-of-range conversions are the likeliest mistakes in fixed-width integer code.  A small C
driver feeds it extreme inputs and parameters; any report aborts the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DRIVER = r"""
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include "iptq_oracle.c"

static uint64_t s = 88172645463325252ull;
static uint64_t rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }

int main(void)
{
    enum { ROWS = 64, COLS = 67 };
    static int32_t x[ROWS * COLS], bias[5 * COLS];
    static uint8_t out[ROWS * COLS];
    static int8_t g8[4096], y8[4096];
    static int32_t g32[4096];
    const int32_t i0s[] = {16, 17, 181, 1000, 65535, (1 << 24) - 1};
    for (int trial = 0; trial < 200; ++trial) {
        for (int i = 0; i < ROWS * COLS; ++i) {
            uint64_t r = rnd();
            x[i] = (r & 7) == 0 ? (int32_t)(r >> 32) : (int32_t)((int64_t)(r >> 40) % 5000 - 2500);
            if ((r & 63) == 1) x[i] = INT32_MIN;
            if ((r & 63) == 2) x[i] = INT32_MAX;
        }
        for (int i = 0; i < 5 * COLS; ++i) bias[i] = (int32_t)(rnd() >> 32);
        orc_softmax_params p = {0};
        p.variant = trial & 1;
        p.i0 = i0s[trial % 6];
        p.n_shift = 0;
        while (((int64_t)p.i0 << (p.n_shift + 1)) < (1 << 15)) p.n_shift++;
        p.m_bits = 31; p.out_bits = 2 + trial % 7;
        p.pre_m = 1 + (int32_t)(rnd() % 32767); p.pre_s = (int32_t)(rnd() % 63);
        if (trial % 3 == 0) { p.pre_m = 1; p.pre_s = 0; }
        p.post.m = (int32_t)(rnd() % 65535) - 32767; p.post.s = (int32_t)(rnd() % 63);
        p.post.zp = (int32_t)(rnd() % 200) - 100; p.post.qmin = 0; p.post.qmax = 255;
        if (iptq_ref_softmax_i32(x, (trial & 2) ? bias : 0, 5, out, ROWS, COLS, &p) != 0) {
            printf("softmax rejected trial %d\n", trial);
            return 2;
        }
        orc_dyadic d = {(int32_t)(rnd() % 65535) - 32767, (int32_t)(rnd() % 63), 3, -128, 127};
        if (iptq_ref_requant(x, out, ROWS * COLS, 1, &d) != 0) return 3;
    }
    /* GELU: constants of scales 2^-4 .. 2^-12 (q_b, q_c as the derivation gives them) */
    const struct { int32_t variant, q_b; int64_t q_c; int32_t k; } gp[] = {
        {1, -62, -13164466, 2}, {1, -245, -3370103149ll, 10}, {0, -41, -1773, 0},
        {1, -15630, -55834574848000000ll, 40}, {0, -10247, -114000000, 12}};
    for (int c = 0; c < 5; ++c) {
        orc_gelu_params p = {0};
        p.variant = gp[c].variant; p.q_b = gp[c].q_b; p.q_c = gp[c].q_c; p.k = gp[c].k;
        p.zp_in = -128 + 51 * c; p.max_abs_q = 255; p.pre_m = 1; p.pre_s = 0;
        {   /* the smallest shift that keeps q * v inside 32 bits for |q| <= 255 */
            int64_t t = -(int64_t)p.q_b, tp = t * t;
            if (p.variant == 1) tp *= tp;
            while (((tp + 2 * (-p.q_c)) >> p.k) * 255 >= ((int64_t)1 << 31)) p.k++;
        }
        p.post.m = -20880; p.post.s = 20 + 8 * c; p.post.zp = -7; p.post.qmin = -128; p.post.qmax = 127;
        for (int i = 0; i < 4096; ++i) { g8[i] = (int8_t)(rnd() >> 56); g32[i] = (int32_t)(rnd() >> 32); }
        g32[0] = INT32_MIN; g32[1] = INT32_MAX;
        if (iptq_ref_gelu_i8(g8, y8, 4096, &p) != 0) { printf("gelu rejected %d\n", c); return 4; }
        p.pre_m = 32767; p.pre_s = c * 15;
        if (iptq_ref_gelu_i32(g32, y8, 4096, &p) != 0) { printf("gelu32 rejected %d\n", c); return 5; }
    }
    printf("ok\n");
    return 0;
}
"""


@pytest.mark.skipif(shutil.which("gcc") is None, reason="gcc not installed")
def test_oracle_has_no_undefined_behaviour(tmp_path):
    src = tmp_path / "driver.c"
    src.write_text(DRIVER)
    exe = tmp_path / "driver"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=gnu99", "-fsanitize=undefined,float-cast-overflow",
                           "-fno-sanitize-recover=all", "-I", os.path.join(ROOT, "oracle"),
                           str(src), "-o", str(exe)])
    res = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "ok" in res.stdout
