"""bench.py's command-line contract, as far as it can be checked without a GPU, and the
workload generators both sides draw from."""
import os
import subprocess
import sys

import numpy as np

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_workload_shapes_match_the_benchmark_configurations():
    c = workloads.CONFIGS
    assert set(c) == {"deit_t", "vit_s", "vit_b", "swin_b", "swin_s_det"}
    # rows x cols of the score matrices and GELU sizes per unit
    expect = {
        "deit_t": [(1 * 3 * 197, 197, 1 * 197 * 768)],
        "vit_s": [(64 * 6 * 197, 197, 64 * 197 * 1536)] * 12,
        "vit_b": [(128 * 12 * 197, 197, 128 * 197 * 3072)] * 12,
        "swin_b": [(64 * 64 * 4 * 49, 49, 64 * 3136 * 512), (64 * 16 * 8 * 49, 49, 64 * 784 * 1024),
                   (64 * 4 * 16 * 49, 49, 64 * 196 * 2048), (64 * 1 * 32 * 49, 49, 64 * 49 * 4096)],
        "swin_s_det": [(2 * 1392 * 3 * 49, 49, 2 * 66800 * 384)],
    }
    for name, units in expect.items():
        cfg = c[name]
        assert cfg["units"] == len(units)
        for u, (rows, cols, gelu_n) in enumerate(units):
            assert cfg["batch"] * cfg["windows"][u] * cfg["heads"][u] * cfg["tokens"][u] == rows
            assert cfg["tokens"][u] == cols
    # the small configuration end to end: seeded, deterministic, in range
    a = workloads.softmax_case("deit_t", 0)
    b = workloads.softmax_case("deit_t", 0)
    assert a.scores.shape == (591, 197) and a.scores.dtype == np.int32
    assert np.array_equal(a.scores, b.scores) and abs(a.scores).max() <= 64 * 127 * 127
    g = workloads.gelu_case("deit_t", 0)
    assert g.x.size == 197 * 768 and g.x.dtype == np.int8 and g.x.min() >= -127
    m = workloads.detection_key_mask()
    assert m.shape == (1392, 49) and 0 < m.sum() < m.size and m.sum(axis=1).max() <= 29
