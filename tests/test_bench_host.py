"""Host-side logic of bench.py (no GPU): the stated accepted-length law, the algorithmic byte counts the
roofline figures are priced with, and the refusal to run on more than one GPU."""
import os
import subprocess
import sys

import pytest

import bench
import deer_inputs as di

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("k,mean", [(32, 8), (32, 24), (16, 4), (4, 3)])
def test_truncated_geometric_law(k, mean):
    rho, e_n = bench.trunc_geom(k, mean)
    p = [(1 - rho) * rho ** i for i in range(k)] + [rho ** k]
    assert abs(sum(p) - 1) < 1e-12
    assert abs(sum(i * pi for i, pi in enumerate(p)) - mean) < 1e-9          # E[a] is the requested mean
    # a < k commits a + 1 tokens (the correction), a = k commits k: E[n] by direct summation
    direct = sum((i + 1) * pi for i, pi in enumerate(p[:-1])) + k * p[-1]
    assert abs(e_n - direct) < 1e-9


def test_verify_bytes_of_the_headline_workload():
    cfg = di.CONFIGS["qwen3_8b"]
    w, kv = bench.verify_bytes(cfg["target"], cfg["prefix"], cfg["k"])
    t = cfg["target"]
    per_layer = (t.d_model * (t.n_q_heads + 2 * t.n_kv_heads) * t.head_dim      # QKV
                 + t.n_q_heads * t.head_dim * t.d_model                         # O
                 + 3 * t.d_model * t.d_ff)                                      # gate, up, down
    assert per_layer == 192_937_984                                             # parameters of one 8B-shaped layer
    assert w == 2.0 * (36 * per_layer + t.d_model * t.vocab)
    assert abs(w - 15.136e9) < 2e6 and abs(w + kv - 15.74e9) < 1e7
    assert kv == 2.0 * 2 * 36 * 8 * 128 * (4096 - 1 + 32)


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
