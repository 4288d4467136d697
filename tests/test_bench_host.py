"""Host-side pieces of bench.py: the byte model behind the roofline figures and
the one-GPU rule.  No GPU is touched."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402


def test_step_bytes_is_the_benchmark_formula():
    """16*n*k + 24*d + 8*k algorithmic bytes per step: 20.68 GB at d=110M, m=1024,
    k=1.1M (the figure the 60 % target is quoted on), 2.106 GB at d=11.2M."""
    d, k, n = 110_000_000, 1_100_000, 1024
    by = bench.step_bytes(d, k, n)
    assert by["total"] == 16 * n * k + 24 * d + 8 * k
    assert abs(by["total"] / 1e9 - 20.68) < 0.01
    assert by["ef"] + by["sp"] + by["lcg"] == by["total"]
    assert abs(bench.step_bytes(11_200_000, 112_000, n)["total"] / 1e9 - 2.106) < 0.002
    # stored bytes: 6 per entry; x = c_t drops both dense reads of x; the fused update reads
    # and writes the parameters instead of writing the preconditioned vector
    assert bench.step_bytes(d, k, n, entry=6)["total"] == 12 * n * k + 24 * d + 6 * k
    assert by["total"] - bench.step_bytes(d, k, n, mode="compressed")["total"] == 8 * d
    assert bench.step_bytes(d, k, n, mode="update")["total"] - by["total"] == 4 * d


def test_more_than_one_gpu_is_refused_before_anything_runs():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
