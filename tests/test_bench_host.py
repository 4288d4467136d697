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


def test_traffic_is_read_from_the_committed_counter_summary(tmp_path):
    """roofline.traffic comes from the profile summary's machine-readable lines, not from a
    constant in bench.py; a missing file or kernel gives None."""
    f = tmp_path / "c.txt"
    f.write_text("prose\ntraffic_bytes_per_launch k_sp 7.5e9\ntraffic_bytes_per_launch k_lcg 7.9e9\n"
                 "traffic_bytes_per_launch broken\n")
    assert bench.measured_traffic("k_lcg", str(f)) == 7.9e9
    assert bench.measured_traffic("k_sp", str(f)) == 7.5e9
    assert bench.measured_traffic("k_ef_hist", str(f)) is None
    assert bench.measured_traffic("k_lcg", str(tmp_path / "absent.txt")) is None
    # the committed summary carries a figure for both window passes, of the right magnitude:
    # between the stored bytes (6 per entry) and the algorithmic bytes (8 per entry) of a launch
    d, k, n = 110_000_000, 1_100_000, 1024
    for kern, part in (("k_sp", "sp"), ("k_lcg", "lcg")):
        t = bench.measured_traffic(kern)
        assert t is not None
        assert bench.step_bytes(d, k, n, entry=6)[part] * 0.98 <= t <= bench.step_bytes(d, k, n)[part]


def test_step_time_statistics():
    st = bench.step_time_stats([3.0, 1.0, 2.0, 10.0])
    assert st == {"median": 2.5, "min": 1.0, "max": 10.0, "mean": 4.0, "n": 4}
    assert bench.step_time_stats([5.0, 1.0, 3.0])["median"] == 3.0


def test_cpu_baseline_reports_host_cores_and_both_legs():
    """On a tiny stand-in workload: the fields the benchmark line must carry."""
    from paper_2306_06098_amd import synth
    wl = synth.Workload("mini", 40_000, 16, 400, 1e-4, 3, 0.9, 5)
    cb = bench.cpu_baseline(wl)
    assert cb["kind"] == "oracle" and cb["unit"] == "steps/s" and cb["cores"] == 1
    assert cb["host_cores"] == os.cpu_count()
    assert cb["value"] > 0 and abs(cb["value"] * cb["seconds_per_step_full_window"] - 1) < 1e-9
    assert cb["seconds_per_step_first_step_measured"] > 0
    t = cb["seconds_per_step_first_step_measured"] + (wl.m - 1) * cb["seconds_per_window_row"] \
        + cb["seconds_coefficient_recursion"]
    assert abs(t - cb["seconds_per_step_full_window"]) < 1e-9
    assert "measured" in cb["sample"] and "full" in cb["sample"]
