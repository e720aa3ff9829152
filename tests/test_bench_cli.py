"""bench.py command-line contract that can be checked without a GPU."""

import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2", "--steps", "1"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_measured_traffic_is_read_from_the_committed_summary():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.measured_traffic("reasoning", 163894, 151936, "fopd_k4_grad_traffic_bytes_per_launch")
    alg = 163894 * 151936 * 4
    assert t is not None and 0.99 * alg < t < 1.02 * alg          # no wasted re-reads
    assert bench.measured_traffic("reasoning", 163895, 151936, "fopd_k4_grad_traffic_bytes_per_launch") is None
    assert bench.measured_traffic("tooluse", 163894, 151936, "fopd_k4_grad_traffic_bytes_per_launch") is None
