"""bench.py's command line, as far as it can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_traffic_figure_comes_from_the_committed_profile():
    sys.path.insert(0, ROOT)
    import bench
    t = bench.measured_traffic("fwd_f16", "c2")
    assert t is not None and 0.9 < t / 189_464_576 < 1.5
    assert bench.measured_traffic("fwd_f16", "no_such_workload") is None
    # ... and only for the kernel it was measured on
    assert bench.measured_traffic("fwd_f16", "c2", kernel="some_other_kernel<1>") is None
