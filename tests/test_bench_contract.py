"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode == 2
    assert "one GPU" in p.stderr and p.stdout.strip() == ""


def test_fingerprint_is_reproducible():
    sys.path.insert(0, ROOT)
    import bench
    a, b = bench.kernel_source_fingerprint(), bench.kernel_source_fingerprint()
    assert a == b and len(a) == 16
    assert bench.counter_traffic() in (None, bench.COUNTER_TRAFFIC["k_place_bytes_per_launch"])
