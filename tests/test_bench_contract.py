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
    from paper_2409_13761_amd import build
    a, b = bench.kernel_source_fingerprint(), bench.kernel_source_fingerprint()
    assert a == b == build.source_fingerprint() and len(a) == 16
    for w in ("70b_long", "8b", "batched_reuse"):
        assert bench.counter_traffic(w) in (None, bench.COUNTER_TRAFFIC[w]["k_place_bytes_per_launch"])
        assert os.path.exists(os.path.join(ROOT, bench.COUNTER_TRAFFIC[w]["profile"]))


def test_the_default_workload_is_the_largest_single_pass_one():
    """The line the driver records is on the 70B long-context workload."""
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert 'default="70b_long"' in src
