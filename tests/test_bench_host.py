"""Host-side checks of bench.py that need no GPU: the one-GPU refusal and the committed counter summary."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)


def test_committed_traffic_matches_the_kernel_source():
    """roofline.traffic comes from the committed counter summary and is dropped when the statistics kernel's
    source no longer matches the fingerprint stored beside it: a change of the kernel without new counters
    fails here instead of silently printing null."""
    sys.path.insert(0, ROOT)
    import bench
    t = bench.committed_traffic()
    assert t is not None, "profiles/stats_partial_kernel_llama3_8b_pmc.txt is older than csrc/stats.hip"
    algorithmic = (6 * 262144 * 4096 * 2 + 262144 * 14336 * 2) / 7
    assert 0.999 < t / algorithmic < 1.01          # nothing is read twice
