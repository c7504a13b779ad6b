"""CPU-only: the parts of bench.py's contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_committed_traffic_is_tied_to_the_kernel_source():
    """roofline.traffic comes from the committed counter summary and is dropped when stats.hip changes."""
    sys.path.insert(0, ROOT)
    import bench
    path = os.path.join(ROOT, "profiles", "stats_partial_kernel_llama3_8b_pmc.txt")
    kv = dict(l.split("=", 1) for l in open(path) if "=" in l and not l.lstrip().startswith("#"))
    kv = {k.strip(): v.strip() for k, v in kv.items()}
    t = bench.committed_traffic()
    if t is not None:                       # hash matches: the number must be the committed one and plausible
        assert t == int(float(kv["traffic_bytes_per_launch_avg"]))
        algo = int(kv["algorithmic_bytes_per_launch_avg"])
        assert 0.99 * algo < t < 1.05 * algo


def test_workload_byte_accounting():
    """Algorithmic bytes of the 8B-shaped model from the layer shapes (681.6 GB with one statistics
    pass per linear layer, 475.5 GB with shared statistics)."""
    sys.path.insert(0, ROOT)
    from paper_2501_16376_amd import synth
    T = synth.CALIB_TOKENS
    block = synth.LLAMA3_8B_BLOCK
    stats = sum(T * n * 2 for _, _, n in block)
    sel = sum(out * n * 4 + out * n // 8 + n * 4 for _, out, n in block)
    assert abs(32 * (stats + sel) / 1e9 - 681.6) < 0.1
    shared = T * 2 * (3 * 4096 + 14336)
    assert abs(32 * (shared + sel) / 1e9 - 475.5) < 0.1
    assert abs(32 * sum(out * n * 2 for _, out, n in block) / 1e9 - 13.96) < 0.01
