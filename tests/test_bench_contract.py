"""Host-side checks of bench.py's contract that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    p = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert p.returncode != 0
    assert "one GPU" in p.stderr or "single" in p.stderr.lower() or "1 GPU" in p.stderr
    assert p.stdout.strip() == ""          # no JSON line is printed for a run that did not happen


def test_recorded_traffic_is_tied_to_the_kernel_sources():
    sys.path.insert(0, ROOT)
    import bench
    import json
    path = os.path.join(ROOT, "profiles", "hbm_traffic_C2.txt")
    rec = json.load(open(path))
    got = bench.recorded_traffic("C2", "head_dz")
    if rec["source_digest"] == bench.kernel_source_digest():
        assert got == rec["kernels"]["k_head_dz"]["hbm_bytes_per_launch"]
    else:
        assert isinstance(got, str) and got.startswith("stale")     # counters taken on other code are not quoted
    assert bench.recorded_traffic("C9", "head_dz") is None
