"""Host-side pieces of bench.py that need no GPU."""
import json
import subprocess
import sys
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_profiled_traffic_figure_is_found():
    import bench
    t = bench.read_traffic("vs_attn:c4")
    assert t is not None and t > 1e9          # bytes per launch, from profiles/c4_hbm_traffic.txt
    assert bench.read_traffic("no_such_kernel:c4") is None


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr
