"""The workgroup -> work item mapping of the attention launches, checked on the host:
tests/sched_check.hip is compiled for the host only and enumerates every hardware
workgroup id for a set of head lists and block counts."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_work_item_is_mapped_exactly_once():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sched_check")
        cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", "-Wno-unused-command-line-argument",
               "-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2407_02490_amd", "csrc"),
               os.path.join(ROOT, "tests", "sched_check.hip"), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        r = subprocess.run([exe], capture_output=True, text=True)
        assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
        assert "FAIL" not in r.stdout and r.stdout.count("ok heads") == 57 and r.stdout.count("ok mixed") == 15


def test_shared_tile_vertical_slash_schedule_covers_every_run_key_once():
    """tests/vs_ring_check.cpp (host only): the four waves of a workgroup yield equally many
    steps, followers read exactly the rows their leader fetched, and the attended keys of every
    wave equal the brute-force cover of the slash runs (App. C.4.2), each key once."""
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "vs_ring_check")
        cmd = ["g++", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "paper_2407_02490_amd", "csrc"),
               os.path.join(ROOT, "tests", "vs_ring_check.cpp"), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        r = subprocess.run([exe], capture_output=True, text=True)
        assert r.returncode == 0 and r.stdout.startswith("ok cases"), r.stdout[-2000:] + r.stderr[-2000:]
