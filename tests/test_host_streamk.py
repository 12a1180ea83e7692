"""The integer arithmetic behind the tiled GEMM's stream-K tail (paper_2507_17769_amd/csrc/sk_decomp.h), checked by
brute force on the host: every (blocks, tail tiles, K length) combination of a grid is walked block by block the way
the kernel walks it."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_stream_k_runs_tile_every_tail_exactly_once():
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "streamk_check")
        cmd = ["g++", "-O2", "-std=c++17", "-D__host__=", "-D__device__=", "-I", os.path.join(ROOT, "paper_2507_17769_amd", "csrc"),
               os.path.join(ROOT, "tests", "streamk_check.cpp"), "-o", exe]
        r = subprocess.run(cmd, capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        r = subprocess.run([exe], capture_output=True, text=True)
        assert r.returncode == 0 and r.stdout.startswith("OK "), r.stdout + r.stderr
        assert int(r.stdout.split()[1]) > 1000
