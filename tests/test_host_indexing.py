"""Index and address arithmetic of the kernels, run on the CPU at the size of the largest workload.

The helpers the kernels use for the bottom layer (partition permutation, segment bounds, row offsets,
launch chunks) are host-callable; tests/host_index_sweep.cpp walks them over all 10^8 positions of the
100M x 128-byte workload, compiled for the host with the address and undefined-behaviour sanitizers,
and checks every value against the array it indexes.  (A launch of 10^8 workgroups of 64 work-items
needs 6.4 * 10^9 work-items in one grid dimension, more than the 32 bits a dispatch counts them in: the
program also checks that the chunked launches stay below that.)"""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_1912_01059_amd", "csrc")


@pytest.fixture(scope="module")
def sweep(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("sweep") / "host_index_sweep")
    cmd = ["hipcc", "-x", "hip", "--cuda-host-only", "-O2", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-I", CSRC, "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "host_index_sweep.cpp"), "-o", exe]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return exe


@pytest.mark.parametrize("args", [
    ["100000000", "128", "24", "4", "32", "1"],     # the 100M x 128 uint8 workload, every position
    ["2147483647", "16", "24", "4", "32", "997"],   # the largest N the ids allow, sampled
    ["70000000", "16", "8", "4", "32", "101"],      # more points than one launch holds, short rows
    ["1000000", "512", "24", "4", "32", "1"],       # the benchmark workload
    ["1200000", "400", "40", "4", "32", "1"],       # rows that are not a multiple of 128 bytes
])
def test_bottom_layer_indices_stay_inside_their_arrays(sweep, args):
    r = subprocess.run([sweep] + args, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert r.stdout.strip().endswith("ok")
    if args[0] in ("100000000", "2147483647", "70000000"):
        assert "does not fit" in r.stdout
