"""Compiles the HIP sources under csrc/ for gfx950 into paper_1912_01059_amd/libggnn.so."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libggnn.so")
SOURCES = ["ggnn_search_reg.hip", "ggnn_search_reg_wide.hip", "ggnn_search_split.hip", "ggnn_search_split_wide.hip",
           "ggnn_search_gv.hip", "ggnn_search_gv_wide.hip", "ggnn_search_any.hip", "ggnn_search_any_wide.hip",
           "ggnn_search_lds.hip", "ggnn_build.hip", "ggnn_api.hip"]
# -ffp-contract=off: float32 arithmetic is exactly what the source says (fused multiply-adds are
# written out where they are wanted), which the bit-for-bit reproducible distances rely on.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC] + os.environ.get("GGNN_EXTRA_FLAGS", "").split()


def _hipcc() -> str:
    for cand in ("hipcc", "/opt/rocm/bin/hipcc"):
        try:
            subprocess.run([cand, "--version"], check=True, capture_output=True)
            return cand
        except (OSError, subprocess.CalledProcessError):
            continue
    raise RuntimeError("hipcc not found")


def _compile(args):
    hipcc, src = args
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    return obj


def build(verbose: bool = False) -> str:
    hipcc = _hipcc()
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 4, 16)) as ex:
        objs = list(ex.map(_compile, [(hipcc, s) for s in SOURCES]))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
