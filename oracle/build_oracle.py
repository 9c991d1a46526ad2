"""Compiles the C oracle (oracle/ggnn_ref.c) into oracle/libggnn_ref.so with gcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "ggnn_ref.c")
LIB = os.path.join(HERE, "libggnn_ref.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "ggnn_ref.h"))):
        return LIB
    # -ffp-contract=off: every float32 product, sum and fused multiply-add is exactly the
    # one written in the source
    cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-ffp-contract=off",
           "-fPIC", "-shared", SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
