"""Compile the CPU oracle (plain C, OpenMP) into oracle/libst_oracle.so.

Test infrastructure only: the product never loads this library."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "st_oracle.c")
LIB = os.path.join(HERE, "libst_oracle.so")

# -ffp-contract=off: no silent fused multiply-adds, so the float32 interpolation that decides
# the predicted class is rounded exactly where the source says.  -mavx2 -mfma only widens the
# loops and lets fmaf() map to one instruction; both are available on every x86-64-v3 host.
FLAGS = ["-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
         "-fno-fast-math", "-mavx2", "-mfma", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
