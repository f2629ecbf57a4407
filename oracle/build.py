"""Compile the CPU oracle (plain C + OpenMP) into oracle/libquik_oracle.so.

Test infrastructure: building the checker is not using it.  The flags matter for
parity: no FMA contraction and no fast-math, so every binary32 operation in the
quantizer is a single correctly rounded IEEE operation.  No -march is given, so
the library runs on any x86-64 host.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "quik_oracle.c")
LIB = os.path.join(HERE, "libquik_oracle.so")

FLAGS = ["-O3", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
         "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
