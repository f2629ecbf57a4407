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
# QUIK_ORACLE_SANITIZE=1: an AddressSanitizer + UndefinedBehaviorSanitizer build under another name, for
#   QUIK_ORACLE_SANITIZE=1 ASAN_OPTIONS=detect_leaks=0 \
#   LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)" \
#   python -m pytest tests/test_oracle_pins.py -m "not gpu"
# (same arithmetic flags; -O1 so that reports name source lines)
SANITIZE = os.environ.get("QUIK_ORACLE_SANITIZE") == "1"
if SANITIZE:
    FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
             *[f for f in FLAGS if f != "-O3"]]
    LIB = os.path.join(HERE, "libquik_oracle_san.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", *FLAGS, SRC, "-o", LIB, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)
