"""Compile the HIP sources of the library for gfx950 into libquik.so (in-tree)."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libquik.so")
SOURCES = ["quik_api.hip", "quik_quantize.hip", "quik_gemm.hip", "quik_gemm_fp6.hip", "quik_gemm_sp24.hip", "quik_unfused.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes", "-Wno-inline-asm",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def exact_allocations(remarks: str):
    """Kernels whose register allocation (VGPRs + AGPRs, granule 8) ends exactly at their highest
    used register while leaving part of the SIMD's 512-register file free.  On MI355X such a kernel
    (the row-quantization kernel at 208 and at 96 registers) now and then read its highest register
    as the work-item id; allocations of 128 or 256 registers never did.  -> [(kernel, total)]"""
    names = re.findall(r"Function Name: (\S+)", remarks)
    vgprs = re.findall(r" VGPRs: (\d+)", remarks)
    agprs = re.findall(r" AGPRs: (\d+)", remarks)
    out = []
    for name, v, a in zip(names, vgprs, agprs):
        total = int(v) + int(a)
        if total % 8 == 0 and 512 % total != 0:
            out.append((name, total))
    return out


def build(verbose: bool = False, extra_flags=()) -> str:
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics", *extra_flags,
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    other = [ln for ln in proc.stderr.splitlines() if "-Rpass-analysis=kernel-resource-usage" not in ln]
    if other:
        print("\n".join(other), file=sys.stderr, flush=True)
    if proc.returncode != 0:
        raise subprocess.CalledProcessError(proc.returncode, cmd)
    for name, total in exact_allocations(proc.stderr):
        # these claim a register above their highest live one on purpose (inline-asm clobber)
        if "quantize_rows_kernel" in name or "quantize_base_kernel" in name:
            continue
        print(f"note: {name} allocates exactly {total} registers", file=sys.stderr, flush=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
