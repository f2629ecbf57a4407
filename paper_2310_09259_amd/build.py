"""Compile the HIP sources of the library for gfx950 into libquik.so (in-tree).

Every source is compiled to an object of its own (in parallel) and the objects are linked;
`build()` recompiles everything, `build(incremental=True)` only the sources that changed since their
object was made (any header change recompiles all)."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libquik.so")
SOURCES = ["quik_api.hip", "quik_quantize.hip", "quik_gemm.hip", "quik_gemm_tiles16.hip", "quik_gemm_stream.hip", "quik_gemm_fp6.hip", "quik_gemm_sp24.hip",
           "quik_unfused.hip", "quik_probe.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes", "-Wno-inline-asm",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]
# kernels that claim a register above their highest live one on purpose (inline-asm clobber), so that
# their allocation is a full share of the register file: see exact_allocations
CLAIMS_FULL_SHARE = ("quantize_rows_kernel", "quantize_base_kernel")


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


def _newest_header() -> float:
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hdrs.append(os.path.join(ROOT, "include", "quik.h"))
    return max(os.path.getmtime(h) for h in hdrs)


def _compile(src: str, extra_flags, verbose: bool):
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics", *extra_flags,
           "-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    return src, obj, proc


def build(verbose: bool = False, extra_flags=(), incremental: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    todo = []
    hdr_time = _newest_header()
    for s in SOURCES:
        obj = os.path.join(OBJ, s.replace(".hip", ".o"))
        fresh = (incremental and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(os.path.join(CSRC, s)), hdr_time))
        if not fresh:
            todo.append(s)
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(todo)))) as pool:
        results = list(pool.map(lambda s: _compile(s, extra_flags, verbose), todo))
    remarks = ""
    for src, obj, proc in results:
        other = [ln for ln in proc.stderr.splitlines()
                 if "-Rpass-analysis=kernel-resource-usage" not in ln and "packed-fp32-ops" not in ln]
        if other:
            print("\n".join(other), file=sys.stderr, flush=True)
        if proc.returncode != 0:
            if os.path.exists(obj):
                os.remove(obj)
            raise subprocess.CalledProcessError(proc.returncode, proc.args)
        remarks += proc.stderr
    bad = [(n, t) for n, t in exact_allocations(remarks) if not any(k in n for k in CLAIMS_FULL_SHARE)]
    if bad:
        # not a note: a kernel with such an allocation has produced wrong results on the hardware, so
        # it must not ship (give it an inline-asm clobber of a higher register, or change its shape)
        for src in todo:
            obj = os.path.join(OBJ, src.replace(".hip", ".o"))
            if os.path.exists(obj):
                os.remove(obj)
        raise RuntimeError("kernels whose register allocation ends exactly on a partial share of the "
                           "register file: " + ", ".join(f"{n} ({t})" for n, t in bad))
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC",
            *[os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    inc = "--incremental" in sys.argv[1:]
    print(build(verbose=True, extra_flags=[a for a in sys.argv[1:] if a != "--incremental"], incremental=inc))
