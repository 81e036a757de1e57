"""Build libhago.so (the C-ABI library) from the HIP sources for gfx950.

hipcc cross-compiles without a GPU.  The library is written next to this file
so that it travels with the source tree.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhago.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC",
    "-ffp-contract=off",                       # simquant: no fused multiply-add
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False, jobs: int = 4) -> str:
    """Compile every .hip file and link the shared library; always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs, objs = [], []
    for src in sources():
        obj = os.path.join(objdir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = [hipcc, *HIPCC_FLAGS, "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs, verbose)
    _drain(procs, verbose)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    subprocess.run(cmd, check=True)
    return LIB


def _drain(procs, verbose):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        # the host pass does not know the packed-fp32 target feature and says so
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + "\n".join(lines))
        if verbose and lines:
            print("\n".join(lines), flush=True)


PHASE_LIB = os.path.join(HERE, "libhago_phase.so")


def build_phase_timing(verbose: bool = False) -> str:
    """Development variant of the library for `bench.py --phase-stamps`: the GEMM kernels write a
    timestamp per workgroup at each phase boundary (first loads, main loop, channel terms,
    requantize, copy-out).  Needs the objects of a normal build() for the other sources."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build", "phase")
    os.makedirs(objdir, exist_ok=True)
    timed = ("qgemm_dma.hip", "qgemm.hip")
    procs, objs = [], []
    for src in sources():
        base = os.path.basename(src)
        if base in timed:
            obj = os.path.join(objdir, base + ".o")
            cmd = [hipcc, *HIPCC_FLAGS, "-DHAGO_PHASE_TIMING", "-c", src, "-o", obj]
            procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        else:
            obj = os.path.join(HERE, "_build", base + ".o")
            if not os.path.exists(obj):
                raise RuntimeError(f"{obj} is missing: run build() first")
        objs.append(obj)
    _drain(procs, verbose)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", PHASE_LIB], check=True)
    return PHASE_LIB


if __name__ == "__main__":
    if "--phase-timing" in sys.argv:
        print(build_phase_timing(verbose="-v" in sys.argv))
    else:
        print(build(verbose="-v" in sys.argv))
