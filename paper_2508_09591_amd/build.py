"""Builds libhiermoe.so (HIP, gfx950 only) in-tree with hipcc.  No GPU is needed to build."""
from __future__ import annotations

import glob
import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libhiermoe.so")
PROBE_SRC = os.path.join(PKG, "bench_probe", "stream_probe.hip")   # bench.py's flat-stream reference, not product
PROBE_LIB = os.path.join(PKG, "libhmprobe.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
    # packed-fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: libhiermoe.so cannot be built")


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build_library(verbose: bool = False) -> str:
    """Compile every csrc/*.hip into libhiermoe.so, and the benchmark's flat-stream probe into a
    library of its own; always recompiles."""
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", tmp, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    tmp = PROBE_LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-o", tmp, PROBE_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
