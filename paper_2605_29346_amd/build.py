"""Builds libzg.so (the C-ABI library: HIP kernels for gfx950 + host planner) in-tree with hipcc, and the
stand-alone memory-ceiling probe zg_ceilings (its output is kept under profiles/)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libzg.so")
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("zg_host.cpp", "zg_device.hip")]
CEILINGS = os.path.join(HERE, "zg_ceilings")
CEILINGS_SRC = os.path.join(HERE, "csrc", "zg_ceilings.hip")
HEADERS = [os.path.join(HERE, "csrc", "zg_internal.h"), os.path.join(ROOT, "include", "zg.h")]


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and os.path.exists(LIB):
        newest = max(os.path.getmtime(f) for f in SOURCES + HEADERS)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-ffp-contract=off", "-Wall", "-Wno-unused-function",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    probe = [hipcc, "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-o", CEILINGS, CEILINGS_SRC]
    if verbose:
        print(" ".join(probe))
    subprocess.run(probe, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
