"""Builds libzg.so (the C-ABI library: HIP kernels for gfx950 + host planner) in-tree with hipcc."""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libzg.so")
SOURCES = [os.path.join(HERE, "csrc", f) for f in ("zg_host.cpp", "zg_device.hip")]
HEADERS = [os.path.join(HERE, "csrc", "zg_internal.h"), os.path.join(HERE, "csrc", "zg_floyd.h"),
           os.path.join(ROOT, "include", "zg.h")]


def hipcc() -> Optional[str]:
    cand = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return cand if os.path.exists(cand) else shutil.which("hipcc")


def source_id() -> Optional[str]:
    """Hash of the library's sources (what zg_build_id() of a current library returns); None if they are not there."""
    h = hashlib.sha256()
    for f in SOURCES + HEADERS:
        if not os.path.exists(f):
            return None
        h.update(os.path.basename(f).encode() + b"\0" + open(f, "rb").read())
    return h.hexdigest()[:16]


def built_id() -> Optional[str]:
    """zg_build_id() of the library on disk, read from the side file the build writes (no need to load it)."""
    try:
        return open(LIB + ".id").read().strip() if os.path.exists(LIB) else None
    except OSError:
        return None


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and built_id() is not None and built_id() == source_id():
        return LIB
    cc = hipcc()
    if cc is None:
        raise RuntimeError("hipcc not found: cannot build libzg.so")
    sid = source_id()
    cmd = [cc, "-x", "hip", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-ffp-contract=off", "-Wall", "-Wno-unused-function", f'-DZG_BUILD_ID="{sid}"',
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
           "-o", LIB] + SOURCES
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    with open(LIB + ".id", "w") as fh:
        fh.write(sid + "\n")
    return LIB


def ensure_current() -> None:
    """Rebuild when the library is missing or was built from other sources, if hipcc is there to do it (tests,
    smoke and the benchmark call this; on a box without hipcc the binding refuses a stale library instead)."""
    if built_id() is not None and built_id() == source_id():
        return
    if hipcc() is not None and source_id() is not None:
        build(force=True)


if __name__ == "__main__":
    print(build(verbose=True))
