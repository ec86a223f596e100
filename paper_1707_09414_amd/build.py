"""Build step: compile the gfx950 broadcast library in-tree with hipcc.

    python -m paper_1707_09414_amd.build

hipcc cross-compiles for gfx950 without a GPU present.  The result,
``paper_1707_09414_amd/lib/libbcast.so``, is what the Python binding loads.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from pathlib import Path

PKG = Path(__file__).resolve().parent
REPO = PKG.parent
CSRC = PKG / "csrc"
LIB = PKG / "lib" / "libbcast.so"
SOURCES = ["kernels.hip", "bcast.cpp", "tune.cpp", "memory.cpp"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = True) -> Path:
    LIB.parent.mkdir(parents=True, exist_ok=True)
    tmp = LIB.with_name("libbcast.so.tmp%d" % os.getpid())
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
        # keep the compiler from forming packed-FP32 instructions (not that a byte mover has any)
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-x", "hip",
        "-I", str(REPO / "include"), "-I", str(CSRC),
    ] + [str(CSRC / s) for s in SOURCES] + ["-o", str(tmp)]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
