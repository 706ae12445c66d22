"""Builds libtensair.so (hand-written HIP for gfx950 + the C-ABI host code) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtensair.so")
SOURCES = ["api.hip", "sample.hip", "sort.hip", "grad.hip", "apply.hip", "dense.hip", "probe.hip", "noalloc.hip"]
HEADERS = ["dev_common.h", "kernels.h", os.path.join("..", "..", "include", "tensair.h")]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # fused multiply-adds only where the source says fmaf
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every kernel and the host code into one shared library."""
    if not force and not stale():
        return LIB
    extra = os.environ.get("TENSAIR_EXTRA_HIPCC_FLAGS", "").split()   # tuning experiments (-DNAME=value)
    cmd = ["hipcc", *FLAGS, *extra, "-o", LIB, *[os.path.join(CSRC, f) for f in SOURCES]]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
