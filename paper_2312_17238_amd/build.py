"""Compile the HIP library for gfx950 into paper_2312_17238_amd/libmoe_offload.so."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe_offload.so")
SOURCES = [os.path.join(CSRC, "moe_offload.hip")]
HEADERS = [os.path.join(CSRC, n) for n in ("kernels.h", "layout.h", "cache.h")] + [
    os.path.join(os.path.dirname(HERE), "include", "moe_offload.h")]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
    "-munsafe-fp-atomics", "-pthread",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


def build(force: bool = True, extra=()) -> str:
    """Compiles every time unless force=False and the library is newer than its sources."""
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        subprocess.check_call([hipcc, *FLAGS, *extra, "-o", LIB, *SOURCES])
    return LIB


if __name__ == "__main__":
    import sys
    print(build(True, sys.argv[1:]))
