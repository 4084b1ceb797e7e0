"""Build the HIP library (C ABI of include/bpe.h) for gfx950, in-tree."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbpe_hip.so")
SOURCES = [os.path.join(CSRC, "bpe.hip")]
INCLUDE = os.path.join(os.path.dirname(HERE), "include")


def headers():
    """Every header the library is compiled from: a change to any of them makes the built library stale."""
    return sorted(glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(INCLUDE, "*.h")))

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # packed fp32 instruction selection is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(f) > t for f in SOURCES + headers())


def build(force: bool = True, extra_flags=()) -> str:
    """Compile csrc/*.hip into libbpe_hip.so with hipcc (cross-compiles without a GPU)."""
    if force or stale():
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-o", LIB, *SOURCES]
        subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())
