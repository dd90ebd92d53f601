"""Builds libvlut.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SRC = os.path.join(_HERE, "csrc", "vlut.hip")
LIB = os.path.join(_HERE, "libvlut.so")
INCLUDE = os.path.join(ROOT, "include")

HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
    # packed-FP32 instruction selection is switched off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off",
]


def build(force: bool = True) -> str:
    """Compiles the library; returns its path.  force=False only builds when the .so is missing or stale."""
    if not force and os.path.exists(LIB):
        csrc = os.path.dirname(SRC)     # vlut.hip includes the kernel headers next to it
        sources = [os.path.join(csrc, f) for f in os.listdir(csrc)] + [os.path.join(INCLUDE, "vlut.h")]
        newest = max(os.path.getmtime(f) for f in sources)
        if os.path.getmtime(LIB) >= newest:
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", INCLUDE, SRC, "-o", LIB]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return LIB


if __name__ == "__main__":
    print(build())
