"""Builds ``csrc/libqsac.so`` for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(CSRC, "libqsac.so")
SOURCES = [os.path.join(CSRC, "qsac.hip")]
HEADERS = [os.path.join(CSRC, "qsac_kernels.hip.h"), os.path.join(ROOT, "include", "qsac.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions stay off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def build(force: bool = True) -> str:
    """Compiles the library; with ``force=False`` only when a source is newer than it."""
    if not force and os.path.exists(LIB):
        t = os.path.getmtime(LIB)
        if all(os.path.getmtime(f) <= t for f in SOURCES + HEADERS):
            return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc] + HIPCC_FLAGS + ["-o", LIB] + SOURCES)
    return LIB


if __name__ == "__main__":
    print(build())
