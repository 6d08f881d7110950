"""Builds ``csrc/libqsac.so`` (the QSAC step) and ``csrc/libqsac_calib.so`` (measurement aids for the
benchmark) for gfx950 with hipcc (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(CSRC, "libqsac.so")
CALIB_LIB = os.path.join(CSRC, "libqsac_calib.so")
TARGETS = {
    LIB: ([os.path.join(CSRC, "qsac.hip")],
          [os.path.join(CSRC, "qsac_kernels.hip.h"), os.path.join(ROOT, "include", "qsac.h")]),
    CALIB_LIB: ([os.path.join(CSRC, "qsac_calib.hip")], [os.path.join(ROOT, "include", "qsac_calib.h")]),
}

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions stay off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"),
]


def build(force: bool = True) -> str:
    """Compiles both libraries; with ``force=False`` only those older than one of their sources."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    for lib, (sources, headers) in TARGETS.items():
        if not force and os.path.exists(lib):
            t = os.path.getmtime(lib)
            if all(os.path.getmtime(f) <= t for f in sources + headers):
                continue
        subprocess.check_call([hipcc] + HIPCC_FLAGS + ["-o", lib] + sources)
    return LIB


if __name__ == "__main__":
    print(build())
