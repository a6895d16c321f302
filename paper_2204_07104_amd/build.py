"""Build the HIP library in-tree:  python -m paper_2204_07104_amd.build

hipcc cross-compiles for gfx950 without a GPU, so this runs anywhere the ROCm toolchain is
installed.  The result (libftk.so next to this file) is what the binding loads.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libftk.so")
SOURCES = ["ftk_api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-munsafe-fp-atomics",
    # The HIP runtime is NOT linked in: a process must hold exactly one copy of it, and PyTorch
    # ships its own.  The binding loads the right one (RTLD_GLOBAL) before this library; a C
    # program links libamdhip64 itself.
    "-no-hip-rt",
    # packed fp32 VALU ops are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unused-value", "-Wno-unused-result",
]


def build(verbose: bool = False) -> str:
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, *[os.path.join(CSRC, s) for s in SOURCES], "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
