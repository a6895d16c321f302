"""Build the HIP library in-tree:  python -m paper_2204_07104_amd.build

hipcc cross-compiles for gfx950 without a GPU, so this runs anywhere the ROCm toolchain is
installed.  The result (libftk.so next to this file) is what the binding loads.

The matrix-core kernels are templates with many instances (order x padded rank x sampling rule x
pass); they are compiled as one translation unit per (kernel family, order), side by side, and
linked with the host file.  Objects live in _build/ (not tracked).
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libftk.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
    # packed fp32 VALU ops are kept off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unused-value", "-Wno-unused-result",
]
# The HIP runtime is NOT linked in: a process must hold exactly one copy of it, and PyTorch
# ships its own.  The binding loads the right one (RTLD_GLOBAL) before this library; a C
# program links libamdhip64 itself.
LINK_FLAGS = ["--offload-arch=gfx950", "-shared", "-fPIC", "-no-hip-rt"]

# (object name, source, extra defines): heaviest first
UNITS = [("api", "ftk_api.hip", [])]
UNITS += [("tiled%d" % n, "ftk_instances.hip", ["-DFTK_INST_FAMILY=2", "-DFTK_INST_ORDER=%d" % n]) for n in range(10, 0, -1)]
UNITS += [("mfma16_%d" % n, "ftk_instances.hip", ["-DFTK_INST_FAMILY=1", "-DFTK_INST_ORDER=%d" % n]) for n in range(6, 0, -1)]


def build(verbose: bool = False, jobs: int = 0) -> str:
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or max(1, min(8, (os.cpu_count() or 2)))

    def compile_unit(unit):
        name, src, defs = unit
        obj = os.path.join(OBJ, name + ".o")
        cmd = [HIPCC, *FLAGS, *defs, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_unit, UNITS))
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, *LINK_FLAGS, *objs, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
