"""Builds the simulator's shared library in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libgnr_sim.so")
SOURCES = ["gnr_kernels.hip", "gnr_api.cpp", "gnr_tables.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         # the kernels combine the lanes of a wave themselves before they touch a shared counter; the
         # compiler's own rewrite of atomics into wave-wide scans only adds code around them
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         # loops are unrolled where the source asks for it (#pragma unroll); unrolling the others by heuristic only
         # lengthened the step kernel and measured slightly slower
         "-fno-unroll-loops"]


def build(verbose: bool = False) -> str:
    cmd = [HIPCC] + FLAGS + [f"-I{INCLUDE}", f"-I{CSRC}"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.check_call(cmd)
    return LIB


def lib_path() -> str:
    """Path of the built library; raises if it has not been built."""
    if not os.path.exists(LIB):
        raise FileNotFoundError(f"{LIB} is missing: run `python -m paper_2602_02987_amd.build` (needs hipcc)")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
