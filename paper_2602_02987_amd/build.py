"""Builds the simulator's shared library in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libgnr_sim.so")
OBJ = os.path.join(HERE, "_build")
# every policy variant of the step kernel is a translation unit of its own, so that they compile side by side
STEP_VARIANTS = ["plain", "rr", "im", "ab", "ab_rr", "ab_im", "ws"]
SOURCES = ["gnr_kernels.hip", "gnr_api.cpp", "gnr_tables.cpp"] + [f"gnr_step_{v}.hip" for v in STEP_VARIANTS]
HEADERS = [os.path.join(CSRC, "gnr_step.h"), os.path.join(CSRC, "gnr_internal.h"), os.path.join(INCLUDE, "gnr_sim.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off",
         # no packed fp32 instructions in device code (the host pass does not know the feature and says so)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         # the kernels combine the lanes of a wave themselves before they touch a shared counter; the
         # compiler's own rewrite of atomics into wave-wide scans only adds code around them
         "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
         # loops are unrolled where the source asks for it (#pragma unroll); unrolling the others by heuristic only
         # lengthened the step kernel and measured slightly slower
         "-fno-unroll-loops",
         # the step kernel lives at its register limit: loop strength reduction and the hoisting of loop invariants
         # in machine code both trade registers for instructions, which here ends in spills (scratch per lane of the
         # sixteen-wave base variant 100 B with them, 28 B without; 1.7 % faster on the largest configuration)
         "-mllvm", "-disable-lsr", "-mllvm", "-disable-machine-licm"]


def _compile(src: str, force: bool, verbose: bool) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    deps = [path] + HEADERS
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) > os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC] + FLAGS + [f"-I{INCLUDE}", f"-I{CSRC}", "-c", path, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, flush=True)
    return obj


def build(verbose: bool = False, force: bool = True, jobs: int | None = None) -> str:
    """Compiles every source (all of them when `force`, else those older than their object) and links the library."""
    os.makedirs(OBJ, exist_ok=True)
    jobs = jobs or min(len(SOURCES), os.cpu_count() or 1, 16)
    with ThreadPoolExecutor(jobs) as pool:
        objs = list(pool.map(lambda s: _compile(s, force, verbose), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def lib_path() -> str:
    """Path of the built library; raises if it has not been built."""
    if not os.path.exists(LIB):
        raise FileNotFoundError(f"{LIB} is missing: run `python -m paper_2602_02987_amd.build` (needs hipcc)")
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, force="--changed" not in sys.argv))
