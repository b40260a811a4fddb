"""Build liblaneallreduce.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblaneallreduce.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip",
    "-Wall", "-Wextra", "-Wno-unused-parameter", "-Wno-unused-const-variable",
    # keep hipcc from forming packed fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]
# (source, object name, extra flags): kernels.hip is built once per element type and launch-shape
# family; the largest units come first so that the pool stays busy to the end
UNITS = [("kernels.hip", f"kernels_dtype{d}_shape{f}.o", [f"-DLA_KERNEL_DTYPE={d}", f"-DLA_KERNEL_SHAPE={f}"])
         for f in (2, 0, 1) for d in (2, 3, 4, 1, 0)] + [
    ("fused.hip", f"fused_dtype{d}.o", [f"-DLA_KERNEL_DTYPE={d}"]) for d in (2, 3, 4, 1, 0)] + [
    ("fusion.cpp", "fusion.o", []),
    ("static_scratch.hip", "static_scratch.o", []), ("dispatch.cpp", "dispatch.o", []), ("runtime.cpp", "runtime.o", []), ("schedule.cpp", "schedule.o", [])]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", "lane_allreduce.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, jobs: int = 8) -> str:
    if not force and not stale():
        return LIB
    os.makedirs(OBJ, exist_ok=True)

    def compile_unit(unit):
        src, obj, extra = unit
        cmd = [HIPCC] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ, obj)]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return os.path.join(OBJ, obj)

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, os.cpu_count() or 1, 16))) as ex:
        objs = list(ex.map(compile_unit, UNITS))
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB


def build_consumer(verbose: bool = False) -> str:
    """tests/consumer/consumer.exe: a HIP host program that uses the library through its C header
    only (no Python, no torch in the process); the GPU tests run it."""
    src = os.path.join(ROOT, "tests", "consumer", "consumer.cpp")
    exe = os.path.join(ROOT, "tests", "consumer", "consumer.exe")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), src, "-o", exe,
           "-L", HERE, "-llaneallreduce", "-Wl,-rpath,$ORIGIN/../../paper_2508_13397_amd"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    build(force=True, verbose="-q" not in sys.argv)
    build_consumer(verbose="-q" not in sys.argv)
    print(LIB)
