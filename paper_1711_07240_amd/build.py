"""Build libcgbn.so for gfx950 in-tree with hipcc (cross-compiles without a GPU).

The host code and the multi-sweep kernels are one translation unit; the NCHW
single-launch kernels are instantiated in ten more (element type x direction
x activation), compiled side by side, then everything is linked into one
shared library."""

from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libcgbn.so")
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the slot loops of the single-launch kernels must unroll fully (register arrays), up to 160 iterations
    "-mllvm", "-pragma-unroll-threshold=100000",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _units(obj_dir):
    """(object file, source, extra flags) of every translation unit."""
    OBJ = obj_dir
    units = [(os.path.join(OBJ, "cgbn.o"), os.path.join(CSRC, "cgbn.hip"), [])]
    for tname, t in (("f32", "float"), ("bf16", "bf16_t")):
        for fwd in (1, 0):
            for act in ((0, 1, 2) if fwd else (0, 1)):       # forward: plain, ReLU, shortcut + ReLU
                obj = os.path.join(OBJ, f"fused_{tname}_{'fwd' if fwd else 'bwd'}_act{act}.o")
                units.append((obj, os.path.join(CSRC, "cgbn_fused_inst.hip"),
                              [f"-DCGBN_INST_T={t}", f"-DCGBN_INST_F32={int(t == 'float')}", f"-DCGBN_INST_FWD={fwd}",
                               f"-DCGBN_INST_ACT={act}"]))
    return units


def build(verbose: bool = True, jobs: int | None = None, extra_flags=(), lib: str = LIB, obj_dir: str = OBJ) -> str:
    """Compile and link; `extra_flags` (e.g. a -D for an instrumented build), `lib` and
    `obj_dir` let a second flavour of the library be built beside the product one."""
    os.makedirs(obj_dir, exist_ok=True)
    units = _units(obj_dir)
    jobs = jobs or max(1, min(len(units), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1)), 16))

    def compile_one(u):
        obj, src, extra = u
        cmd = [HIPCC] + FLAGS + list(extra_flags) + extra + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, units))
    cmd = [HIPCC, "--offload-arch=gfx950", "-fno-gpu-rdc", "-shared", "-fPIC", "-o", lib] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    build()
    sys.exit(0)
