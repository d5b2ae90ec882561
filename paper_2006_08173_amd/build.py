"""Builds the HIP library `liblgn.so` in-tree for gfx950 (MI355X) with hipcc."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
# LGN_LIB points the binding at another build of the library (A/B timing of kernel variants)
LIB = os.environ.get("LGN_LIB") or os.path.join(PKG, "liblgn.so")
SOURCES = ["api.hip", "stats.hip", "solver.hip", "stream.hip", "stream_f32.hip", "stream_bf16.hip",
           "stream_f16.hip", "prefix.hip", "alloc.hip"]
HEADERS = [os.path.join(CSRC, "lgn_device.hpp"), os.path.join(CSRC, "solver_device.hpp"),
           os.path.join(CSRC, "fpcode_device.hpp"), os.path.join(CSRC, "stream_kernels.hpp"), os.path.join(CSRC, "launch.hpp"),
           os.path.join(os.path.dirname(PKG), "include", "lgn.h")]


def hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    return "hipcc"


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-fno-gpu-flush-denormals-to-zero", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 (one object each, in parallel) and link them into one
    shared library.  Cross-compiles without a GPU."""
    if not force and not is_stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(PKG, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1, 8)) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True)
    print(LIB)
