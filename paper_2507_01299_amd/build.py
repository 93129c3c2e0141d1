"""Build liblarosa.so (HIP kernels + C ABI) for gfx950 in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblarosa.so")
SOURCES = ["api.hip", "gemv.hip", "fused.hip", "batched.hip", "topk.hip", "elementwise.hip", "offline.hip", "w4.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build_library(verbose: bool = False) -> str:
    """Compile every source to an object file (in parallel), then link liblarosa.so."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cflags = [f for f in FLAGS if f != "-shared"]

    def compile_one(src):
        obj = os.path.join(objdir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc()] + cflags + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=CSRC)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    link = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True, cwd=CSRC)
    return LIB


def build_diag(verbose: bool = False) -> str:
    """Compile the diagnostic programs csrc/diag_phase_clock.hip (the batch-1 projection kernels) and
    csrc/diag_batched_clock.hip (the batched projection and the per-token Top-K kernel), each the library's own
    kernels with their phase clocks compiled in plus a small driver, into _build/.  Not needed by the library."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    exes = []
    for name in ("diag_phase_clock", "diag_batched_clock"):
        exe = os.path.join(objdir, name)
        cmd = [hipcc()] + [f for f in FLAGS if f not in ("-shared", "-fPIC")] + [os.path.join(CSRC, name + ".hip"),
                                                                                 "-o", exe]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True, cwd=CSRC)
        exes.append(exe)
    return " ".join(exes)


if __name__ == "__main__":
    import sys
    print(build_diag(verbose=True) if "--diag" in sys.argv[1:] else build_library(verbose=True))
