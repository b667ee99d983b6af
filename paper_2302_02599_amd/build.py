"""Builds the HIP library in-tree: paper_2302_02599_amd/libckpt_dp.so for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libckpt_dp.so")
SOURCES = ["ckpt_dp.hip", "ckpt_host.cpp", "ckpt_schedule.cpp", "ckpt_linearize.cpp"]
ROOFS_LIB = os.path.join(HERE, "libckpt_roofs.so")
ROOFS_SOURCES = ["ckpt_roofs.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-fno-honor-nans",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(lib: str, sources, verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-o", tmp]
    cmd += ["-x", "hip"] + [os.path.join(CSRC, s) for s in sources]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, lib)
    return lib


def build_library(verbose: bool = False) -> str:
    """Compile every source with hipcc (cross-compiles without a GPU): the solver library and
    the benchmark's roof microbenchmarks (a library of their own, not loaded by the solver)."""
    _compile(ROOFS_LIB, ROOFS_SOURCES, verbose)
    return _compile(LIB, SOURCES, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
