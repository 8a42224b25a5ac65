"""Builds libdrot.so (the HIP kernels and the C ABI of include/drot.h) in-tree for gfx950."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
SOURCES = [os.path.join(_PKG, "csrc", "drot.hip")]
LIB_PATH = os.path.join(_PKG, "libdrot.so")
# the launch planner alone, compiled for the host: what the CPU tests of the path selection load
PLAN_SOURCE = os.path.join(_PKG, "csrc", "drot_plan_host.cpp")
PLAN_LIB_PATH = os.path.join(_PKG, "libdrot_plan.so")
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # hardware fp32 atomic add for the group-lasso accumulators (coarse-grained device memory)
    "-munsafe-fp-atomics",
    # device code only: the kernels never see a NaN (the host rejects NaN arguments; infinities are used and kept),
    # so maxima need no quieting of their inputs and fold into the cross-lane steps of the wave reductions
    "-Xarch_device", "-fno-honor-nans",
    # a product and a sum become one fused operation only where the source says fmaf: the sweeps promise each other
    # the same bits, and with fusion left to the compiler that would hang on which statements share a basic block
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-function",
]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    out = "\n".join(ln for ln in proc.stdout.splitlines() if "packed-fp32-ops" not in ln)
    if proc.returncode != 0:
        raise RuntimeError(f"{cmd[0]} failed:\n{proc.stdout}")
    if verbose and out.strip():
        print(out)


def build_plan(verbose: bool = False) -> str:
    """Compile the launch planner with the host compiler (no GPU code in it)."""
    _run(["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", PLAN_LIB_PATH, PLAN_SOURCE], verbose)
    return PLAN_LIB_PATH


def build(verbose: bool = False) -> str:
    """Compile the HIP sources into libdrot.so (and the host-only planner library); returns the library path."""
    _run(["hipcc", *HIPCC_FLAGS, "-I", os.path.join(_ROOT, "include"), "-o", LIB_PATH, *SOURCES], verbose)
    build_plan(verbose)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
