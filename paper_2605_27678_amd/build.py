"""Builds libhp.so (the C-ABI library: host plan builder + gfx950 kernels) with
hipcc, in-tree, next to the sources' package."""
from __future__ import annotations

import os
import shutil
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libhp.so")
SOURCES = ["hp_api.hip", "hp_plan.cpp"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "-shared",
    "--offload-arch=gfx950",
    # keep hipcc from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the backward fold is a fixed-order chain of plain binary32 adds
    "-ffp-contract=off", "-fno-fast-math",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc_path() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found: the HIP library cannot be built on this machine")


def build_library(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source for gfx950 into paper_2605_27678_amd/libhp.so."""
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags,
           "-I", os.path.join(_ROOT, "include"), "-I", CSRC,
           "-o", LIB_PATH, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose and res.stderr.strip():
        print(res.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
