"""Builds libgbmuf.so (gfx950) in-tree with hipcc.  Run as ``python -m paper_1909_09010_amd.build``."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libgbmuf.so")
SOURCES = ["gbmuf_plan.hip", "gbmuf_kernels.hip"]

# -ffp-contract=off: the method's fp32 arithmetic rounds every multiply and add separately.
# The packed-fp32 feature is switched off on purpose (scalar fp32 VALU ops only).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_library(verbose: bool = True, extra_flags=()) -> str:
    """Compiles every HIP source into paper_1909_09010_amd/libgbmuf.so (always recompiles)."""
    cmd = [hipcc(), *HIPCC_FLAGS, *extra_flags, "-o", LIB_PATH] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB_PATH


if __name__ == "__main__":
    build_library(extra_flags=sys.argv[1:])
