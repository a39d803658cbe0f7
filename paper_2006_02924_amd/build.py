"""Builds ``libadasum.so`` (gfx950) in-tree with hipcc.

Usage: ``python -m paper_2006_02924_amd.build``.  hipcc cross-compiles without a
GPU.  The library is written next to this file so that it travels with the
source tree.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libadasum.so")
# a measuring tool (the memory system's ceiling for the combine pass's access pattern)
CEILING_PATH = os.path.join(HERE, "pattern_ceiling")

SOURCES = ["adasum_kernels.hip", "adasum_api.cpp", "adasum_plan.cpp"]

# -packed-fp32-ops off: the compiler must not form packed fp32 instructions.
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the HIP library cannot be built")
    return exe


def build_library(verbose: bool = True, extra_flags=(), out_path: str = LIB_PATH) -> str:
    cmd = [hipcc(), "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden", "-Wall", "-Wno-unused-command-line-argument",
           *DEVICE_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, *extra_flags]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    cmd += ["-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out_path


def build_pattern_ceiling(verbose: bool = True, out_path: str = CEILING_PATH) -> str:
    cmd = [hipcc(), "-O3", "-std=c++17", "-Wall", "-Wno-unused-command-line-argument", *DEVICE_FLAGS,
           os.path.join(CSRC, "pattern_ceiling.hip"), "-o", out_path]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out_path


if __name__ == "__main__":
    build_library()
    build_pattern_ceiling()
    print(LIB_PATH)
    print(CEILING_PATH)
    sys.exit(0)
