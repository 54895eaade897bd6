"""Compiles the HIP/C++ sources into paper_2510_00606_amd/libelaswave.so for gfx950.

hipcc cross-compiles without a GPU, so this runs anywhere the ROCm toolchain is installed.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libelaswave.so")
SOURCES = [os.path.join(HERE, "csrc", name) for name in (
    "plan.cpp",              # planner: overlap in run-length form, tile tables, queries
    "partition.cpp",         # minimax layer partition
    "runtime.hip",           # error capture, knobs, scratch regions, ew_set_param & co.
    "copy.hip",              # ew_plan_upload, ew_pack, ew_unpack, ew_memcpy
    "cksum.hip",             # ew_snapshot, ew_verify
    "unpack_snapshot.hip",   # ew_unpack_snapshot
    "adam.hip",              # ew_adam_step, ew_grad_ship, host replay
)]


def hipcc_path() -> str:
    p = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(p):
        raise RuntimeError("hipcc not found: the ROCm toolchain is required to build libelaswave.so")
    return p


def build_library(verbose: bool = True) -> str:
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-function",
        "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
        "-x", "hip", *SOURCES, "-o", LIB + ".tmp",
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
