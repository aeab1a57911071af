"""Build libferret.so (host planner + HIP kernels) for gfx950 with hipcc, in-tree.

    python -m paper_2503_12053_amd.build [--force]

The library lands next to this file so that it travels with the source tree; nothing is
installed.  hipcc cross-compiles: no GPU is needed to build.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libferret.so")
SOURCES = [os.path.join(CSRC, "ferret_host.cpp"), os.path.join(CSRC, "ferret_planner.cpp"),
           os.path.join(CSRC, "ferret_kernels.hip")]
HEADERS = [os.path.join(CSRC, "ferret_internal.h"), os.path.join(ROOT, "include", "ferret.h"),
           os.path.join(ROOT, "include", "ferret_planner.h")]
ARCH = "gfx950"


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found (looked on PATH and in /opt/rocm/bin)")
    return exe


def command(out: str = LIB) -> list:
    return [hipcc(), f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC", "-shared",
            # keep the compiler from forming packed-fp32 instructions
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-Wno-unused-parameter",
            "-I", os.path.join(ROOT, "include"), "-I", CSRC,
            "-x", "hip", *SOURCES, "-o", out]


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(f) <= t for f in SOURCES + HEADERS + [__file__])


def build(force: bool = False, verbose: bool = True) -> str:
    if not force and up_to_date():
        return LIB
    cmd = command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(force="--force" in sys.argv)
    print(LIB)
