"""Build libferret.so (host planner + HIP kernels) for gfx950 with hipcc, in-tree.

    python -m paper_2503_12053_amd.build [--force]
    python -m paper_2503_12053_amd.build --sanitize [dir]     host code under ASan/UBSan and TSan (no GPU needed)

The library lands next to this file so that it travels with the source tree; nothing is
installed.  hipcc cross-compiles: no GPU is needed to build.
"""
from __future__ import annotations

import hashlib
import os
import re
import shutil
import subprocess
import sys
import tempfile

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


FLAGS = [f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-parameter",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


_TOKEN = re.compile(r'''"(?:\\.|[^"\\])*"|'(?:\\.|[^'\\])*'|//[^\n]*|/\*.*?\*/''', re.S)


def _code_only(text: str) -> str:
    """The source text without comments and with runs of white space collapsed (string and character literals are
    kept as they are): what the compiler sees, so that editing a comment does not change the hash below."""
    text = _TOKEN.sub(lambda m: m.group(0) if m.group(0)[0] in "\"'" else " ", text)
    return " ".join(text.split())


def source_hash() -> str:
    """First 12 hex digits of the SHA-256 over the code (comments stripped) of every source and header the library
    is built from, in a fixed order, and the compiler flags.  The library reports it through ferret_version(), so
    that a measurement can say which sources it belongs to and a stored profile summary can be matched against the
    build that is timed."""
    h = hashlib.sha256()
    for path in sorted(SOURCES + HEADERS):
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "r", encoding="utf-8") as f:
            h.update(_code_only(f.read()).encode())
    h.update(" ".join(f for f in FLAGS if not f.startswith("/") and os.sep not in f).encode())
    return h.hexdigest()[:12]


def command(out: str = LIB) -> list:
    """The whole library as ONE hipcc command (every source one translation unit each)."""
    return [hipcc(), *FLAGS, f'-DFERRET_SOURCE_HASH="{source_hash()}"', "-shared", "-x", "hip", *SOURCES, "-o", out]


def compile_jobs(objdir: str) -> list:
    """(command, object) per translation unit.  The kernels file is compiled three times with FERRET_TU = 0, 1, 2
    (small kernels + launch logic / step kernels for fp32 storage / for bf16 storage) so that the parts build
    in parallel; the two host files are one unit each."""
    jobs = []
    kernels = os.path.join(CSRC, "ferret_kernels.hip")
    for tu in (0, 1, 2):
        obj = os.path.join(objdir, f"ferret_kernels_tu{tu}.o")
        jobs.append(([hipcc(), *FLAGS, f"-DFERRET_TU={tu}", "-c", "-x", "hip", kernels, "-o", obj], obj))
    for src in SOURCES:
        if src != kernels:
            obj = os.path.join(objdir, os.path.basename(src) + ".o")
            jobs.append(([hipcc(), *FLAGS, f'-DFERRET_SOURCE_HASH="{source_hash()}"', "-c", "-x", "hip", src, "-o", obj], obj))
    return jobs


SANITIZERS = {"address": ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"],
              "thread": ["-fsanitize=thread"]}


def build_sanitized(kind: str, out: str, verbose: bool = False) -> str:
    """Host-only executable for sanitizer runs (no GPU, no hipcc): the library's host sources, the stand-in launchers
    and the driver under tests/sanitize/, compiled with the host C++ compiler and -fsanitize=address,undefined
    (kind "address") or -fsanitize=thread (kind "thread").  Run it as `<out> all` or `<out> planner`; it exits
    non-zero when one of its checks or the sanitizer fails."""
    cxx = shutil.which("g++") or shutil.which("c++")
    if cxx is None:
        raise RuntimeError("no host C++ compiler found")
    san = os.path.join(ROOT, "tests", "sanitize")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", *SANITIZERS[kind], "-Wall", "-Wno-unused-parameter",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           *[s for s in SOURCES if not s.endswith(".hip")],
           os.path.join(san, "stub_launchers.cpp"), os.path.join(san, "host_driver.cpp"), "-pthread", "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    return all(os.path.getmtime(f) <= t for f in SOURCES + HEADERS + [__file__])


def build(force: bool = False, verbose: bool = True) -> str:
    if not force and up_to_date():
        return LIB
    with tempfile.TemporaryDirectory(prefix="ferret_build_") as objdir:
        jobs = compile_jobs(objdir)
        procs = []
        for cmd, _ in jobs:                              # all translation units at once
            if verbose:
                print(" ".join(cmd), flush=True)
            procs.append(subprocess.Popen(cmd))
        failed = [cmd for (cmd, _), p in zip(jobs, procs) if p.wait() != 0]
        if failed:
            raise subprocess.CalledProcessError(1, failed[0])
        link = [hipcc(), f"--offload-arch={ARCH}", "-shared", "-fPIC", *[obj for _, obj in jobs], "-o", LIB]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    if "--sanitize" in sys.argv:           # python -m paper_2503_12053_amd.build --sanitize [dir]: build and run both
        outdir = sys.argv[sys.argv.index("--sanitize") + 1] if len(sys.argv) > sys.argv.index("--sanitize") + 1 \
            else tempfile.mkdtemp(prefix="ferret_sanitize_")
        for kind, what in (("address", "all"), ("thread", "planner")):
            exe = build_sanitized(kind, os.path.join(outdir, f"host_driver_{kind}"), verbose=True)
            subprocess.run([exe, what], check=True)
        print("sanitizer runs clean")
        sys.exit(0)
    build(force="--force" in sys.argv)
    print(LIB)
