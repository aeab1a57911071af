"""The public headers as a C compiler sees them: tests/c/consumer.c (plain C99, -pedantic -Wall -Wextra -Werror)
is compiled with gcc against include/ferret.h and include/ferret_planner.h, linked to libferret.so and run.  It makes
host-only calls and prints the layout of every public struct; this test compares those layouts with the ctypes
mirrors in the Python binding (which are written by hand) and the values with what the binding gets for the
same calls.  No GPU is needed."""
import ctypes
import os
import re
import shutil
import subprocess

import pytest

from paper_2503_12053_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PKG = os.path.join(ROOT, "paper_2503_12053_amd")

MIRRORS = {"ferret_tensor": B.ferret_tensor, "ferret_tuning": B.ferret_tuning, "ferret_adaptive": B.ferret_adaptive,
           "ferret_accumulate": B.ferret_accumulate, "ferret_layer": B.ferret_layer}
RENAMED = {("ferret_adaptive", "lambda"): "lambda_"}          # `lambda` is a Python keyword


@pytest.fixture(scope="module")
def consumer_output(tmp_path_factory):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc is not installed")
    B.load()
    exe = str(tmp_path_factory.mktemp("c_consumer") / "consumer")
    rocm_lib = "/opt/rocm/lib"
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "c", "consumer.c"), "-o", exe, "-L", PKG, "-lferret",
           f"-Wl,-rpath,{PKG}", f"-Wl,-rpath-link,{rocm_lib}"]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = rocm_lib + os.pathsep + env.get("LD_LIBRARY_PATH", "")
    run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "failures 0" in run.stdout and "FAILED" not in run.stdout
    return run.stdout


def test_headers_compile_as_c99_and_host_calls_behave(consumer_output):
    assert consumer_output.count("\n") > 40


def test_ctypes_mirrors_match_the_c_layouts(consumer_output):
    sizes = {m.group(1): int(m.group(2)) for m in re.finditer(r"^layout (\w+) sizeof (\d+)$", consumer_output, re.M)}
    fields = {(m.group(1), m.group(2)): (int(m.group(3)), int(m.group(4)))
              for m in re.finditer(r"^layout (\w+)\.(\w+) offset (\d+) size (\d+)$", consumer_output, re.M)}
    assert set(sizes) == set(MIRRORS)
    for name, cls in MIRRORS.items():
        assert ctypes.sizeof(cls) == sizes[name], name
        c_fields = [f for (s, f) in fields if s == name]
        assert len(c_fields) == len(cls._fields_), f"{name}: the C program and the mirror list different fields"
        for f in c_fields:
            desc = getattr(cls, RENAMED.get((name, f), f))
            assert (desc.offset, desc.size) == fields[(name, f)], f"{name}.{f}"


def test_constants_and_values_match_the_binding(consumer_output):
    val = {m.group(1): int(m.group(2)) for m in re.finditer(r"^value (\w+) (-?\d+)$", consumer_output, re.M)}
    for name in ("FERRET_OK", "FERRET_EINVAL", "FERRET_ESTATE", "FERRET_ENOMEM", "FERRET_EDEVICE", "FERRET_F32",
                 "FERRET_BF16_MASTER_F32", "FERRET_MAX_STAGES", "FERRET_ALIGN_ELEMS", "FERRET_ITERS_FULL",
                 "FERRET_RING_DEPTH_MINIMAL", "FERRET_NOALLOC_MAX_CHUNKS"):
        assert val[name] == getattr(B, name), name
    plan = B.ferret_plan_buckets([(5000, 0), (33, 0), (2048, 1), (7, 2), (4096, 2)], 3, [2, 1, 0], 2, 3, B.FERRET_F32, 0)
    assert val["n_chunks"] == plan.n_chunks and val["flat_elems"] == plan.flat_elems
    assert val["ring_elems"] == plan.ring_elems and val["workspace_bytes"] == plan.workspace_bytes
    for j in range(3):
        assert val[f"stage{j}_flat_offset"] == plan.stage_flat_offset(j)
        assert val[f"stage{j}_ring_offset"] == plan.stage_ring_offset(j)
        assert val[f"stage{j}_slot_stride"] == plan.stage_slot_stride(j)
        assert val[f"stage{j}_chunk_elems"] == plan.stage_chunk_elems(j)
        assert val[f"stage{j}_n_chunks"] == plan.stage_n_chunks(j)
    tuned = B.ferret_plan_buckets([(5000, 0), (33, 0), (2048, 1), (7, 2), (4096, 2)], 3, [2, 1, 0], B.FERRET_ITERS_FULL,
                                  B.FERRET_RING_DEPTH_MINIMAL, B.FERRET_BF16_MASTER_F32, 0,
                                  dict(chunk_bytes=32 * 1024, resident_cap=3, newest_from_master=1))
    assert val["tuned_stage0_chunk_elems"] == tuned.stage_chunk_elems(0)
    layers = [(1.0, 2.0, 1000.0, 500.0), (1.5, 2.5, 4000.0, 300.0), (0.5, 1.0, 2000.0, 200.0), (1.0, 1.5, 500.0, 10.0)]
    pipe = B.ferret_pipeline_plan(layers, 1.5, 1e9, 0.01, 1.0)
    assert val["pipeline_n_stages"] == pipe.n_stages and val["pipeline_n_workers"] == pipe.n_workers
    assert val["pipeline_n_moves"] == len(pipe.moves)
    assert val["pipeline_rate_micro"] == int(pipe.rate * 1e6 + 0.5)
