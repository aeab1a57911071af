"""The host half of the library under sanitizers (no GPU): ferret_host.cpp and ferret_planner.cpp are compiled with
the host C++ compiler together with stand-in launchers and a driver that runs the host path of every entry point
(tests/sanitize/), once with AddressSanitizer + UndefinedBehaviorSanitizer and once, for the planner's worker
threads, with ThreadSanitizer.  A report from a sanitizer or a failed check in the driver fails the test."""
import os
import shutil
import subprocess

import pytest

from paper_2503_12053_amd import build


@pytest.mark.parametrize("kind,what", [("address", "all"), ("thread", "planner")])
def test_host_code_runs_clean_under_sanitizer(kind, what, tmp_path):
    if shutil.which("g++") is None and shutil.which("c++") is None:
        pytest.skip("no host C++ compiler")
    probe = tmp_path / "probe.cpp"
    probe.write_text("int main() { return 0; }\n")
    flags = build.SANITIZERS[kind]
    if subprocess.run([shutil.which("g++") or "c++", *flags, str(probe), "-o", str(tmp_path / "probe")],
                      capture_output=True).returncode != 0:
        pytest.skip(f"the host compiler has no {flags[0]} runtime")
    exe = build.build_sanitized(kind, str(tmp_path / f"host_driver_{kind}"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", TSAN_OPTIONS="halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, what], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-4000:]
    assert "failures 0" in run.stdout
    assert "Sanitizer" not in run.stderr, run.stderr[-4000:]
