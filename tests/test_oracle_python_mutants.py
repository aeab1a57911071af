"""The pins must also notice mistakes in the Python layer of the oracle (the order in which Alg. 1's blocks
are composed, the ring of versions): one expression of oracle/ferret_oracle.py is changed in a copy, the copy
shadows the real module in a child process, and the pin tests must fail.  CPU only."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ferret_oracle.py")
PINS = ["test_oracle_pins.py", "test_oracle_lambda_pins.py", "test_oracle_accumulate_pins.py"]

MUTANTS = [
    ("iterations use the lambda from before its step",
     "    lam_used = float(lam) if lambda_step_last else lam_new\n    if bf16:",
     "    lam_used = float(lam)\n    if bf16:"),
    ("one-pass ordering ignored",
     "    lam_used = float(lam) if lambda_step_last else lam_new\n    if bf16:",
     "    lam_used = lam_new\n    if bf16:"),
    ("accumulation compensates with the lambda from before its step",
     "    lam_used = float(lam) if lambda_step_last else lam_new\n    out = accumulate_stage(",
     "    lam_used = float(lam)\n    out = accumulate_stage("),
    ("lambda block not skipped without staleness... and run without a learning rate",
     "    if eta_lambda > 0 and tau >= 1:\n        lam_new, r_new, a_new, sums = lambda_update(",
     "    if tau >= 1:\n        lam_new, r_new, a_new, sums = lambda_update("),
    ("warm-up: one version too many assumed", "        return min(self.tau[j], len(self.versions[j]) - 1)",
     "        return min(self.tau[j], len(self.versions[j]))"),
    ("ring keeps one version too few", "        if len(self.versions[j]) > self.R:", "        if len(self.versions[j]) >= self.R:"),
    ("window taken from the oldest versions", "        window = held[len(held) - 1 - tau:]", "        window = held[:tau + 1]"),
    ("empty loop reports boundary 0", "    if Kp == 0:\n        return [tau]", "    if Kp == 0:\n        return [0]"),
]


def _run_pins(shadow_root):
    env = dict(os.environ)
    env["PYTHONPATH"] = os.pathsep.join([shadow_root, ROOT])
    env["FERRET_ORACLE_LIB"] = os.path.join(ROOT, "oracle", "libferret_oracle.so")
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + [os.path.join(ROOT, "tests", p) for p in PINS]
    return subprocess.run(cmd, cwd=shadow_root, env=env, capture_output=True, text=True)


def _shadow(tmp_path, text):
    pkg = tmp_path / "oracle"
    pkg.mkdir()
    (pkg / "__init__.py").write_text("")
    (pkg / "ferret_oracle.py").write_text(text)
    shutil.copy(os.path.join(ROOT, "oracle", "planner_oracle.py"), pkg / "planner_oracle.py")
    return str(tmp_path)


@pytest.fixture(scope="module", autouse=True)
def _built():
    from oracle import ferret_oracle
    ferret_oracle.build()


def test_unmodified_copy_passes_and_is_the_module_under_test(tmp_path):
    text = open(SRC).read()
    r = _run_pins(_shadow(tmp_path, text))
    assert r.returncode == 0, r.stdout[-2000:]
    # the shadow really is what the pins import: a copy that cannot be imported must break them
    broken = tmp_path / "b"
    broken.mkdir()
    r = _run_pins(_shadow(broken, "raise ImportError('shadow module reached')\n"))
    assert r.returncode != 0 and "shadow module reached" in (r.stdout + r.stderr)


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_python_level_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not unique: {old!r}"
    r = _run_pins(_shadow(tmp_path, text.replace(old, new)))
    assert r.returncode != 0, f"no pin noticed: {name}"
