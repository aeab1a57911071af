"""The planner pins must notice plausible mistakes in the planner oracle.

Each mutant is oracle/planner_oracle.py with ONE expression changed; the planner pins are run against it in a
child process (environment variable FERRET_PLANNER_ORACLE) and must fail.  CPU only.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "planner_oracle.py")
PINS = "tests/test_oracle_planner_pins.py"

MUTANTS = [
    ("recomputation missing from the delay of a gradient",
     "expo = -c * ((P + j) * S.t_f + (P - i + j) * S.t_b + r * (P - i + j) * S.t_f)",
     "expo = -c * ((P + j) * S.t_f + (P - i + j) * S.t_b)"),
    ("recomputation missing from the worker's period",
     "return math.exp(expo) * v_d / (lcm * (S.t_f + S.t_b + r * S.t_f))",
     "return math.exp(expo) * v_d / (lcm * (S.t_f + S.t_b))"),
    ("omission of later stages ignored in the update frequency",
     "lcm = _lcm(C.omit[n][k] + 1 for k in range(i, P))", "lcm = _lcm(C.omit[n][k] + 1 for k in range(i, i + 1))"),
    ("accumulated gradients not averaged", "out += S.w[i] / total_w * (1.0 / ca) * sum(", "out += S.w[i] / total_w * sum("),
    ("stage weight share dropped", "out += S.w[i] / total_w * (1.0 / ca) * sum(", "out += (1.0 / ca) * sum("),
    ("omitted stages still keep their versions",
     "versions = 1 + math.ceil((P - i - 1) / C.accum[n][i]) - C.omit[n][i]",
     "versions = 1 + math.ceil((P - i - 1) / C.accum[n][i])"),
    ("version count without the current weights",
     "versions = 1 + math.ceil((P - i - 1) / C.accum[n][i]) - C.omit[n][i]",
     "versions = math.ceil((P - i - 1) / C.accum[n][i]) - C.omit[n][i]"),
    ("recomputation frees every activation of the stage",
     "out += versions * (S.w[i] + S.a[i] - C.recompute[n] * S.a_inner[i])",
     "out += versions * (S.w[i] + S.a[i] - C.recompute[n] * S.a[i])"),
    ("worker 0 left out of the sums", "live = [n for n, d in enumerate(C.delay) if d >= 0]",
     "live = [n for n, d in enumerate(C.delay) if d > 0]"),
    ("accumulation raised by one instead of to the next useful value",
     "    return math.ceil(d / (cur - 1))", "    return ca + 1"),
    ("omission period off by one", "out.omit[n][j] = P - 1 - j", "out.omit[n][j] = P - j"),
    ("merit inverted", "merit = math.inf if dR >= 0 else dM / dR", "merit = math.inf if dR >= 0 else dR / dM"),
    ("worker count rounded down", "N = math.ceil((S.t_f + S.t_b + c_r * S.t_f) / t_d)",
     "N = max(1, math.floor((S.t_f + S.t_b + c_r * S.t_f) / t_d))"),
    ("stage closed when the bound is reached instead of exceeded", "        if t_sum > t_c:", "        if t_sum >= t_c:"),
    ("stage times summed instead of the slowest stage",
     "return Stages(w, a, inner, max(tf), max(tb))", "return Stages(w, a, inner, sum(tf), sum(tb))"),
    ("bounds below the largest layer kept", "            if t_c >= floor_:", "            if t_c >= 0:"),
]


def _run_pins(path=None):
    env = dict(os.environ)
    if path:
        env["FERRET_PLANNER_ORACLE"] = path
    else:
        env.pop("FERRET_PLANNER_ORACLE", None)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", PINS], cwd=ROOT, env=env,
                          capture_output=True, text=True)


def test_unmodified_planner_oracle_passes_through_the_same_harness(tmp_path):
    copy = tmp_path / "planner_oracle_copy.py"
    copy.write_text(open(SRC).read())
    r = _run_pins(str(copy))
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_planner_pins_catch_mutant(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site not unique: {old!r}"
    mutant = tmp_path / "planner_oracle_mutant.py"
    mutant.write_text(text.replace(old, new))
    r = _run_pins(str(mutant))
    assert r.returncode != 0, f"no planner pin noticed: {name}"
