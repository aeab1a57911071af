"""The pins must notice plausible mistakes in the oracle.

Each mutant is the oracle's C source with ONE line changed (a dropped term, a flipped sign, a wrong
index, truncation instead of rounding ...), compiled to a scratch library; the pin tests are then run
against it in a child process (environment variable FERRET_ORACLE_LIB) and must fail.  The mistakes
are planted in the oracle, on the CPU, never in the GPU path.
"""
import os
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "ferret_oracle.c")
PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_lambda_pins.py", "tests/test_oracle_accumulate_pins.py",
        "tests/test_oracle_penalized_pins.py"]

MUTANTS = [
    ("square of the original gradient instead of the current iterate",
     "static double compensate_one(double g, const double *v, int32_t tau, int32_t Kp, double lambda)\n{",
     "static double compensate_one(double g, const double *v, int32_t tau, int32_t Kp, double lambda)\n{\n    const double g_first = g;",
     "        g = g + lambda * g * g * dtheta;", "        g = g + lambda * g_first * g_first * dtheta;"),
    ("drift taken as old minus new", None, None,
     "        double dtheta = v[s_hi] - v[s_lo];", "        double dtheta = v[s_lo] - v[s_hi];"),
    ("gradient not squared", None, None,
     "        g = g + lambda * g * g * dtheta;", "        g = g + lambda * g * dtheta;"),
    ("lambda dropped", None, None,
     "        g = g + lambda * g * g * dtheta;", "        g = g + g * g * dtheta;"),
    ("compensation term subtracted", None, None,
     "        g = g + lambda * g * g * dtheta;", "        g = g - lambda * g * g * dtheta;"),
    ("segment boundaries rounded up", None, None,
     "    return (int32_t)(((int64_t)i * (int64_t)tau) / (int64_t)Kp);",
     "    return (int32_t)(((int64_t)i * (int64_t)tau + Kp - 1) / (int64_t)Kp);"),
    ("iteration count not capped by the staleness", None, None,
     "    return K < tau ? K : tau;", "    return K;"),
    ("update applied to the stale snapshot", None, None,
     "        double updated = v[tau] - eta * g;", "        double updated = v[0] - eta * g;"),
    ("update uses the uncompensated gradient", None, None,
     "        double updated = v[tau] - eta * g;", "        double updated = v[tau] - eta * g_start;"),
    ("gradient ascent", None, None,
     "        double updated = v[tau] - eta * g;", "        double updated = v[tau] + eta * g;"),
    ("bf16 by truncation", None, None,
     "    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))", "    if (0)"),
    ("bf16 ties away from zero", None, None,
     "    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u)))", "    if (rest >= 0x8000u)"),
    ("bf16 update bypasses the master", None, None,
     "        double updated = (double)master[e] - eta * g;", "        double updated = v[tau] - eta * g;"),
    ("lambda step with the wrong sign", None, None,
     "    double lambda_new = lambda - eta_lambda * derivative;", "    double lambda_new = lambda + eta_lambda * derivative;"),
    ("derivative without the factor two", None, None,
     "    double derivative = -2.0 * (dot_a_dr - lambda * dot_a_a);", "    double derivative = -(dot_a_dr - lambda * dot_a_a);"),
    ("dv_r without the (1 - alpha) factor", None, None,
     "        double dv_r = (1.0 - alpha) * (g - (double)v_r[e]);", "        double dv_r = (g - (double)v_r[e]);"),
    ("moving averages swapped weights", None, None,
     "        double r = alpha * (double)v_r[e] + (1.0 - alpha) * g;", "        double r = (1.0 - alpha) * (double)v_r[e] + alpha * g;"),
    ("v_a built from the total drift sign-flipped", None, None,
     "        double first_step = widen_at(V1, e, bf16) - widen_at(V0, e, bf16);",
     "        double first_step = widen_at(V0, e, bf16) - widen_at(V1, e, bf16);"),
    ("accumulated sum ignored at the update", None, None,
     "        float updated = (float)(base - eta * scale * total);", "        float updated = (float)(base - eta * scale * g);"),
    ("sum not cleared after the update", None, None,
     "        accum_out[e] = 0.0f;", "        accum_out[e] = (float)total;"),
    ("scale not applied", None, None,
     "        float updated = (float)(base - eta * scale * total);", "        float updated = (float)(base - eta * total);"),
    ("gap taken with its sign", None, None,
     "        double gap = fabs(newest - widen_at(V0, e, bf16)) * inv_c + 1.0;",
     "        double gap = (newest - widen_at(V0, e, bf16)) * inv_c + 1.0;"),
    ("gap without the + 1", None, None,
     "        double gap = fabs(newest - widen_at(V0, e, bf16)) * inv_c + 1.0;",
     "        double gap = fabs(newest - widen_at(V0, e, bf16)) * inv_c;"),
    ("penalty multiplies instead of divides", None, None,
     "        double g = scale * widen_at(g0, e, bf16) / gap;", "        double g = scale * widen_at(g0, e, bf16) * gap;"),
]


def _build(source_text, out):
    with tempfile.NamedTemporaryFile("w", suffix=".c", delete=False) as f:
        f.write(source_text)
        path = f.name
    try:
        subprocess.run(["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-o", out, path,
                        "-lm"], check=True, capture_output=True)
    finally:
        os.unlink(path)


def _run_pins(lib, pins=PINS):
    env = dict(os.environ, FERRET_ORACLE_LIB=lib)
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins],
                          cwd=ROOT, env=env, capture_output=True, text=True)


def test_unmodified_source_passes_through_the_same_harness(tmp_path):
    lib = str(tmp_path / "clean.so")
    _build(open(SRC).read(), lib)
    r = _run_pins(lib)
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,pre_old,pre_new,old,new", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_pins_catch_mutant(tmp_path, name, pre_old, pre_new, old, new):
    src = open(SRC).read()
    if pre_old:
        assert pre_old in src
        src = src.replace(pre_old, pre_new)
    assert src.count(old) >= 1, f"mutation site for '{name}' not found: the oracle changed, update this test"
    src = src.replace(old, new)
    lib = str(tmp_path / "mutant.so")
    _build(src, lib)
    # run the pin file of the mutated block first (cheap); any failing pin is enough
    site = src.index(new)
    first = PINS[3] if site > src.index("==== step-size-penalising") else (
        PINS[2] if site > src.index("==== gradient accumulation") else (
            PINS[1] if site > src.index("==== adaptive lambda") else PINS[0]))
    r = _run_pins(lib, [first])
    if r.returncode == 0:
        r = _run_pins(lib)
    assert r.returncode != 0, f"no pin noticed: {name}"
