"""Pins for the oracle's "update lambda" block (Alg. 1 with eta_lambda > 0)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import ferret_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked_lambda.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        out[k] = [float(x) for x in v]
    return out


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def test_hand_worked_lambda_block():
    gold = _golden()
    lam, r, a, sums = O.lambda_update(_f32([2, 1]), _f32([1, 1]), _f32([1.5, 0.5]), 0.2, 0.5, 0.1,
                                      _f32([1, 0]), _f32([0.5, -1]))
    assert lam == pytest.approx(gold["lambda_new"][0], rel=1e-12)
    assert np.array_equal(r, _f32(gold["v_r_new"])) and np.array_equal(a, _f32(gold["v_a_new"]))
    assert sums[0] == gold["dot_a_dr"][0] and sums[1] == gold["dot_a_a"][0]


def test_lambda_step_is_gradient_descent_on_the_stated_objective():
    """lambda' - lambda = -eta_lambda * d/dlambda ||dv_r - lambda v_a||^2, derivative taken by central
    differences in exact rational arithmetic (exact for a quadratic)."""
    rng = np.random.default_rng(3)
    n = 7
    g = [Fraction(int(x), 8) for x in rng.integers(-20, 20, n)]
    vr = [Fraction(int(x), 8) for x in rng.integers(-20, 20, n)]
    va = [Fraction(int(x), 16) for x in rng.integers(-20, 20, n)]
    alpha, eta_l, lam = Fraction(3, 4), Fraction(1, 32), Fraction(1, 4)

    def objective(l):
        return sum(((1 - alpha) * (gi - ri) - l * ai) ** 2 for gi, ri, ai in zip(g, vr, va))

    h = Fraction(1, 2)
    derivative = (objective(lam + h) - objective(lam - h)) / (2 * h)
    want = lam - eta_l * derivative
    got, _, _, _ = O.lambda_update(_f32([float(x) for x in g]), _f32([0] * n), _f32([0] * n), float(lam),
                                   float(alpha), float(eta_l), _f32([float(x) for x in vr]),
                                   _f32([float(x) for x in va]))
    assert got == float(want)                 # every quantity is exactly representable
    assert objective(want) < objective(lam)   # and the step does descend


def test_exact_line_minimum_with_the_right_step_size():
    """With eta_lambda = 1 / (2 <v_a,v_a>) one step lands on the least-squares lambda (library lstsq)."""
    rng = np.random.default_rng(4)
    n = 200
    g, vr, va = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    alpha = 0.9
    dv = (1 - alpha) * (g.astype(np.float64) - vr)
    best = np.linalg.lstsq(va.astype(np.float64)[:, None], dv, rcond=None)[0][0]
    eta = 1.0 / (2.0 * float(va.astype(np.float64) @ va.astype(np.float64)))
    got, _, _, _ = O.lambda_update(g, g, g, 0.37, alpha, eta, vr, va)
    assert got == pytest.approx(best, rel=1e-10)
    again, _, _, _ = O.lambda_update(g, g, g, got, alpha, eta, vr, va)      # already at the minimum
    assert again == pytest.approx(got, rel=1e-10)


def test_moving_averages_converge_geometrically():
    """Constant inputs: after n calls v_r = (1 - alpha^n) g and v_a = (1 - alpha^n) g^2 (V1 - V0)
    (alpha = 3/4: every intermediate value is an exact binary fraction, and the two weights of the
    average differ, so swapping them shows)."""
    g, V0, V1 = _f32([2.0, -1.0]), _f32([1.0, 1.0]), _f32([1.25, 0.5])
    alpha = 0.75
    r, a = _f32([0, 0]), _f32([0, 0])
    for n in range(1, 9):
        _, r, a, _ = O.lambda_update(g, V0, V1, 0.2, alpha, 0.0, r, a)
        f = 1 - alpha ** n
        assert np.array_equal(r, _f32([2 * f, -1 * f]))
        assert np.array_equal(a, _f32([4 * 0.25 * f, 1 * -0.5 * f]))
    assert r[0] == np.float32(2 * (1 - 6561 / 65536))


def test_zero_learning_rate_keeps_lambda_and_matches_fixed_lambda_path():
    rng = np.random.default_rng(5)
    n = 300
    V = [rng.standard_normal(n).astype(np.float32) * 0.3 for _ in range(4)]
    g = rng.standard_normal(n).astype(np.float32)
    vr, va = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
    out = O.compensate_stage_adaptive(V, g, None, -1, 0.3, 0.9, 0.0, 0.01, vr, va)
    new, g_out, _ = O.compensate_stage_f32(V, g, -1, 0.3, 0.01)
    assert out["lam"] == 0.3 and np.array_equal(out["new"], new) and np.array_equal(out["g"], g_out)
    assert np.array_equal(out["v_r"], vr) and np.array_equal(out["v_a"], va)


def test_iterations_use_the_updated_lambda():
    V = [_f32([1.0]), _f32([1.5])]
    out = O.compensate_stage_adaptive(V, _f32([2.0]), None, -1, 0.2, 0.5, 0.1, 0.0, _f32([1.0]), _f32([0.5]))
    # dv_r = .5, <v_a,dv_r> = .25, <v_a,v_a> = .25: lambda' = .2 + .2(.25 - .05) = .24 ; g_1 = 2 + .24*4*.5 = 2.48
    assert out["lam"] == pytest.approx(0.24, rel=1e-12)
    assert out["g"][0] == pytest.approx(2.48, rel=1e-12)


def test_one_pass_ordering_uses_the_lambda_it_was_given():
    """Same hand-worked case with the lambda step applied after the iterations: lambda and the averages come
    out as before, the compensated gradient is the one of the old lambda."""
    V = [_f32([1.0]), _f32([1.5])]
    out = O.compensate_stage_adaptive(V, _f32([2.0]), None, -1, 0.2, 0.5, 0.1, 0.0, _f32([1.0]), _f32([0.5]),
                                      lambda_step_last=True)
    ref = O.compensate_stage_adaptive(V, _f32([2.0]), None, -1, 0.2, 0.5, 0.1, 0.0, _f32([1.0]), _f32([0.5]))
    assert out["lam"] == pytest.approx(0.24, rel=1e-12)
    assert out["g"][0] == pytest.approx(2.4, rel=1e-7)      # not 2.48
    assert np.array_equal(out["v_r"], ref["v_r"]) and np.array_equal(out["v_a"], ref["v_a"])


def test_one_pass_ordering_is_alg1_shifted_by_one_call():
    """With the weights held fixed (eta = 0) the lambda block sees the same inputs in either ordering, so the
    lambda sequences agree and call t of the one-pass ordering compensates with the lambda that Alg. 1's
    ordering used at call t-1."""
    rng = np.random.default_rng(11)
    n = 200
    V = [(rng.standard_normal(n) * 0.3).astype(np.float32) for _ in range(3)]
    state = {False: (0.2, np.zeros(n, np.float32), np.zeros(n, np.float32)),
             True: (0.2, np.zeros(n, np.float32), np.zeros(n, np.float32))}
    used = {False: [], True: []}
    for t in range(4):
        g = rng.standard_normal(n).astype(np.float32)
        for last in (False, True):
            lam, vr, va = state[last]
            out = O.compensate_stage_adaptive(V, g, None, -1, lam, 0.75, 0.05, 0.0, vr, va, lambda_step_last=last)
            # which lambda scaled this call's iterations: recover it from the first iteration on one element
            fixed = [O.compensate_stage_f32(V, g, -1, x, 0.0)[1] for x in (lam, out["lam"])]
            used[last].append(0 if np.array_equal(out["g"], fixed[0]) else 1)
            assert np.array_equal(out["g"], fixed[used[last][-1]])
            state[last] = (out["lam"], out["v_r"], out["v_a"])
        assert state[False][0] == state[True][0]
        assert np.array_equal(state[False][1], state[True][1]) and np.array_equal(state[False][2], state[True][2])
    # the first call has zero averages: lambda does not move and both fixed-lambda results coincide
    assert used[False][1:] == [1, 1, 1] and used[True][1:] == [0, 0, 0]


def test_staleness_zero_skips_the_block():
    out = O.compensate_stage_adaptive([_f32([1.0, 2.0])], _f32([1.0, 1.0]), None, -1, 0.2, 0.5, 0.1, 0.5,
                                      _f32([3.0, 3.0]), _f32([4.0, 4.0]))
    assert out["lam"] == 0.2 and np.array_equal(out["v_r"], _f32([3, 3])) and np.array_equal(out["v_a"], _f32([4, 4]))
    assert np.array_equal(out["new"], _f32([0.5, 1.5]))


def test_bf16_inputs_widen_exactly():
    import torch
    g = torch.tensor([2.0, 1.0]).to(torch.bfloat16)
    V0, V1 = torch.tensor([1.0, 1.0]).to(torch.bfloat16), torch.tensor([1.5, 0.5]).to(torch.bfloat16)
    lam, r, a, _ = O.lambda_update(g, V0, V1, 0.2, 0.5, 0.1, _f32([1, 0]), _f32([0.5, -1]), bf16=True)
    assert lam == pytest.approx(0.1, rel=1e-12)
    assert np.array_equal(r, _f32([1.5, 0.5])) and np.array_equal(a, _f32([1.25, -0.75]))
