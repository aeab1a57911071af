"""Pins for the oracle's step-size-penalising comparison methods (Step-Aware, Gap-Aware as read here)."""
import numpy as np
import pytest

from oracle import ferret_oracle as O


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def _rand(n, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


def test_hand_worked_gap_aware():
    # V[0] = 1, V[tau] = 1.5, C = 0.25: G = 0.5/0.25 + 1 = 3 ; g = 6: step 6/3 = 2 ; eta 0.125: 1.5 - 0.25 = 1.25
    out = O.penalized_stage(_f32([1.0]), _f32([1.5]), _f32([6.0]), None, 0.125, 1.0, 4.0)
    assert out["g"][0] == 2.0 and out["new"][0] == np.float32(1.25)
    # the gap is a distance: the same with the weight having moved the other way
    out = O.penalized_stage(_f32([2.0]), _f32([1.5]), _f32([6.0]), None, 0.125, 1.0, 4.0)
    assert out["g"][0] == 2.0 and out["new"][0] == np.float32(1.25)


def test_hand_worked_step_aware():
    # tau = 4: eta/4.  V[tau] = 2, g = -8, eta = 0.5: 2 - 0.125 * (-8) = 3
    out = O.penalized_stage(_f32([0.0]), _f32([2.0]), _f32([-8.0]), None, 0.5, 0.25, 0.0)
    assert out["g"][0] == -2.0 and out["new"][0] == np.float32(3.0)


def test_no_penalty_is_plain_sgd_and_matches_the_main_oracle_without_iterations():
    n = 400
    V0, V1, g = _rand(n, 1, 0.3), _rand(n, 2, 0.3), _rand(n, 3)
    out = O.penalized_stage(V0, V1, g, None, 0.05, 1.0, 0.0)
    new, g_ref, _ = O.compensate_stage_f32([V0, V1], g, 0, 0.5, 0.05)          # K = 0: no compensation
    assert np.array_equal(out["new"], new) and np.array_equal(out["g"], g_ref)
    # zero gap: the gap-aware divisor is exactly 1
    out = O.penalized_stage(V1, V1, g, None, 0.05, 1.0, 123.0)
    assert np.array_equal(out["new"], new)


def test_penalty_only_ever_shrinks_the_step():
    n = 1000
    V0, V1, g = _rand(n, 4, 0.3), _rand(n, 5, 0.3), _rand(n, 6)
    out = O.penalized_stage(V0, V1, g, None, 0.05, 1.0, 7.0)
    assert np.all(np.abs(out["g"]) <= np.abs(g.astype(np.float64)))
    gap = np.abs(V1.astype(np.float64) - V0.astype(np.float64)) * 7.0 + 1.0
    np.testing.assert_allclose(out["g"] * gap, g.astype(np.float64), rtol=1e-14)


def test_bf16_goes_through_the_master():
    import torch
    bf = lambda x: torch.tensor(x).to(torch.bfloat16)
    out = O.penalized_stage(bf([1.0]), bf([1.5]), bf([6.0]), _f32([1.50390625]), 2.0 ** -8, 1.0, 4.0, bf16=True)
    # step 2 ; master 1.50390625 - 2/256 = 1.49609375 = 0x3FBF8000 : tie, odd below -> rounds up to 0x3FC0
    assert out["g"][0] == 2.0 and out["master"][0] == np.float32(1.49609375) and out["new"][0] == 0x3FC0
