"""Pins for the oracle's gradient-accumulation path (T2) and for the version count the paper gives."""
import math

import numpy as np
import pytest

from oracle import ferret_oracle as O


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def _rand(n, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


def test_single_accumulation_step_is_algorithm_1():
    n = 500
    V = [_rand(n, s, 0.3) for s in range(4)]
    g = _rand(n, 9)
    out = O.accumulate_stage(V, g, None, -1, 0.4, 0.05, 1.0, True, np.zeros(n, np.float32))
    new, g_ref, _ = O.compensate_stage_f32(V, g, -1, 0.4, 0.05)
    assert np.array_equal(out["new"], new) and np.array_equal(out["g"], g_ref)
    assert not out["accum"].any()


def test_hand_worked_two_arrivals():
    # current version 2.0.  Arrival 1: g=1, taken one version ago (1.5 -> 2.0), lambda .5: 1 + .5*1*.5 = 1.25
    # arrival 2: g=-2, taken on the current version (tau=0): stays -2.  sum = -0.75
    # mean (scale .5), eta .1: theta = 2.0 - .1*.5*(-.75) = 2.0375
    a1 = O.accumulate_stage([_f32([1.5]), _f32([2.0])], _f32([1.0]), None, -1, 0.5, 0.1, 0.5, False, _f32([0.0]))
    assert a1["accum"][0] == np.float32(1.25) and a1["g"][0] == 1.25 and "new" not in a1
    a2 = O.accumulate_stage([_f32([2.0])], _f32([-2.0]), None, -1, 0.5, 0.1, 0.5, True, a1["accum"])
    assert a2["new"][0] == np.float32(2.0375) and a2["accum"][0] == 0.0


def test_without_compensation_accumulation_is_sgd_on_the_summed_gradient():
    n, c = 300, 4
    V = [_rand(n, 20 + s, 0.3) for s in range(3)]
    gs = [_rand(n, 30 + k) for k in range(c)]
    acc = np.zeros(n, np.float32)
    for k, g in enumerate(gs):
        out = O.accumulate_stage(V[k % 3:], g, None, -1, 0.0, 0.01, 1.0, k == c - 1, acc)
        acc = out["accum"]
    want = V[-1].astype(np.float64) - 0.01 * np.sum([g.astype(np.float64) for g in gs], axis=0)
    np.testing.assert_allclose(out["new"], want, rtol=2e-6, atol=1e-7)      # fp32 running sum


def test_bf16_update_goes_through_the_master():
    import torch
    V = [torch.tensor([1.0]).to(torch.bfloat16), torch.tensor([1.5]).to(torch.bfloat16)]
    out = O.accumulate_stage(V, torch.tensor([2.0]).to(torch.bfloat16), _f32([1.50390625]), -1, 0.5, 2.0 ** -8, 1.0,
                             True, _f32([1.0]), bf16=True)
    # g_1 = 2 + .5*4*.5 = 3 ; sum = 4 ; master = 1.50390625 - 4/256 = 1.48828125 = 0x3FBE8000 -> tie -> even 0x3FBE
    assert out["g"][0] == 3.0 and out["master"][0] == np.float32(1.48828125) and out["new"][0] == 0x3FBE


@pytest.mark.parametrize("P", [2, 3, 5, 8])
@pytest.mark.parametrize("ca", [1, 2, 3, 4])
def test_versions_needed_match_the_papers_count(P, ca):
    """Stage j of a P-stage pipeline sees its gradient P-j-1 micro-steps after the forward pass.  With
    an update every c^a micro-steps, the staleness counted in versions never exceeds
    ceil((P-j-1)/c^a), so 1 + ceil((P-j-1)/c^a) stored versions suffice (and are reached)."""
    for j in range(P):
        d = P - j - 1
        worst = 0
        for m in range(0, 10 * ca):                     # micro-step of the forward pass
            version_at_forward = m // ca
            version_at_arrival = (m + d) // ca
            worst = max(worst, version_at_arrival - version_at_forward)
        assert worst == math.ceil(d / ca)


def test_accumulation_with_lambda_block_hand_worked():
    """g = 2, V = (1, 1.5), v_r = 1, v_a = .5, alpha = .5, eta_lambda = .1, lambda = .2:
    dv_r = .5, <v_a,dv_r> = .25, <v_a,v_a> = .25, lambda' = .2 + .2 (.25 - .05) = .24, g_1 = 2 + .24*4*.5 = 2.48;
    running sum 1 + 2.48 = 3.48; update with scale .5, eta .1: 1.5 - .1*.5*3.48 = 1.326."""
    f = lambda *x: np.asarray(x, dtype=np.float32)
    out = O.accumulate_stage_adaptive([f(1.0), f(1.5)], f(2.0), None, -1, 0.2, 0.5, 0.1, 0.1, 0.5, True, f(1.0),
                                      f(1.0), f(0.5))
    assert out["lam"] == pytest.approx(0.24, rel=1e-12)
    assert out["g"][0] == pytest.approx(2.48, rel=1e-7)
    assert out["new"][0] == np.float32(1.326)
    assert out["accum"][0] == 0.0
    assert out["v_r"][0] == np.float32(1.5) and out["v_a"][0] == np.float32(0.25 + 0.5 * 4 * 0.5)
    # not the last arrival of its group: only the sum moves
    out = O.accumulate_stage_adaptive([f(1.0), f(1.5)], f(2.0), None, -1, 0.2, 0.5, 0.1, 0.1, 0.5, False, f(1.0),
                                      f(1.0), f(0.5))
    assert out["accum"][0] == np.float32(3.48) and "new" not in out


def test_accumulation_with_zero_lambda_rate_or_no_staleness_is_plain_accumulation():
    rng = np.random.default_rng(3)
    n = 100
    V = [(rng.standard_normal(n) * 0.2).astype(np.float32) for _ in range(3)]
    g, acc = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
    vr, va = rng.standard_normal(n).astype(np.float32), rng.standard_normal(n).astype(np.float32)
    a = O.accumulate_stage_adaptive(V, g, None, -1, 0.3, 0.9, 0.0, 0.01, 1.0, True, acc, vr, va)
    b = O.accumulate_stage(V, g, None, -1, 0.3, 0.01, 1.0, True, acc)
    assert a["lam"] == 0.3 and np.array_equal(a["new"], b["new"]) and np.array_equal(a["v_r"], vr)
    a = O.accumulate_stage_adaptive(V[-1:], g, None, -1, 0.3, 0.9, 0.1, 0.01, 1.0, True, acc, vr, va)
    assert a["lam"] == 0.3 and np.array_equal(a["v_a"], va)
