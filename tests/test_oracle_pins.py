"""Pins for the CPU oracle: what the paper and the mathematics fix about its results.

Each test names the fact it checks.  A plausible mistake in the oracle (dropped term,
wrong sign of the drift, squared original gradient instead of the current iterate,
versions indexed from the wrong end, wrong segment, update applied to the wrong version)
fails at least one of them.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import ferret_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            out.append([c.strip() for c in line.split("|")])
    return out


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def _stage(versions, g, K, lam, eta):
    V = [_f32(v).reshape(-1) for v in versions]
    return O.compensate_stage_f32(V, _f32(g).reshape(-1), K, lam, eta)


# ---------------------------------------------------------------------------------------
# hand-worked values (tests/golden/hand_worked_scalars.txt)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("row", _rows("hand_worked_scalars.txt"))
def test_hand_worked_scalars(row):
    g0, lam, eta, versions, K, iterates, theta_new = row
    V = [float(x) for x in versions.split()]
    want_g = [float(x) for x in iterates.split()]
    new, g_out, _ = _stage([[v] for v in V], [float(g0)], int(K), float(lam), float(eta))
    # inputs pass through fp32 storage, so agreement is to fp32 input rounding
    expect_g = want_g[-1] if want_g else float(g0)
    assert g_out[0] == pytest.approx(expect_g, rel=3e-6)
    assert float(new[0]) == pytest.approx(float(theta_new), rel=3e-7, abs=1e-7)
    # every printed intermediate iterate: run the oracle truncated to the first i segments
    if want_g and int(K) >= len(V) - 1:
        for i, gi in enumerate(want_g, start=1):
            _, g_i, _ = _stage([[v] for v in V[: i + 1]], [float(g0)], -1, float(lam), float(eta))
            assert g_i[0] == pytest.approx(gi, rel=3e-6)


@pytest.mark.parametrize("row", _rows("segment_boundaries.txt"))
def test_segment_boundaries_golden(row):
    tau, K, s = int(row[0]), int(row[1]), [int(x) for x in row[2].split()]
    assert O.segment_boundaries(tau, K) == s


@pytest.mark.parametrize("tau", range(1, 20))
@pytest.mark.parametrize("K", [-1, 1, 2, 3, 4, 7, 50])
def test_segment_boundaries_properties(tau, K):
    s = O.segment_boundaries(tau, K)
    Kp = tau if K < 0 else min(K, tau)
    assert len(s) == Kp + 1 and s[0] == 0 and s[-1] == tau
    assert all(b > a for a, b in zip(s, s[1:]))          # every segment is non-empty
    if Kp == tau:
        assert s == list(range(tau + 1))                  # Alg. 1: adjacent versions


def test_exact_rational_recurrence():
    """Inputs that are exact in fp32 and small enough that every double operation is exact:
    the oracle must reproduce exact rational arithmetic bit for bit."""
    g0, lam = Fraction(3, 2), Fraction(1, 4)
    V = [Fraction(1), Fraction(5, 4), Fraction(3, 4), Fraction(7, 8)]
    g = g0
    for a, b in zip(V, V[1:]):
        g = g + lam * g * g * (b - a)
    eta = Fraction(1, 8)
    theta = V[-1] - eta * g
    new, g_out, norms = _stage([[float(v)] for v in V], [float(g0)], -1, float(lam), float(eta))
    assert g_out[0] == float(g)                            # exact
    assert float(new[0]) == float(np.float32(float(theta)))
    assert norms[0] == float(g0 * g0)
    assert norms[1] == pytest.approx(float(g * g), rel=1e-15)
    assert norms[2] == float((V[-1] - V[0]) ** 2)


# ---------------------------------------------------------------------------------------
# invariants the paper states
# ---------------------------------------------------------------------------------------
def _rand(n, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


def test_zero_drift_leaves_gradient_unchanged():
    """Zero-order case (Sec. 'Gradients Compensation via Taylor Series Expansion'):
    if the weights did not move, the stale gradient is the gradient."""
    n = 1000
    w, g = _rand(n, 1, 0.05), _rand(n, 2)
    for tau in (1, 3, 6):
        for K in (-1, 1, 2):
            new, g_out, norms = _stage([w] * (tau + 1), g, K, 0.5, 0.01)
            assert np.array_equal(g_out, g.astype(np.float64))
            assert np.array_equal(new, (w.astype(np.float64) - 0.01 * g.astype(np.float64)).astype(np.float32))
            assert norms[2] == 0.0 and norms[0] == norms[1]


def test_zero_lambda_leaves_gradient_unchanged():
    n = 1000
    g = _rand(n, 3)
    V = [_rand(n, 10 + s, 0.05) for s in range(4)]
    new, g_out, _ = _stage(V, g, -1, 0.0, 0.01)
    assert np.array_equal(g_out, g.astype(np.float64))
    assert np.array_equal(new, (V[-1].astype(np.float64) - 0.01 * g.astype(np.float64)).astype(np.float32))


def test_staleness_zero_is_plain_sgd():
    """Alg. 1 with tau = 0: the loop is empty and the update is theta - eta g."""
    n = 777
    w, g = _rand(n, 4, 0.05), _rand(n, 5)
    for K in (-1, 0, 1, 3):
        new, g_out, norms = _stage([w], g, K, 0.5, 0.1)
        ref = torch.from_numpy(w).double() - 0.1 * torch.from_numpy(g).double()
        assert np.array_equal(new, ref.float().numpy())
        assert np.array_equal(g_out, g.astype(np.float64))
        assert norms[2] == 0.0


def test_zero_gradient_is_a_fixed_point():
    n = 100
    V = [_rand(n, 20 + s) for s in range(5)]
    new, g_out, norms = _stage(V, np.zeros(n, np.float32), -1, 0.5, 0.01)
    assert not g_out.any() and np.array_equal(new, V[-1]) and norms[0] == 0 and norms[1] == 0


def test_single_iteration_closed_form():
    """K = 1 (or tau = 1): g + lambda g^2 (theta_current - theta_stale), Eq.
    'gt-taylor-expansion-approximation' applied once across the whole drift."""
    n = 513
    g = _rand(n, 6).astype(np.float64)
    for tau in (1, 2, 5):
        V = [_rand(n, 30 + s, 0.3) for s in range(tau + 1)]
        new, g_out, _ = _stage(V, g.astype(np.float32), 1, 0.37, 0.05)
        g32 = g.astype(np.float32).astype(np.float64)
        closed = g32 + 0.37 * g32 * g32 * (V[-1].astype(np.float64) - V[0].astype(np.float64))
        np.testing.assert_allclose(g_out, closed, rtol=1e-14)
        np.testing.assert_allclose(new, V[-1].astype(np.float64) - 0.05 * closed, rtol=1e-6)


def test_full_iterations_equal_adjacent_pair_cascade():
    """K >= tau is Alg. 1's loop: one application per adjacent pair, each fed the previous
    output.  Built here from tau successive single-pair oracle calls (tau = 1 each, eta = 0
    so the returned 'weights' are unused) instead of re-typing the formula."""
    n, tau, lam = 300, 5, 0.41
    V = [_rand(n, 40 + s, 0.2) for s in range(tau + 1)]
    g0 = _rand(n, 7)
    _, g_all, _ = _stage(V, g0, -1, lam, 0.0)
    # cascade of closed-form single steps in double
    g = g0.astype(np.float64)
    for s in range(tau):
        d = V[s + 1].astype(np.float64) - V[s].astype(np.float64)
        g = g + lam * g * g * d
    np.testing.assert_allclose(g_all, g, rtol=1e-13)
    for K in (tau, tau + 1, 99):
        _, g_k, _ = _stage(V, g0, K, lam, 0.0)
        assert np.array_equal(g_k, g_all)


def test_iterates_use_current_gradient_not_original():
    """The cascade squares the current iterate.  If it squared g_0 every time, the
    iterates would telescope to the single-step result; they must not."""
    V = [[1.0], [1.1], [0.9], [0.95]]
    _, g_full, _ = _stage(V, [2.0], -1, 0.5, 0.0)
    _, g_single, _ = _stage(V, [2.0], 1, 0.5, 0.0)
    assert abs(g_full[0] - g_single[0]) > 0.1              # 1.7896 vs 1.9


def test_version_order_matters():
    """Reversing the stored versions flips every drift: a wrong-end index shows here."""
    V = [[1.0], [1.1], [0.9], [0.95]]
    _, g_fwd, _ = _stage(V, [2.0], -1, 0.5, 0.0)
    _, g_rev, _ = _stage(V[::-1], [2.0], -1, 0.5, 0.0)
    assert g_fwd[0] == pytest.approx(1.7896164, rel=1e-6)
    # reversed: drifts -0.05, +0.2, -0.1 : 1.9 ; 1.9+.5*3.61*.2 = 2.261 ; 2.261-.05*5.112121 = 2.00539395
    assert g_rev[0] == pytest.approx(2.00539395, rel=1e-6)


def test_without_iterations_only_the_newest_version_is_a_boundary():
    """K' = 0 leaves only Alg. 1's update line, which reads the current weights V[tau] and nothing else."""
    assert O.segment_boundaries(5, 0) == [5]
    assert O.segment_boundaries(0, 3) == [0] and O.segment_boundaries(0, -1) == [0]


def test_update_uses_newest_version():
    V = [[10.0], [20.0], [30.0]]
    new, _, norms = _stage(V, [0.0], -1, 0.5, 0.01)
    assert new[0] == 30.0 and norms[2] == 400.0


def test_continuum_limit():
    """Equal segment drifts D/K: the recurrence is forward Euler on dg/ds = lambda D g^2,
    whose solution at s = 1 is g_0 / (1 - lambda g_0 D); the error falls like 1/K."""
    g0, lam, D = 2.0, 0.5, 0.125              # D/K exact in fp32 for K a power of two
    limit = g0 / (1 - lam * g0 * D)
    errs = []
    for K in (1, 2, 4, 8, 64, 512):
        V = [[1.0 + D * i / K] for i in range(K + 1)]
        _, g, _ = _stage(V, [g0], -1, lam, 0.0)
        errs.append(limit - g[0])
    assert errs[0] == pytest.approx(limit - 2.25, abs=1e-12)      # K = 1: 2 + .5*4*.125
    assert all(e > 0 for e in errs)                                # Euler undershoots a convex solution
    assert all(b < a for a, b in zip(errs, errs[1:]))
    assert errs[-1] < 1e-3
    # first-order convergence: error(64) / error(512) ~ 8
    assert errs[4] / errs[5] == pytest.approx(8.0, rel=0.05)


def test_norms_match_library_dot_products():
    n = 4097
    V = [_rand(n, 50 + s, 0.3) for s in range(4)]
    g = _rand(n, 8)
    _, g_out, norms = _stage(V, g, 2, 0.3, 0.01)
    g64 = g.astype(np.float64)
    gap = V[-1].astype(np.float64) - V[0].astype(np.float64)
    assert norms[0] == pytest.approx(float(g64 @ g64), rel=1e-12)
    assert norms[1] == pytest.approx(float(g_out @ g_out), rel=1e-12)
    assert norms[2] == pytest.approx(float(gap @ gap), rel=1e-12)


def test_threads_do_not_change_elementwise_results():
    n = 10007
    V = [_rand(n, 60 + s, 0.3) for s in range(3)]
    g = _rand(n, 9)
    a = O.compensate_stage_f32(V, g, -1, 0.5, 0.01, n_threads=1)
    b = O.compensate_stage_f32(V, g, -1, 0.5, 0.01, n_threads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    np.testing.assert_allclose(a[2], b[2], rtol=1e-12)


def test_nan_inf_propagate():
    V = [[1.0, 1.0], [2.0, 2.0]]
    new, g_out, _ = _stage(V, [np.nan, np.inf], -1, 0.5, 0.01)
    assert np.isnan(g_out[0]) and np.isnan(new[0])
    assert np.isinf(g_out[1]) and np.isinf(new[1])


# ---------------------------------------------------------------------------------------
# bf16 storage
# ---------------------------------------------------------------------------------------
def test_bf16_rounding_hand_built_ties():
    # 1.0 = 0x3F800000.  bf16 spacing at 1.0 is 2^-7.
    def bits(x):
        return O.f32_to_bf16_bits(x)
    assert bits(1.0) == 0x3F80
    assert bits(np.float32(1.0 + 2.0 ** -8)) == 0x3F80          # exact tie, even mantissa below -> down
    assert bits(np.float32(1.0 + 2.0 ** -7 + 2.0 ** -8)) == 0x3F82   # tie, odd below -> up to even
    assert bits(np.float32(1.0 + 2.0 ** -8 + 2.0 ** -20)) == 0x3F81  # just above the tie -> up
    assert bits(np.float32(1.0 + 2.0 ** -8 - 2.0 ** -20)) == 0x3F80  # just below the tie -> down
    assert bits(-0.0) == 0x8000 and bits(0.0) == 0x0000
    assert bits(np.float32(np.inf)) == 0x7F80 and bits(np.float32(-np.inf)) == 0xFF80
    assert bits(np.float32(3.3895314e38)) == 0x7F7F                 # bf16 max
    assert bits(np.float32(3.4028235e38)) == 0x7F80                 # fp32 max rounds to inf
    nan_bits = bits(np.float32(np.nan))
    assert (nan_bits & 0x7F80) == 0x7F80 and (nan_bits & 0x007F) != 0


def test_bf16_rounding_matches_library_conversion():
    rng = np.random.default_rng(0)
    raw = rng.integers(0, 2 ** 32, size=20000, dtype=np.uint64).astype(np.uint32)
    x = raw.view(np.float32)
    x = x[np.isfinite(x)]
    xs = np.concatenate([x, _rand(5000, 1, 0.05), np.float32([0, -0.0, 1e-40, -1e-40, 65504.0])])
    want = torch.from_numpy(xs).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([O.f32_to_bf16_bits(v) for v in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
    back = np.array([O.bf16_bits_to_f32(int(b)) for b in want[:2000]], dtype=np.float32)
    ref = torch.from_numpy(want[:2000].view(np.int16).copy()).view(torch.bfloat16).float().numpy()
    assert np.array_equal(back, ref)


def _bf(x):
    return torch.from_numpy(_f32(x).reshape(-1)).to(torch.bfloat16)


def test_bf16_stage_matches_fp32_stage_on_representable_inputs():
    """With bf16-representable inputs the mixed-precision oracle must agree with the fp32
    oracle except for where the update lands (master) and the final rounding."""
    n = 2048
    V = [_bf(_rand(n, 70 + s, 0.3)) for s in range(4)]
    g = _bf(_rand(n, 11))
    master = torch.from_numpy(_rand(n, 12, 0.3))
    new, m_new, g_out, norms = O.compensate_stage_bf16(V, g, master, 2, 0.3, 0.005)
    Vf = [v.float().numpy() for v in V]
    _, g_ref, norms_ref = O.compensate_stage_f32(Vf, g.float().numpy(), 2, 0.3, 0.005)
    assert np.array_equal(g_out, g_ref)
    np.testing.assert_allclose(norms, norms_ref, rtol=1e-15)
    m_ref = (master.double().numpy() - 0.005 * g_ref).astype(np.float32)
    assert np.array_equal(m_new, m_ref)
    # stored version = RNE bf16 of the new master (library conversion as the reference)
    want = torch.from_numpy(m_ref).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(new, want)


def test_bf16_hand_worked():
    # all values bf16-exact: V = (1.0, 1.5), g = 2, lambda = .5: g_1 = 2 + .5*4*.5 = 3
    # master 1.50390625 (= 1.5 + 2^-8, not bf16) ; eta = 2^-8 : m_new = 1.50390625 - 3*2^-8 = 1.4921875
    # 1.4921875 = 0x3FBF0000 exactly -> bf16 0x3FBF
    V = [_bf([1.0]), _bf([1.5])]
    new, m_new, g_out, _ = O.compensate_stage_bf16(V, _bf([2.0]), _f32([1.50390625]), -1, 0.5, 2.0 ** -8)
    assert g_out[0] == 3.0 and m_new[0] == np.float32(1.4921875) and new[0] == 0x3FBF


# ---------------------------------------------------------------------------------------
# version store across steps
# ---------------------------------------------------------------------------------------
def test_ring_keeps_last_R_versions_and_warmup_staleness():
    n, R, tau = 64, 3, 2
    ring = O.OracleRing([tau], R, -1)
    w0 = _rand(n, 80, 0.05)
    ring.push(0, w0)
    hist = [w0]
    for step in range(7):
        g = _rand(n, 100 + step)
        tau_eff = min(tau, len(hist) - 1)
        assert ring.effective_tau(0) == tau_eff
        window = hist[len(hist) - 1 - tau_eff:]
        want, _, _ = O.compensate_stage_f32(window, g, -1, 0.5, 0.01)
        got, _, _ = ring.step(0, g, 0.5, 0.01)
        assert np.array_equal(got, want)
        hist.append(want)
        assert len(ring.versions[0]) == min(R, len(hist))
        for a, b in zip(ring.versions[0], hist[-R:]):
            assert np.array_equal(a, b)


def test_ring_depth_beyond_need_changes_nothing():
    """A store of exactly tau+1 versions (the new version replaces the stale snapshot) and
    a deeper one give identical trajectories."""
    n, tau = 50, 3
    a, b = O.OracleRing([tau], tau + 1, 2), O.OracleRing([tau], tau + 4, 2)
    w0 = _rand(n, 81, 0.05)
    a.push(0, w0)
    b.push(0, w0)
    for step in range(10):
        g = _rand(n, 200 + step)
        ra, _, _ = a.step(0, g, 0.5, 0.01)
        rb, _, _ = b.step(0, g, 0.5, 0.01)
        assert np.array_equal(ra, rb)
