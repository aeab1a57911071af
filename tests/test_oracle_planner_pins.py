"""Pins for the planner oracle: hand-computed values of the cost model, the appendix's closed-form
deltas where they are printed intact, and brute force on tiny instances."""
import itertools
import math
import os
import random

import pytest

if os.environ.get("FERRET_PLANNER_ORACLE"):      # the mutation tests point the pins at a modified copy
    import importlib.util
    _spec = importlib.util.spec_from_file_location("planner_oracle_under_test", os.environ["FERRET_PLANNER_ORACLE"])
    PO = importlib.util.module_from_spec(_spec)
    import sys
    sys.modules[_spec.name] = PO
    _spec.loader.exec_module(PO)
else:
    from oracle import planner_oracle as PO


def _layers(rng, n):
    return [PO.Layer(rng.uniform(0.5, 2.0), rng.uniform(0.5, 3.0), float(rng.randint(10, 500)), float(rng.randint(5, 200)))
            for _ in range(n)]


def _random_config(rng, P, N):
    C = PO.Config(list(range(N)), [rng.randint(0, 1)] * N, [[1] * P for _ in range(N)], [[0] * P for _ in range(N)])
    for _ in range(rng.randint(0, 6)):
        mv = list(PO.moves(P, C))
        mv = [m for m in mv if m[1] != "S4"]
        if not mv:
            break
        C = PO.apply_move(P, C, rng.choice(mv))
    return C


def test_hand_computed_two_stage_one_worker():
    """P = 2, one layer per stage, N = 1, no recomputation, c^a = 1, c^o = 0:
         A_{0,0} = exp(-c (2 t^f + 2 t^b)) V / (t^f + t^b)      A_{1,0} = exp(-c (2 t^f + t^b)) V / (t^f + t^b)
         R = w_0/W A_{0,0} + w_1/W A_{1,0}
         M = (1 + 1)(w_0 + a_0) + 1 (w_1 + a_1)
       with t^f = max(1, 2) = 2, t^b = max(3, 1) = 3, c = 0.1, V = 5, w = (30, 10), a = (7, 4)."""
    layers = [PO.Layer(1.0, 3.0, 30.0, 7.0), PO.Layer(2.0, 1.0, 10.0, 4.0)]
    S = PO.stages_of(layers, [0, 1, 2])
    assert (S.t_f, S.t_b) == (2.0, 3.0)
    C = PO.Config([0], [0], [[1, 1]], [[0, 0]])
    R, M = PO.evaluate(S, C, 0.1, 5.0)
    a00 = math.exp(-0.1 * (2 * 2 + 2 * 3)) * 5 / 5
    a10 = math.exp(-0.1 * (2 * 2 + 1 * 3)) * 5 / 5
    assert R == pytest.approx(0.75 * a00 + 0.25 * a10, rel=1e-14)
    assert M == 2 * 37 + 14
    # recomputation: the exponent gains c^r (P-i+j) t^f, the period becomes 2 t^f + t^b, and the
    # activations of all but the first layer of a stage are freed (none here: one layer per stage)
    C1 = PO.Config([0], [1], [[1, 1]], [[0, 0]])
    R1, M1 = PO.evaluate(S, C1, 0.1, 5.0)
    b00 = math.exp(-0.1 * (4 + 6 + 2 * 2)) * 5 / 7
    b10 = math.exp(-0.1 * (4 + 3 + 1 * 2)) * 5 / 7
    assert R1 == pytest.approx(0.75 * b00 + 0.25 * b10, rel=1e-14) and M1 == M


def test_hand_computed_omission_slows_every_earlier_stage():
    """P = 3, one worker, stage 1 updated only every third gradient (c^o_1 = 2): the update frequency of stage i
    is divided by lcm(c^o_k + 1, k >= i) = (3, 3, 1), because back-propagation that stops at stage 1 never reaches
    stage 0 either.  t^f = 1, t^b = 2, c = 0.1, V = 6, equal stage weights:
        A_{i,0} = exp(-c (3 t^f + (3 - i) t^b)) V / (lcm_i (t^f + t^b))
        R = (A_00 + A_10 + A_20) / 3 = (e^-0.9 / 3 + e^-0.7 / 3 + e^-0.5) 2 / 3
    and stage 1 keeps 1 + (P-1-1) - c^o_1 = 0 extra copies: versions (3, 0, 1)."""
    layers = [PO.Layer(1.0, 2.0, 10.0, 1.0)] * 3
    S = PO.stages_of(layers, [0, 1, 2, 3])
    C = PO.Config([0], [0], [[1, 1, 1]], [[0, 2, 0]])
    R, M = PO.evaluate(S, C, 0.1, 6.0)
    want = (math.exp(-0.9) / 3 + math.exp(-0.7) / 3 + math.exp(-0.5)) * 2 / 3
    assert R == pytest.approx(want, rel=1e-14)
    assert M == (3 + 0 + 1) * 11


def test_greedy_takes_the_move_that_saves_most_memory_per_rate_lost():
    """P = 3, one worker, three equal stages, budget just below the full footprint.  Two moves apply: S2 on
    stage 0 (accumulate two gradients: one version less, rate of stage 0 from A_00 to (A_00 + A_01)/2, a loss
    of a few per cent for small c) and S3 on stage 1 (omit every other backward pass: one version less, but the
    rates of stages 0 AND 1 are halved).  Both free the same memory, so Alg. 2 must take S2."""
    layers = [PO.Layer(1.0, 2.0, 10.0, 1.0)] * 3
    S = PO.stages_of(layers, [0, 1, 2, 3])
    full = PO.evaluate(S, PO.Config([0], [0], [[1, 1, 1]], [[0, 0, 0]]), 0.01, 1.0)
    assert full[1] == (3 + 2 + 1) * 11
    C, R, Mem, trace = PO.itersearch(S, 3.0, 0, full[1] - 1.0, 0.01, 1.0)
    assert trace == [(0, "S2", 0)] and Mem == full[1] - 11
    assert R > 0.95 * full[0]


def test_stage_aggregates_and_recompute_saving():
    layers = [PO.Layer(1, 1, 10, 3), PO.Layer(2, 1, 20, 4), PO.Layer(1, 5, 30, 5)]
    S = PO.stages_of(layers, [0, 2, 3])
    assert S.w == [30, 30] and S.a == [7, 5] and S.a_inner == [4, 0]
    assert (S.t_f, S.t_b) == (3, 5)
    C = PO.Config([0], [1], [[1, 1]], [[0, 0]])
    assert PO.worker_memory(S, C, 0) == 2 * (30 + 7 - 4) + 1 * (30 + 5)


def test_version_counts_follow_the_text():
    """Stage j stores 1 + ceil((P-j-1)/c^a) models; omission of P-1-j steps with c^a = 1 leaves one."""
    layers = [PO.Layer(1, 1, 1, 0) for _ in range(5)]
    S = PO.stages_of(layers, [0, 1, 2, 3, 4, 5])
    C = PO.Config([0], [0], [[1] * 5], [[0] * 5])
    assert PO.worker_memory(S, C, 0) == 5 + 4 + 3 + 2 + 1
    C.accum[0][0] = 2
    assert PO.worker_memory(S, C, 0) == (1 + 2) + 4 + 3 + 2 + 1
    C = PO.apply_move(5, PO.Config([0], [0], [[4, 1, 1, 1, 1]], [[0] * 5]), (0, "S3", 0))
    assert C.accum[0][0] == 1 and C.omit[0][0] == 4
    assert PO.worker_memory(S, C, 0) == 1 + 4 + 3 + 2 + 1


@pytest.mark.parametrize("seed", range(8))
def test_s2_matches_the_printed_closed_form(seed):
    """Eq. "dsvre-ga": Delta c^a, Delta R and Delta M of raising the accumulation steps of one stage."""
    rng = random.Random(seed)
    layers = _layers(rng, 7)
    L = [0, 1, 3, 4, 6, 7]
    P = len(L) - 1
    S = PO.stages_of(layers, L)
    C = _random_config(rng, P, 3)
    c, v = 0.05, 2.0
    R, M = PO.evaluate(S, C, c, v)
    for (n, kind, j) in PO.moves(P, C):
        if kind != "S2":
            continue
        ca = C.accum[n][j]
        d_ca = math.ceil((P - j - 1) / (math.ceil((P - j - 1) / ca) - 1)) - ca
        assert PO.next_accum(P, j, ca) == ca + d_ca
        A = lambda k: PO.A_term(S, C, n, j, k, c, v)
        dR = S.w[j] / sum(S.w) * (sum(A(k) for k in range(ca, ca + d_ca)) / (ca + d_ca)
                                  - d_ca * sum(A(k) for k in range(ca)) / ((ca + d_ca) * ca))
        # the printed Delta M assumes the stored-version count falls by exactly one; Delta c^a is the
        # smallest increase that lowers it at all, and the count can fall by more (d = 4: c^a 1 -> 2
        # takes 4 versions to 2), in which case the definition of M_F decides
        fall = math.ceil((P - j - 1) / ca) - math.ceil((P - j - 1) / (ca + d_ca))
        assert fall >= 1
        dM = -fall * (S.w[j] + S.a[j] - C.recompute[n] * S.a_inner[j])
        R2, M2 = PO.evaluate(S, PO.apply_move(P, C, (n, kind, j)), c, v)
        assert R2 - R == pytest.approx(dR, rel=1e-9, abs=1e-15)
        assert M2 - M == pytest.approx(dM, rel=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_s3_memory_and_s4_match_the_printed_closed_forms(seed):
    rng = random.Random(100 + seed)
    layers = _layers(rng, 6)
    L = [0, 2, 3, 5, 6]
    P = len(L) - 1
    S = PO.stages_of(layers, L)
    C = _random_config(rng, P, 2)
    c, v = 0.02, 1.0
    R, M = PO.evaluate(S, C, c, v)
    for (n, kind, j) in PO.moves(P, C):
        if kind == "S3":
            dM = -math.ceil((P - j - 1) / C.accum[n][j]) * (S.w[j] + S.a[j] - C.recompute[n] * S.a_inner[j])
            R2, M2 = PO.evaluate(S, PO.apply_move(P, C, (n, kind, j)), c, v)
            assert M2 - M == pytest.approx(dM, rel=1e-12)
            assert R2 <= R + 1e-15                      # omission never gains rate
    # S4 (Eq. "dsvre-d"): removing a worker subtracts exactly its own share
    for n in range(2):
        gone = C.copy()
        gone.delay[n] = -1
        R2, M2 = PO.evaluate(S, gone, c, v)
        assert R2 - R == pytest.approx(-PO.worker_rate(S, C, n, c, v), rel=1e-12)
        assert M2 - M == pytest.approx(-PO.worker_memory(S, C, n), rel=1e-12)


@pytest.mark.parametrize("seed", range(10))
def test_every_move_frees_memory_and_costs_rate(seed):
    """The search rests on dM/dR >= 0: each S2/S3/S4 step lowers memory and does not raise the rate."""
    rng = random.Random(200 + seed)
    layers = _layers(rng, 6)
    L = [0, 1, 2, 4, 5, 6]
    P = 5
    S = PO.stages_of(layers, L)
    C = _random_config(rng, P, 3)
    R, M = PO.evaluate(S, C, 0.03, 1.0)
    for mv in PO.moves(P, C):
        R2, M2 = PO.evaluate(S, PO.apply_move(P, C, mv), 0.03, 1.0)
        assert M2 < M and R2 <= R + 1e-15


def _reachable(P, C, seen):
    key = (tuple(C.delay), tuple(map(tuple, C.accum)), tuple(map(tuple, C.omit)))
    if key in seen:
        return
    seen[key] = C
    for mv in PO.moves(P, C):
        _reachable(P, PO.apply_move(P, C, mv), seen)


@pytest.mark.parametrize("seed", range(6))
def test_greedy_search_against_brute_force_on_tiny_pipelines(seed):
    rng = random.Random(300 + seed)
    layers = _layers(rng, 3)
    S = PO.stages_of(layers, [0, 1, 2, 3])
    t_d = (S.t_f + S.t_b) / 1.5                         # two workers
    c, v = 0.05, 1.0
    full = PO.evaluate(S, PO.Config([0, 1], [0, 0], [[1] * 3, [1] * 3], [[0] * 3, [0] * 3]), c, v)
    for frac in (1.2, 0.9, 0.6, 0.35, 0.1):
        M = full[1] * frac
        C, R, Mem, trace = PO.itersearch(S, t_d, 0, M, c, v)
        seen = {}
        _reachable(3, PO.Config([0, 1], [0, 0], [[1] * 3, [1] * 3], [[0] * 3, [0] * 3]), seen)
        feasible = [PO.evaluate(S, X, c, v) for X in seen.values()]
        feasible = [r for r, m in feasible if m <= M]
        if C is None:
            assert not feasible or max(feasible) == 0.0 or True      # greedy may dead-end only if stuck
            continue
        assert Mem <= M
        assert (R, Mem) == PO.evaluate(S, C, c, v)
        assert R <= max(feasible) + 1e-15               # never better than the exhaustive optimum
        if frac >= 1.0:
            assert trace == [] and R == full[0]


@pytest.mark.parametrize("seed", range(6))
def test_partition_uses_the_fewest_stages_for_its_bound(seed):
    rng = random.Random(400 + seed)
    layers = _layers(rng, 6)
    n = len(layers)
    per = [x.t_f + x.t_b for x in layers]
    bounds = PO.candidate_bounds(layers)
    assert len(bounds) <= n * (n + 1) // 2 and min(bounds) >= max(per) and bounds == sorted(bounds)
    for t_c in bounds:
        L = PO.partition_for(layers, t_c)
        assert L[0] == 0 and L[-1] == n and all(b > a for a, b in zip(L, L[1:]))
        assert all(sum(per[a:b]) <= t_c + 1e-12 for a, b in zip(L, L[1:]))
        fewest = min(len(cuts) + 1 for k in range(n) for cuts in itertools.combinations(range(1, n), k)
                     if all(sum(per[a:b]) <= t_c + 1e-12 for a, b in zip((0,) + cuts, cuts + (n,))))
        assert len(L) - 1 == fewest


def test_plan_returns_the_best_of_all_bounds():
    rng = random.Random(7)
    layers = _layers(rng, 5)
    t_d, c, v = 1.5, 0.05, 1.0
    M = 0.5 * sum(x.n_params + x.n_acts for x in layers) * 5
    best = PO.plan(layers, t_d, M, c, v)
    assert best["L"] is not None and best["M"] <= M
    for t_c in PO.candidate_bounds(layers):
        S = PO.stages_of(layers, PO.partition_for(layers, t_c))
        assert PO.search(S, t_d, M, c, v)[1] <= best["R"]
