"""CPU oracle of Ferret's pipeline planner -- TEST INFRASTRUCTURE ONLY.

Plain Python, written from the paper's definitions; shares nothing with the C++ planner in
libferret.  Covers
  * the cost model: adaptation rate R_F^T and memory footprint M_F of a partition L and a
    pipeline configuration C (Sec. "Fine-grained Pipeline Parallelism", Eq. "ferret-svre"),
  * the moves S2 (more gradient accumulation), S3 (back-propagation omission), S4 (worker
    removal) of Sec. "Iterative Configuration Search",
  * Alg. 2 "Iterative Configuration Search" (greedy: while over budget, apply the move with the
    largest memory saved per rate lost; tried with and without activation recomputation),
  * Alg. 3 "Brute-force planning" (candidate stage-time bounds, greedy contiguous partition).

Deltas of a move are obtained by evaluating the cost model before and after the move, i.e. from
the definition, not from the closed forms in the appendix "Adaptation Rate and Memory Reduction
for S1-S4" (tests compare the two where the printed closed forms are intact: S2 and S4).

Readings where the paper is garbled or silent (mirrored by the C++ planner):
  P1  the sums over workers run over every worker with c_n^d >= 0 (the printed limits
      "n = 1 .. N-1" would drop worker 0).
  P2  Alg. 3 collects the candidate bounds t^c = sum over a run of consecutive layers of
      (t^f_j + t^b_j) (printed: t^f_j + t^f_j) and keeps those that are at least as large as the
      largest single layer (printed with the inequality reversed, which would keep only bounds no
      stage can satisfy).
  P3  for a given partition, t^f and t^b are the per-stage maxima of the notation section; Alg. 3's
      call search(t^d, t^c, L, M) passes t^c only as the bound that produced L.
  P4  S3's rate change touches every stage i <= j (their LCM denominators contain c^o_j + 1); the
      printed sum limits "i = 0 .. P-1-j" are taken as a slip for that.
  P5  the last stage (P-j-1 = 0) keeps one version whatever is done: S2 and S3 do not apply to it.
  P6  S2 applies when c^o_j = 0 and ceil((P-j-1)/c^a_j) >= 2; S3 applies when c^o_j = 0 and
      ceil((P-j-1)/c^a_j) = 1 (the paper's "Delta c^a = +infinity"); S4 applies to a live worker
      whose stages 0..P-2 all have c^o != 0.
  P7  a move that loses no rate (Delta R = 0) and saves memory has infinite merit and is taken first;
      ties go to the first move in the order worker, then S2 < S3 < S4, then stage.
  P9  Eq. "dsvre-ga" prints Delta M of S2 as one stage-unit; Delta c^a is the smallest increase that
      lowers ceil((P-j-1)/c^a) at all and the ceiling can fall by more than one (P-j-1 = 4:
      c^a 1 -> 2 takes it from 4 to 2); the definition of M_F is followed.
  P8  if no move applies and the budget is still exceeded the search fails (rate 0, infeasible).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple


@dataclass
class Layer:
    t_f: float
    t_b: float
    n_params: float
    n_acts: float


@dataclass
class Config:
    """C = {c_n^d, c_n^r, c_{n,j}^a, c_{n,j}^o}: per worker delay (-1 = removed), recomputation flag,
    per worker and stage accumulation steps and omission steps."""
    delay: List[int]
    recompute: List[int]
    accum: List[List[int]]
    omit: List[List[int]]

    def copy(self) -> "Config":
        return Config(list(self.delay), list(self.recompute), [list(r) for r in self.accum],
                      [list(r) for r in self.omit])


@dataclass
class Stages:
    """Per-stage aggregates of a partition L (notation section)."""
    w: List[float]          # |w_j|
    a: List[float]          # |a_j|
    a_inner: List[float]    # activations of all but the first layer of the stage (what T1 frees)
    t_f: float              # max over stages of the summed forward times
    t_b: float


def stages_of(layers: Sequence[Layer], L: Sequence[int]) -> Stages:
    w, a, inner, tf, tb = [], [], [], [], []
    for lo, hi in zip(L, L[1:]):
        seg = layers[lo:hi]
        w.append(sum(x.n_params for x in seg))
        a.append(sum(x.n_acts for x in seg))
        inner.append(sum(x.n_acts for x in seg[1:]))
        tf.append(sum(x.t_f for x in seg))
        tb.append(sum(x.t_b for x in seg))
    return Stages(w, a, inner, max(tf), max(tb))


def _lcm(values) -> int:
    out = 1
    for v in values:
        out = out * v // math.gcd(out, v)
    return out


def A_term(S: Stages, C: Config, n: int, i: int, j: int, c: float, v_d: float) -> float:
    """A_{i,j} of Eq. "ferret-svre" for worker n."""
    P = len(S.w)
    r = C.recompute[n]
    expo = -c * ((P + j) * S.t_f + (P - i + j) * S.t_b + r * (P - i + j) * S.t_f)
    lcm = _lcm(C.omit[n][k] + 1 for k in range(i, P))
    return math.exp(expo) * v_d / (lcm * (S.t_f + S.t_b + r * S.t_f))


def worker_rate(S: Stages, C: Config, n: int, c: float, v_d: float) -> float:
    P = len(S.w)
    total_w = sum(S.w)
    out = 0.0
    for i in range(P):
        ca = C.accum[n][i]
        out += S.w[i] / total_w * (1.0 / ca) * sum(A_term(S, C, n, i, j, c, v_d) for j in range(ca))
    return out


def worker_memory(S: Stages, C: Config, n: int) -> float:
    P = len(S.w)
    out = 0.0
    for i in range(P):
        versions = 1 + math.ceil((P - i - 1) / C.accum[n][i]) - C.omit[n][i]
        out += versions * (S.w[i] + S.a[i] - C.recompute[n] * S.a_inner[i])
    return out


def evaluate(S: Stages, C: Config, c: float, v_d: float) -> Tuple[float, float]:
    """(R_F^T, M_F)."""
    live = [n for n, d in enumerate(C.delay) if d >= 0]
    return (sum(worker_rate(S, C, n, c, v_d) for n in live), sum(worker_memory(S, C, n) for n in live))


# ---- the moves -----------------------------------------------------------------------------
def next_accum(P: int, j: int, ca: int) -> Optional[int]:
    """S2: the smallest c^a' > c^a that lowers ceil((P-j-1)/c^a) by one; None if that is impossible."""
    d = P - j - 1
    cur = math.ceil(d / ca) if d > 0 else 0
    if cur < 2:
        return None
    return math.ceil(d / (cur - 1))


def moves(P: int, C: Config):
    """All applicable moves in the tie-break order: (worker, kind, stage)."""
    for n, dly in enumerate(C.delay):
        if dly < 0:
            continue
        for j in range(P - 1):
            if C.omit[n][j] == 0 and next_accum(P, j, C.accum[n][j]) is not None:
                yield (n, "S2", j)
        for j in range(P - 1):
            if C.omit[n][j] == 0 and math.ceil((P - j - 1) / C.accum[n][j]) == 1:
                yield (n, "S3", j)
        if all(C.omit[n][j] != 0 for j in range(P - 1)):      # vacuously true for a one-stage pipeline
            yield (n, "S4", -1)


def apply_move(P: int, C: Config, move) -> Config:
    n, kind, j = move
    out = C.copy()
    if kind == "S2":
        out.accum[n][j] = next_accum(P, j, C.accum[n][j])
    elif kind == "S3":
        out.accum[n][j] = 1
        out.omit[n][j] = P - 1 - j
    else:
        out.delay[n] = -1
    return out


# ---- Alg. 2 ----------------------------------------------------------------------------------
def itersearch(S: Stages, t_d: float, c_r: int, M: float, c: float, v_d: float):
    P = len(S.w)
    N = math.ceil((S.t_f + S.t_b + c_r * S.t_f) / t_d)
    C = Config(list(range(N)), [c_r] * N, [[1] * P for _ in range(N)], [[0] * P for _ in range(N)])
    R, Mem = evaluate(S, C, c, v_d)
    trace = []
    while Mem > M:
        best, best_merit, best_state = None, -1.0, None
        for mv in moves(P, C):
            C2 = apply_move(P, C, mv)
            R2, M2 = evaluate(S, C2, c, v_d)
            dR, dM = R2 - R, M2 - Mem
            if dM >= 0:
                continue
            merit = math.inf if dR >= 0 else dM / dR
            if merit > best_merit:
                best, best_merit, best_state = mv, merit, (C2, R2, M2)
        if best is None:
            return None, 0.0, Mem, trace
        C, R, Mem = best_state
        trace.append(best)
    return C, R, Mem, trace


def search(S: Stages, t_d: float, M: float, c: float, v_d: float):
    r0 = itersearch(S, t_d, 0, M, c, v_d)
    r1 = itersearch(S, t_d, 1, M, c, v_d)
    return r1 if r1[1] > r0[1] else r0


# ---- Alg. 3 ----------------------------------------------------------------------------------
def candidate_bounds(layers: Sequence[Layer]) -> List[float]:
    n = len(layers)
    per_layer = [x.t_f + x.t_b for x in layers]
    floor_ = max(per_layer)
    out = set()
    for k in range(n):
        for i in range(n - k):
            t_c = sum(per_layer[i:i + k + 1])
            if t_c >= floor_:
                out.add(t_c)
    return sorted(out)


def partition_for(layers: Sequence[Layer], t_c: float) -> List[int]:
    L, t_sum = [0], 0.0
    for i, x in enumerate(layers):
        t_sum += x.t_f + x.t_b
        if t_sum > t_c:
            L.append(i)
            t_sum = x.t_f + x.t_b
    L.append(len(layers))
    return L


def plan(layers: Sequence[Layer], t_d: float, M: float, c: float, v_d: float):
    best = dict(L=None, C=None, R=0.0, M=None, t_c=0.0)
    for t_c in candidate_bounds(layers):
        L = partition_for(layers, t_c)
        S = stages_of(layers, L)
        C, R, Mem, _ = search(S, t_d, M, c, v_d)
        if R > best["R"]:
            best = dict(L=L, C=C, R=R, M=Mem, t_c=t_c)
    return best
