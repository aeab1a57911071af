"""Property tests (hypothesis) of the host side: layout, ring arithmetic, byte accounting, for arbitrary
small plans.  CPU only."""
import math

import pytest
from hypothesis import given, settings, strategies as st

from oracle import ferret_oracle as O
from paper_2503_12053_amd import binding as B


@pytest.fixture(scope="module", autouse=True)
def _lib():
    from paper_2503_12053_amd import build
    build.build(verbose=False)
    B.load()


stage_lists = st.lists(st.lists(st.integers(1, 5000), min_size=1, max_size=4), min_size=1, max_size=6)


def elt_of(prec):
    return 4 if prec == B.FERRET_F32 else 2


@settings(max_examples=60, deadline=None, derandomize=True)
@given(sizes=stage_lists, data=st.data())
def test_layout_and_state_invariants(sizes, data):
    P = len(sizes)
    R = data.draw(st.integers(1, 9))
    tau = [data.draw(st.integers(0, R - 1)) for _ in range(P)]
    K = data.draw(st.sampled_from([-1, 0, 1, 2, 3, 7]))
    prec = data.draw(st.sampled_from([B.FERRET_F32, B.FERRET_BF16_MASTER_F32]))
    minimal = data.draw(st.booleans())
    chunk = data.draw(st.sampled_from([0, 1024, 4096]))
    tuning = data.draw(st.sampled_from([None, dict(cache_policy=1), dict(cache_policy=2, resident_cap=3),
                                        dict(chunk_bytes=1), dict(chunk_bytes=30_000), dict(chunk_bytes=1 << 22),
                                        dict(slot_align_elems=512, slot_skew_elems=24, blocks_per_cu=2)]))
    if tuning and "chunk_bytes" in tuning:
        chunk = 0
    tensors = [(n, j) for j, ss in enumerate(sizes) for n in ss]
    plan = B.ferret_plan_buckets(tensors, P, tau, K, B.FERRET_RING_DEPTH_MINIMAL if minimal else R, prec, chunk, tuning)
    if tuning and "chunk_bytes" in tuning:
        # the byte target picks the multiple of 1024 elements nearest to target / (bytes per element in flight)
        for j in range(P):
            kp = tau[j] if K < 0 else min(K, tau[j])
            per = elt_of(prec) * (min(kp + 1, 9) if kp <= 8 else 8) + 2 * elt_of(prec) + (0 if prec == B.FERRET_F32 else 8)
            per += elt_of(prec) if kp == 0 and tau[j] > 0 else 0
            want = max(1, (tuning["chunk_bytes"] + per * 512) // (per * 1024)) * 1024
            assert plan.stage_chunk_elems(j) == min(want, 1 << 24), (j, kp, per)
    elt = 4 if prec == B.FERRET_F32 else 2
    # regions: disjoint, ordered, inside the totals
    ring, flat, i = [], [], 0
    for j, ss in enumerate(sizes):
        n_j = plan.stage_numel(j)
        assert n_j % B.FERRET_ALIGN_ELEMS == 0 and sum(ss) <= n_j < sum(ss) + B.FERRET_ALIGN_ELEMS * len(ss)
        end = 0
        for n in ss:
            off = plan.tensor_offset(i)
            assert off % B.FERRET_ALIGN_ELEMS == 0 and off >= end and off + n <= n_j
            end = off + n
            i += 1
        depth = plan.stage_ring_depth(j)
        assert depth == (tau[j] + 1 if minimal else R)
        assert plan.stage_slot_stride(j) >= n_j
        flat.append((plan.stage_flat_offset(j), plan.stage_flat_offset(j) + n_j))
        ring += [(plan.slot_offset(j, s), plan.slot_offset(j, s) + n_j) for s in range(depth)]
    for regions, total in ((flat, plan.flat_elems), (ring, plan.ring_elems)):
        regions.sort()
        assert regions[-1][1] <= total and all(a[1] <= b[0] for a, b in zip(regions, regions[1:]))
    assert all(lo % 4 == 0 for lo, _ in flat + ring)                   # 16-byte aligned starts
    assert plan.ring_bytes == plan.ring_elems * elt
    assert plan.n_chunks == sum(-(-plan.stage_numel(j) // plan.stage_chunk_elems(j)) for j in range(P))
    assert all(plan.stage_chunk_elems(j) % 1024 == 0 and plan.stage_chunk_elems(j) >= 1024 for j in range(P))
    assert plan.chunk_elems == max(plan.stage_chunk_elems(j) for j in range(P))
    if chunk:
        assert all(plan.stage_chunk_elems(j) == chunk for j in range(P))
    # ring arithmetic for an arbitrary valid state
    heads = [data.draw(st.integers(0, plan.stage_ring_depth(j) - 1)) for j in range(P)]
    valid = [data.draw(st.integers(1, plan.stage_ring_depth(j))) for j in range(P)]
    plan.set_state(heads, valid)
    want_bytes = 0
    for j in range(P):
        depth = plan.stage_ring_depth(j)
        t = min(tau[j], valid[j] - 1)
        assert plan.stage_effective_staleness(j) == t
        bounds = O.segment_boundaries(t, K)
        slots = plan.stage_read_slots(j)
        assert slots == [(heads[j] - (t - s)) % depth for s in bounds]
        assert slots[-1] == heads[j]                                    # the newest version is always read
        w = plan.stage_write_slot(j)
        assert w == (heads[j] + 1) % depth
        assert w not in slots[1:]                                       # only the oldest slot may be overwritten
        kp = O.effective_iters(K, t)
        want_bytes += sum(sizes[j]) * (elt * (kp + 3) + (8 if prec == B.FERRET_BF16_MASTER_F32 else 0))
    assert plan.step_bytes == want_bytes


@settings(max_examples=200, deadline=None, derandomize=True)
@given(tau=st.integers(0, 60), K=st.integers(-1, 70))
def test_segments_partition_the_version_steps(tau, K):
    s = O.segment_boundaries(tau, K)
    kp = O.effective_iters(K, tau)
    assert kp == (tau if K < 0 else min(K, tau))
    if kp == 0:
        assert s == [tau]
        return
    assert s[0] == 0 and s[-1] == tau and len(s) == kp + 1
    lengths = [b - a for a, b in zip(s, s[1:])]
    assert min(lengths) >= 1 and max(lengths) - min(lengths) <= 1      # segments as even as integers allow
    assert sum(lengths) == tau
