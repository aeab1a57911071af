"""GPU parity: the HIP path (called through the C ABI) against the CPU oracle, element by
element, on identical seeded inputs.  Tolerances are defined in tests/parity_util.py.

Run on an MI355X with:  python -u -m pytest tests -m gpu -x -v --timeout 300 --timeout-method thread
"""
import os

import numpy as np
import pytest
import torch

from oracle import ferret_oracle as O
from paper_2503_12053_amd import binding as B
from paper_2503_12053_amd import workloads as W

import parity_util as PU

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m 'not gpu' elsewhere)")
    B.load()          # raises if libferret.so is not built: there is no fallback
    print("device:", torch.cuda.get_device_name(0), flush=True)


def _run(w, amplified=False, label="", **kw):
    print(f"[case] {label or w.name} amplified={amplified} {kw}", flush=True)
    plan, st, host = PU.load_workload(w, amplified=amplified, **kw)
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    stats = PU.check_step_against_oracle(w, plan, st, host, K=kw.get("n_iters"), n_threads=4, label=label)
    return plan, st, host, stats


# ---- the benchmark configurations -------------------------------------------------------------
@pytest.mark.parametrize("idx", [1, 2, 3])
@pytest.mark.parametrize("amplified", [False, True])
def test_benchmark_configs_small(idx, amplified):
    _run(W.make_workload(idx), amplified)


@pytest.mark.parametrize("amplified", [False, True])
def test_benchmark_config_4_full_size(amplified):
    """ViT-B-sized: the launch configuration the benchmark times (default chunking and grid)."""
    _run(W.make_workload(4), amplified)


@pytest.mark.timeout(900)
def test_benchmark_config_5_full_size():
    """350 M parameters, bf16 + fp32 master, heavy-tailed gradients; whole arrays are compared."""
    w = W.make_workload(5)
    plan, st, host, stats = _run(w, False)
    # the heavy tail makes the compensation visible in the master (|g| ~ 1 entries)
    assert plan.step_bytes == sum((14 + 2 * min(4, t)) * n for t, n in zip(w.staleness, w.stage_numel()))


def test_benchmark_config_5_shape_amplified_two_stages():
    """Same dtype path with the compensation term at a few per cent, on a 2-stage cut of the shape."""
    w = W.custom_workload("mixed_amplified", [[21_875_000 // 8], [21_875_000 // 8]], [15, 3], 16, 4, lam=0.3,
                          lr=0.005, precision="bf16", seed=41, heavy_tail=(0.01, 3.0))
    _run(w, True)


# ---- ragged shapes, many chunks, tiny stages ---------------------------------------------------
RAGGED = [
    ("one_element", [[1]], [1], 2, -1),
    ("odd_tensors", [[1, 3, 1001, 64, 4097], [7], [5000, 13]], [2, 1, 0], 3, -1),
    ("tail_of_8", [[1024 * 3 + 8]], [1], 2, 1),
    ("multi_chunk_ragged", [[10_000, 33, 70_001], [2048], [123_457]], [3, 2, 1], 4, 2),
]


@pytest.mark.parametrize("name,sizes,tau,R,K", RAGGED)
@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("chunk_units", [0, 3, 8])
def test_ragged_shapes(name, sizes, tau, R, K, precision, chunk_units):
    unit = 1024 if precision == "f32" else 2048
    w = W.custom_workload(name, sizes, tau, R, K, precision=precision, seed=7)
    _run(w, True, chunk_elems=chunk_units * unit)


# ---- iteration counts: none, single step, segments, one per version step, streamed ---------------
@pytest.mark.parametrize("K", [0, 1, 2, 3, 4, 5, 6, -1])
@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_iteration_counts(K, precision):
    w = W.custom_workload("iters", [[40_000, 24], [9_000], [31_000]], [7, 4, 0], 8, K, precision=precision, seed=11)
    plan, st, host, _ = _run(w, True, n_iters=K)
    for j, tau in enumerate(w.staleness):
        assert plan.stage_effective_iters(j) == O.effective_iters(K, tau)


def test_deep_staleness_streamed_path():
    w = W.custom_workload("deep", [[70_000], [50_000]], [15, 11], 16, -1, seed=12, lam=0.3)
    _run(w, True)


# ---- ring positions and the in-place case --------------------------------------------------------
@pytest.mark.parametrize("head_shift", [0, 1, 2, 3])
def test_every_head_position(head_shift):
    w = W.custom_workload("heads", [[30_000], [30_000], [30_000], [30_000]], [3, 2, 1, 0], 4, 2, seed=13)
    _run(w, True, heads=[head_shift, head_shift + 1, head_shift + 2, head_shift + 3])


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_minimal_ring_new_version_replaces_stale_snapshot(precision):
    """Ring depth tau_j + 1: the slot written is the slot of V[0], read in the same pass."""
    w = W.custom_workload("inplace", [[50_000, 17], [20_000], [4_000]], [2, 1, 0], 3, -1, precision=precision, seed=14)
    plan, st, host = PU.load_workload(w, amplified=True, ring_depth=B.FERRET_RING_DEPTH_MINIMAL)
    for j in range(3):
        assert plan.stage_write_slot(j) == plan.stage_read_slots(j)[0]
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    PU.check_step_against_oracle(w, plan, st, host)


@pytest.mark.parametrize("precision,depth", [("f32", 4), ("f32", 0), ("bf16", 4), ("bf16", 0)])
def test_many_steps_with_warmup_and_wraparound(precision, depth):
    """From a single pushed version through 2R+3 steps: warm-up staleness, eviction, wrap-around;
    every step's new version is compared with the oracle's version store."""
    tau = [3, 1, 0]
    w = W.custom_workload("steps", [[20_000, 9], [6_000], [3_001]], tau, depth or 4, 2, precision=precision, seed=15)
    plan = B.plan_for_workload(w, ring_depth=depth)
    st = B.DeviceState(plan, PU.tensors_of(w))
    ring = O.OracleRing(tau, 4 if depth else 99, 2, precision)   # oracle never needs more than tau+1
    for j in range(3):
        d = W.generate_stage(w, j, True, n_versions=1)
        init = d.master if precision == "bf16" else d.versions[0]          # fp32 initial weights
        src = torch.zeros(plan.flat_elems, dtype=torch.float32, device="cuda")
        st.set_flat(src, j, init)
        B.ferret_push_version(plan, st.ring, st.master, j, src)
        torch.cuda.synchronize()
        want0 = init.to(torch.bfloat16) if precision == "bf16" else init
        assert torch.equal(st.get_version(j, 0), want0)
        ring.push(j, want0, init if precision == "bf16" else None)
    assert plan.get_state() == ([0, 0, 0], [1, 1, 1])
    for step in range(11):
        for j in range(3):
            g = W.draw_grads(w, j, w.stage_numel()[j], amplified=True, step=step)
            g = g.to(torch.bfloat16) if precision == "bf16" else g
            st.set_flat(st.grads, j, g)
            assert plan.stage_effective_staleness(j) == ring.effective_tau(j)
        slots = [plan.stage_write_slot(j) for j in range(3)]
        st.step(w.lam, w.lr)
        torch.cuda.synchronize()
        norms = st.norms.cpu().numpy()
        for j in range(3):
            g = st.get_flat(st.grads, j)
            new, g_ref, n_ref = ring.step(j, g, np.float32(w.lam), np.float32(w.lr))
            tag = f"step {step} stage {j}"
            PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), g_ref, tag + " g")
            if precision == "f32":
                got = st.get_version(j, slots[j]).numpy()
                PU.assert_close_f32(got, new, tag + " version")
                ring.versions[j][-1] = got.copy()          # keep both sides on identical inputs
            else:
                got = PU.bits_of(st.get_version(j, slots[j]))
                got_m = st.get_flat(st.master, j).numpy()
                PU.assert_close_f32(got_m, ring.master[j], tag + " master")
                slack = PU.master_slack(ring.master[j], w.lr, np.maximum(np.abs(g_ref), np.abs(g.float().numpy())),
                                        plan.stage_effective_iters(j))
                PU.assert_master_within_slack(got_m, ring.master[j], slack, tag + " master")
                PU.assert_bf16_within_one_ulp(got, new, tag + " version", abs_slack=slack)
                PU.assert_bf16_is_rounded_master(got, got_m, tag + " version vs own master")
                ring.versions[j][-1] = got.copy()
                ring.master[j] = got_m.copy()
            np.testing.assert_allclose(norms[j], n_ref, rtol=PU.RTOL, atol=1e-30)
        st.commit()
    heads, valid = plan.get_state()
    assert valid == [plan.stage_ring_depth(j) for j in range(3)]


# ---- properties that hold at any size ---------------------------------------------------------
def test_zero_lambda_and_zero_drift_leave_gradient_bit_exact():
    w = W.make_workload(2)
    plan, st, host = PU.load_workload(w, amplified=True)
    st.step(0.0, w.lr)
    torch.cuda.synchronize()
    for j in range(w.n_stages):
        assert torch.equal(st.get_flat(st.grad_out, j), host[j].grads)
    # zero drift: every slot holds the same weights
    for j in range(w.n_stages):
        for s in range(w.ring_depth):
            st.set_version(j, s, host[j].versions[-1])
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    norms = st.norms.cpu().numpy()
    for j in range(w.n_stages):
        assert torch.equal(st.get_flat(st.grad_out, j), host[j].grads)
        want = host[j].versions[-1].double() - float(np.float32(w.lr)) * host[j].grads.double()
        PU.assert_close_f32(st.get_version(j, plan.stage_write_slot(j)).numpy(), want.numpy(), "sgd")
        assert norms[j][2] == 0.0 and norms[j][0] == norms[j][1]


def test_outputs_do_not_depend_on_optional_outputs_or_grid():
    w = W.custom_workload("grid", [[300_000, 40], [77_777]], [3, 1], 4, 2, seed=16)
    results = []
    for tuning, norms, gout in [(None, True, True), (dict(blocks_per_cu=-1), True, True),
                                (dict(blocks_per_cu=1), False, False), (dict(blocks_per_cu=3), True, False),
                                (dict(slot_align_elems=4096, slot_skew_elems=520), False, True),
                                (dict(resident_cap=3), True, True), (dict(resident_cap=-1, blocks_per_cu=2), True, True),
                                (dict(cache_policy=1), True, True), (dict(cache_policy=2), True, False),
                                (dict(cache_policy=2, resident_cap=2), False, True),
                                (dict(xcd_group=1, cache_policy=2), True, True), (dict(xcd_group=3, cache_policy=2), True, True),
                                (dict(xcd_group=16), True, False), (dict(xcd_group=64, resident_cap=3), True, True)]:
        plan, st, host = PU.load_workload(w, amplified=True, tuning=tuning)
        st.step(w.lam, w.lr, norms=norms, grad_out=gout)
        torch.cuda.synchronize()
        results.append(([st.get_version(j, plan.stage_write_slot(j)) for j in range(2)],
                        st.norms.cpu().clone() if norms else None))
    for new, nrm in results[1:]:
        for a, b in zip(new, results[0][0]):
            assert torch.equal(a, b)
        if nrm is not None:
            assert torch.equal(nrm, results[0][1])      # per-chunk partials summed in chunk order


def test_chunk_sizes_change_nothing_but_the_grouping_of_the_norm_sums():
    """Per-stage chunk sizes (the default rule, a byte target, one explicit size) give bit-identical versions and
    compensated gradients; the norms are the same sums grouped differently."""
    w = W.custom_workload("chunking", [[200_000, 24], [90_001], [50_000], [30_000]], [7, 3, 1, 0], 8, -1, seed=26)
    results = []
    for kw in [dict(tuning=dict(chunk_bytes=48 * 1024)), dict(), dict(chunk_elems=1024),
               dict(tuning=dict(chunk_bytes=16 * 1024)), dict(tuning=dict(chunk_bytes=300_000))]:
        plan, st, host = PU.load_workload(w, amplified=True, **kw)
        st.step(w.lam, w.lr)
        torch.cuda.synchronize()
        results.append((st.ring.clone(), st.grad_out.clone(), st.norms.cpu().numpy().astype(np.float64),
                        [plan.stage_chunk_elems(j) for j in range(4)]))
    assert results[0][3] == [1024, 2048, 3072, 4096] and results[3][3] == [1024] * 4     # 40, 24, 16, 12 bytes in flight
    assert results[1][3] == [2048] * 4                                                  # the default for a small plan
    assert results[4][3] == [7168, 12288, 18432, 24576]
    for ring, g, norms, _ in results[1:]:
        assert torch.equal(ring, results[0][0]) and torch.equal(g, results[0][1])
        np.testing.assert_allclose(norms, results[0][2], rtol=1e-6)


def test_step_is_repeatable_and_does_not_touch_inputs():
    w = W.custom_workload("repeat", [[100_000]], [2], 4, -1, seed=17)
    plan, st, host = PU.load_workload(w, amplified=True)
    ring_before = st.ring.clone()
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    first = st.ring.clone()
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    assert torch.equal(first, st.ring)
    slot = plan.stage_write_slot(0)
    for s in range(4):
        if s != slot:
            assert torch.equal(st.get_version(0, s), ring_before[plan.slot_offset(0, s):][:100_000].cpu())
    assert torch.equal(st.get_flat(st.grads, 0), host[0].grads)


def test_runs_on_a_side_stream():
    w = W.custom_workload("stream", [[200_000], [50_000]], [1, 0], 2, 1, seed=18)
    plan, st, host = PU.load_workload(w, amplified=True)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    st.step(w.lam, w.lr, stream=s)
    s.synchronize()
    PU.check_step_against_oracle(w, plan, st, host)


def test_nan_and_inf_propagate_like_the_oracle():
    w = W.custom_workload("nonfinite", [[4096]], [2], 3, -1, seed=19)
    plan, st, host = PU.load_workload(w, amplified=True)
    g = host[0].grads.clone()
    g[5], g[6], g[7] = float("nan"), float("inf"), float("-inf")
    host[0].grads = g
    st.set_flat(st.grads, 0, g)
    st.step(w.lam, w.lr, norms=False)
    torch.cuda.synchronize()
    ref = PU.oracle_stage(w, host[0], 2, -1)
    got_g = st.get_flat(st.grad_out, 0).numpy()
    assert np.isnan(got_g[5]) and np.isnan(ref["g"][5])
    PU.assert_close_f32(got_g, ref["g"], "g with non-finite entries")
    PU.assert_close_f32(st.get_version(0, plan.stage_write_slot(0)).numpy(), ref["new"], "version with non-finite entries")


# ---- push_version --------------------------------------------------------------------------------
@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_push_version_copies_rounds_and_advances(precision):
    w = W.custom_workload("push", [[5000, 3], [2049]], [1, 0], 3, 1, precision=precision, seed=20)
    plan = B.plan_for_workload(w)
    st = B.DeviceState(plan, PU.tensors_of(w))
    src = torch.randn(plan.flat_elems, device="cuda") * 0.05
    # values exactly between two bf16 neighbours, to see ties-to-even on the device
    src[:4] = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7 + 2.0 ** -8, -(1.0 + 2.0 ** -8), 65280.0 + 128.0])
    B.ferret_push_version(plan, st.ring, st.master, -1, src)
    torch.cuda.synchronize()
    assert plan.get_state() == ([0, 0], [1, 1])
    for j in range(2):
        n, fo = plan.stage_numel(j), plan.stage_flat_offset(j)
        got = st.ring[plan.slot_offset(j, 0):][:n].cpu()
        want = src[fo:fo + n].cpu()
        if precision == "bf16":
            want_bits = np.array([O.f32_to_bf16_bits(x) for x in want[:64].numpy()], dtype=np.uint16)
            assert np.array_equal(PU.bits_of(got[:64]), want_bits)
            assert torch.equal(got, want.to(torch.bfloat16))
            assert torch.equal(st.master[fo:fo + n].cpu(), want)
        else:
            assert torch.equal(got, want)
    # second push of one stage goes to slot 1 and leaves the other stage alone
    B.ferret_push_version(plan, st.ring, None, 1, src * 2)
    torch.cuda.synchronize()
    assert plan.get_state() == ([0, 1], [1, 2])
    n, fo = plan.stage_numel(1), plan.stage_flat_offset(1)
    assert torch.equal(st.ring[plan.slot_offset(1, 1):][:n].float().cpu(),
                       (src[fo:fo + n] * 2).to(st.storage).float().cpu())


def test_copy_bytes():
    a = torch.randn(3_000_001 * 4, device="cuda")
    b = torch.zeros_like(a)
    B.ferret_copy_bytes(b, a, a.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


# ---- HIP graph capture -----------------------------------------------------------------------------
def test_graph_of_one_ring_rotation_replays_like_eager_steps():
    """The library launches on the caller's stream and allocates nothing, so a full rotation of the ring
    (ring_depth steps; afterwards every head is back at its starting slot) can be captured once and
    replayed.  Every replay is checked against eager execution of the same steps, with eager work and
    synchronisations between the replays."""
    w = W.custom_workload("graph", [[60_000, 8], [20_000]], [2, 1], 3, -1, seed=61)
    plan_g, st_g, _ = PU.load_workload(w, amplified=True)
    plan_e, st_e, _ = PU.load_workload(w, amplified=True)
    R = w.ring_depth

    def rotation(st):
        for _ in range(R):
            st.step(w.lam, w.lr)
            st.commit()

    heads0 = plan_g.get_state()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            rotation(st_g)
    torch.cuda.current_stream().wait_stream(side)
    assert plan_g.get_state() == heads0                     # host state is back at the start
    for replay in range(4):
        g = W.draw_grads(w, 0, w.stage_numel()[0], amplified=True, step=100 + replay)
        for st in (st_g, st_e):                             # new gradients, eager work between replays
            st.set_flat(st.grads, 0, g)
        torch.cuda.synchronize()
        graph.replay()
        rotation(st_e)
        torch.cuda.synchronize()
        assert torch.equal(st_g.ring, st_e.ring), f"replay {replay}"
        assert torch.equal(st_g.norms, st_e.norms) and torch.equal(st_g.grad_out, st_e.grad_out)


# ---- limits of the interface -----------------------------------------------------------------------
@pytest.mark.parametrize("n_stages", [17, 40, B.FERRET_MAX_STAGES])
def test_many_stages_up_to_the_maximum(n_stages):
    """More than 16 stages takes the second half of the scalar stage lookup; 64 is the documented maximum."""
    rng = np.random.default_rng(n_stages)
    sizes = [[int(rng.integers(1, 6000))] + ([int(rng.integers(1, 300))] if j % 3 == 0 else []) for j in range(n_stages)]
    tau = [int(rng.integers(0, 8)) for _ in range(n_stages)]
    w = W.custom_workload(f"stages{n_stages}", sizes, tau, 8, 3, seed=70 + n_stages)
    _run(w, True)
    w16 = W.custom_workload(f"stages{n_stages}_bf16", sizes, tau, 8, -1, precision="bf16", seed=71 + n_stages)
    _run(w16, True)


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_deep_ring_and_long_iteration_chains(precision):
    """tau = 32 with one iteration per version step: the streamed path's batches of four plus a remainder;
    tau = 9 and 8 sit on both sides of the unrolled limit."""
    w = W.custom_workload("deep_ring", [[9_000], [5_000], [5_000], [3_000]], [32, 9, 8, 30], 33, -1, precision=precision,
                          seed=72, lam=0.05)
    w.drift_std = 0.01
    _run(w, False)
    w2 = W.custom_workload("deep_ring_k7", [[9_000], [5_000]], [32, 20], 33, 7, precision=precision, seed=73, lam=0.3)
    _run(w2, True, n_iters=7)


@pytest.mark.parametrize("chunk", [65_536, 1 << 20])
def test_large_chunks_loop_inside_a_workgroup(chunk):
    w = W.custom_workload("big_chunks", [[1_500_000, 77], [300_001]], [3, 1], 4, 2, seed=74)
    _run(w, True, chunk_elems=chunk)
    w16 = W.custom_workload("big_chunks_bf16", [[1_500_000, 77], [300_001]], [3, 1], 4, 2, precision="bf16", seed=75)
    _run(w16, True, chunk_elems=chunk)


# ---- checkpoint / resume -----------------------------------------------------------------------------
@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_resume_from_saved_ring_state(precision):
    """Everything a stage's update path needs to resume is the ring contents, the master and the two
    integers per stage from ferret_plan_get_state; a fresh plan given those continues bit for bit."""
    w = W.custom_workload("resume", [[25_000, 16], [7_777]], [2, 1], 3, -1, precision=precision, seed=81)
    plan_a, st_a, _ = PU.load_workload(w, amplified=True)

    def advance(st, first_step, n):
        for k in range(first_step, first_step + n):
            for j in range(2):
                g = W.draw_grads(w, j, w.stage_numel()[j], amplified=True, step=k)
                st.set_flat(st.grads, j, g.to(st.storage))
            st.step(w.lam, w.lr)
            st.commit()

    advance(st_a, 0, 4)
    torch.cuda.synchronize()
    heads, valid = plan_a.get_state()
    saved_ring = st_a.ring.clone()
    saved_master = None if st_a.master is None else st_a.master.clone()
    plan_b = B.plan_for_workload(w)
    st_b = B.DeviceState(plan_b, PU.tensors_of(w))
    st_b.ring.copy_(saved_ring)
    if saved_master is not None:
        st_b.master.copy_(saved_master)
    plan_b.set_state(heads, valid)
    advance(st_a, 4, 3)
    advance(st_b, 4, 3)
    torch.cuda.synchronize()
    assert plan_a.get_state() == plan_b.get_state()
    assert torch.equal(st_a.ring, st_b.ring)
    if saved_master is not None:
        assert torch.equal(st_a.master, st_b.master)


# ---- bf16: newest version recomputed from the master ------------------------------------------------
@pytest.mark.parametrize("K", [0, 1, 3, -1])
def test_newest_from_master_gives_identical_results(K):
    """When the newest stored version is the rounded master (as the generator and the library always
    make it), skipping its read must not change a single bit; the oracle is the judge of both."""
    w = W.custom_workload("elide", [[70_000, 40], [30_001], [9_000], [2_048]], [12, 3, 1, 0], 13, K, precision="bf16",
                          seed=91, lam=0.3)
    plan_r, st_r, host = PU.load_workload(w, amplified=True, n_iters=K)
    plan_e, st_e, _ = PU.load_workload(w, amplified=True, n_iters=K, tuning=dict(newest_from_master=1))
    for st in (st_r, st_e):
        st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    PU.check_step_against_oracle(w, plan_e, st_e, host, K=K)
    assert torch.equal(st_r.ring, st_e.ring) and torch.equal(st_r.master, st_e.master)
    assert torch.equal(st_r.grad_out, st_e.grad_out) and torch.equal(st_r.norms, st_e.norms)
    # and it stays true over further steps, because each step stores the rounding of its new master
    for k in range(3):
        for st in (st_r, st_e):
            st.commit()
            st.step(w.lam, w.lr, grad_out=False)
    torch.cuda.synchronize()
    assert torch.equal(st_r.ring, st_e.ring) and torch.equal(st_r.master, st_e.master)


# ---- many small random configurations ------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(int(os.environ.get("FERRET_RANDOM_CASES", "100"))))
def test_random_configurations(seed):
    """Random stage counts, tensor sizes (ragged on purpose), staleness, ring depth, iteration count,
    storage type, chunk size and launch shape, each compared with the oracle."""
    rng = np.random.default_rng(1000 + seed)
    n_stages = int(rng.integers(1, 7))
    R = int(rng.integers(1, 10))
    tau = [int(rng.integers(0, R)) for _ in range(n_stages)]
    sizes = [[int(rng.choice([1, 7, 8, 9, 63, 500, 1024, 2047, 2049, 5000, 30_000]) * rng.integers(1, 4))
              for _ in range(int(rng.integers(1, 5)))] for _ in range(n_stages)]
    K = int(rng.choice([-1, 0, 1, 2, 3, 5, 9]))
    precision = "bf16" if seed % 2 else "f32"
    depth = B.FERRET_RING_DEPTH_MINIMAL if seed % 5 == 0 else R
    chunk = int(rng.choice([0, 1024, 3072, 8192]))
    tuning = [None, dict(blocks_per_cu=2), dict(resident_cap=2), dict(blocks_per_cu=-1, resident_cap=-1),
              dict(cache_policy=2), dict(chunk_bytes=int(rng.choice([1, 20_000, 200_000])), cache_policy=1),
              dict(cache_policy=2, resident_cap=3), dict(xcd_group=int(rng.choice([2, 5, 16])), cache_policy=2),
              dict(xcd_group=int(rng.choice([1, 3, 40])))][seed % 9]
    if tuning and "chunk_bytes" in tuning:
        chunk = 0                                   # a byte target and an explicit size exclude each other
    w = W.custom_workload(f"random{seed}", sizes, tau, R, K, precision=precision, seed=2000 + seed,
                          lam=float(rng.choice([0.1, 0.5, -0.3])), lr=float(rng.choice([0.01, 0.2])))
    heads = [int(rng.integers(0, 16)) for _ in range(n_stages)]
    _run(w, True, chunk_elems=chunk, tuning=tuning, ring_depth=depth, n_iters=K, heads=heads)


@pytest.mark.parametrize("active", [[1, 0, 1, 0], [0, 0, 0, 1], [0, 1, 1, 0], [0, 0, 0, 0], [1, 1, 1, 1]])
@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("blocks_per_cu", [0, 2])
def test_stepping_a_subset_of_stages(precision, blocks_per_cu, active):
    """Stages that take part get exactly what the full step gives them; the others are left alone and have
    nothing to commit."""
    w = W.custom_workload("subset", [[30_000, 8], [12_345], [4_096], [9_000]], [3, 2, 1, 0], 4, 2, precision=precision,
                          seed=61)
    tuning = dict(blocks_per_cu=blocks_per_cu) if blocks_per_cu else None
    plan, st, host = PU.load_workload(w, amplified=True, tuning=tuning)
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    full_ring, full_norms, full_g = st.ring.clone(), st.norms.clone(), st.grad_out.clone()
    full_master = None if st.master is None else st.master.clone()
    plan2, st2, _ = PU.load_workload(w, amplified=True, tuning=tuning)
    before_ring = st2.ring.clone()
    before_master = None if st2.master is None else st2.master.clone()
    st2.norms.fill_(5.0)
    B.ferret_compensate_stages(plan2, st2.ring, st2.grads, st2.master, active, w.lam, w.lr, st2.norms, st2.grad_out,
                               st2.workspace)
    torch.cuda.synchronize()
    for j in range(4):
        lo = plan2.stage_ring_offset(j)
        hi = lo + plan2.stage_slot_stride(j) * plan2.stage_ring_depth(j)
        f0, f1 = plan2.stage_flat_offset(j), plan2.stage_flat_offset(j) + plan2.stage_numel(j)
        want_ring = full_ring if active[j] else before_ring
        assert torch.equal(st2.ring[lo:hi], want_ring[lo:hi]), f"stage {j} ring"
        if st2.master is not None:
            want_m = full_master if active[j] else before_master
            assert torch.equal(st2.master[f0:f1], want_m[f0:f1]), f"stage {j} master"
        if active[j]:
            assert torch.equal(st2.norms[j], full_norms[j]) and torch.equal(st2.grad_out[f0:f1], full_g[f0:f1])
            B.ferret_push_version(plan2, st2.ring, None, j, None)
        else:
            assert not st2.norms[j].any()
            with pytest.raises(B.FerretError) as e:
                B.ferret_push_version(plan2, st2.ring, None, j, None)
            assert e.value.status == B.FERRET_ESTATE


@pytest.mark.parametrize("n_reads", [1, 3, 5, 8])
@pytest.mark.parametrize("cap", [0, 3])
def test_stream_mix_adds_its_streams(n_reads, cap):
    n = 3 * 2048 + 1024 + 4                      # whole workgroups, a partial one, a ragged tail
    stride = n + 12
    src = torch.randn(n_reads * stride, device="cuda")
    dst = torch.full((n + 4,), 7.0, device="cuda")
    B.ferret_stream_mix(dst, src, stride * 4, n_reads, n * 4, cap)
    torch.cuda.synchronize()
    want = torch.zeros(n, device="cuda")
    parts = [src[i * stride:i * stride + n] for i in range(n_reads)]
    want = parts[0].clone()
    for p in parts[1:]:
        want = want + p                           # same left-to-right fp32 order as the kernel
    assert torch.equal(dst[:n], want) and bool((dst[n:] == 7.0).all())


def test_stream_mix_rejects_overlap_and_bad_counts():
    buf = torch.zeros(4096, device="cuda")
    for args in [(buf[1024:], buf, 1024 * 4, 2, 1024 * 4 + 16, 0),      # dst overlaps the second source
                 (buf[2048:], buf, 512 * 4, 2, 1024 * 4, 0),            # sources overlap each other
                 (buf[2048:], buf, 1024 * 4, 9, 16, 0),
                 (buf[2048:], buf, 1024 * 4, 0, 16, 0)]:
        with pytest.raises(B.FerretError) as e:
            B.ferret_stream_mix(*args)
        assert e.value.status == B.FERRET_EINVAL


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_stage_beyond_four_gibibytes_sampled(precision):
    """One stage whose fp32 slot-shaped buffers are larger than 4 GiB (element and byte offsets beyond 32 bits
    inside a stage): the step runs at full size; windows at the start, across the 4 GiB byte boundary and at the
    ragged end are compared with the oracle element by element (the operation is elementwise, so the oracle of a
    window is the window of the oracle), and the norms with fp64 reductions over the whole stage."""
    n_big = (1 << 30) + (1 << 20) + 3 * 2048 + 1024 + 8
    lam, lr, K = 0.5, 0.01, -1
    bf16 = precision == "bf16"
    dt = torch.bfloat16 if bf16 else torch.float32
    plan = B.ferret_plan_buckets([(10_000, 0), (n_big, 1)], 2, [1, 2], K, 3,
                                 B.FERRET_BF16_MASTER_F32 if bf16 else B.FERRET_F32, 0)
    assert plan.stage_numel(1) == n_big and plan.stage_numel(1) * 4 > (1 << 32)
    gen = torch.Generator(device="cuda").manual_seed(71)
    ring = torch.empty(plan.ring_elems, device="cuda", dtype=dt).normal_(0.0, 0.05, generator=gen)
    grads = torch.empty(plan.flat_elems, device="cuda", dtype=dt).normal_(0.0, 1.0, generator=gen)
    master = torch.empty(plan.flat_elems, device="cuda").normal_(0.0, 0.05, generator=gen) if bf16 else None
    grad_out = torch.zeros(plan.flat_elems, device="cuda")
    norms = torch.zeros(2, 3, device="cuda")
    workspace = torch.zeros(plan.workspace_bytes // 4, device="cuda")
    plan.set_state([2, 2], [3, 3])
    assert plan.stage_read_slots(1) == [0, 1, 2] and plan.stage_write_slot(1) == 0
    off = [plan.slot_offset(1, s) for s in range(3)]
    f0 = plan.stage_flat_offset(1)
    W_ = 1 << 19
    windows = [(0, W_), ((1 << 30) - W_, (1 << 30) + W_), (n_big - W_, n_big)]
    before = [[ring[off[s] + a: off[s] + b].cpu().clone() for s in range(3)] for a, b in windows]
    master_before = [master[f0 + a: f0 + b].cpu().clone() for a, b in windows] if bf16 else None
    # reference sums for the norms, taken before the step overwrites the oldest slot
    def sq_sum(x):
        return sum(float((p.double() ** 2).sum()) for p in x.split(1 << 28))
    want_n0 = sq_sum(grads[f0: f0 + n_big])
    want_n2 = sum(float(((a.double() - b.double()) ** 2).sum())
                  for a, b in zip(ring[off[2]: off[2] + n_big].split(1 << 28), ring[off[0]: off[0] + n_big].split(1 << 28)))
    B.ferret_compensate_step(plan, ring, grads, master, lam, lr, norms, grad_out, workspace)
    torch.cuda.synchronize()
    for k, ((a, b), vs) in enumerate(zip(windows, before)):
        g = grads[f0 + a: f0 + b].cpu()
        assert g.numel() == b - a and all(v.numel() == b - a for v in vs)
        tag = f"window [{a}, {b})"
        got_new = ring[off[0] + a: off[0] + b].cpu()
        if bf16:
            new, m_new, g_ref, _ = O.compensate_stage_bf16(vs, g, master_before[k], K, np.float32(lam), np.float32(lr))
            got_m = master[f0 + a: f0 + b].cpu().numpy()
            PU.assert_close_f32(got_m, m_new, tag + " master")
            slack = PU.master_slack(m_new, lr, np.maximum(np.abs(g_ref), np.abs(g.float().numpy())), 2)
            PU.assert_master_within_slack(got_m, m_new, slack, tag + " master")
            PU.assert_bf16_within_one_ulp(PU.bits_of(got_new), new, tag + " new version", abs_slack=slack)
            PU.assert_bf16_is_rounded_master(PU.bits_of(got_new), got_m, tag)
        else:
            new, g_ref, _ = O.compensate_stage_f32(vs, g, K, np.float32(lam), np.float32(lr))
            PU.assert_close_f32(got_new.numpy(), new, tag + " new version")
        PU.assert_close_f32(grad_out[f0 + a: f0 + b].cpu().numpy(), g_ref, tag + " g_K'")
    got = norms.cpu().numpy().astype(np.float64)
    assert got[1, 0] == pytest.approx(want_n0, rel=PU.RTOL)
    assert got[1, 2] == pytest.approx(want_n2, rel=PU.RTOL)
    assert got[1, 1] == pytest.approx(sq_sum(grad_out[f0: f0 + n_big]), rel=PU.RTOL)
    # the slots that are only read are untouched
    for s in (1, 2):
        for (a, b), vs in zip(windows, before):
            assert torch.equal(ring[off[s] + a: off[s] + b].cpu(), vs[s])


# ---- per-launch timing sessions ------------------------------------------------------------------------
def test_profile_session_belongs_to_the_thread_that_began_it():
    """Only the owner's launches are recorded; another thread can neither begin a second session nor end this one."""
    import threading
    w = W.custom_workload("prof", [[50_000], [20_000]], [1, 0], 2, 1, seed=88)
    plan, st, _ = PU.load_workload(w, amplified=True)
    torch.cuda.synchronize()
    B.ferret_profile_begin(8)
    other = {}

    def intruder():
        try:
            B.ferret_profile_begin(4)
        except B.FerretError as e:
            other["begin"] = e.status
        plan2, st2, _ = PU.load_workload(w, amplified=True)
        st2.step(w.lam, w.lr)                       # a launch from another thread: not recorded
        torch.cuda.synchronize()
        try:
            B.ferret_profile_end(8)
        except B.FerretError as e:
            other["end"] = e.status

    t = threading.Thread(target=intruder)
    t.start()
    t.join()
    assert other == {"begin": B.FERRET_ESTATE, "end": B.FERRET_ESTATE}
    for _ in range(3):
        st.step(w.lam, w.lr)
    ms = B.ferret_profile_end(8)
    assert len(ms) == 3 and all(0.0 < x < 50.0 for x in ms)
    with pytest.raises(B.FerretError) as e:
        B.ferret_profile_end(8)
    assert e.value.status == B.FERRET_ESTATE
