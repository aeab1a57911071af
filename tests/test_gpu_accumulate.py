"""GPU parity of the gradient-accumulation step (T2) against the oracle."""
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
        pytest.fail("these tests need a GPU")
    B.load()


def _accum_call(plan, st, accum, scale, mode, staleness, lam, lr):
    B.ferret_accumulate_step(plan, st.ring, st.grads, st.master, accum, scale, mode, staleness, lam, lr,
                             st.norms, st.grad_out, st.workspace)
    torch.cuda.synchronize()


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_accumulation_groups_with_varying_staleness(precision):
    """Three stages with c^a = 3, 2, 1 and delays of 4, 3, 0 micro-steps; staleness counted in versions
    changes from arrival to arrival; some calls skip a stage, some only accumulate, some update."""
    ca, delay = [3, 2, 1], [4, 3, 0]
    tau_max = [-(-d // c) for d, c in zip(delay, ca)]                  # ceil: 2, 2, 0
    w = W.custom_workload("accumulate", [[30_000, 40], [9_001], [4_096]], tau_max, 3, -1, precision=precision, seed=51,
                          lam=0.4, lr=0.02)
    plan, st, host = PU.load_workload(w, amplified=True, ring_depth=B.FERRET_RING_DEPTH_MINIMAL)
    assert [plan.stage_ring_depth(j) for j in range(3)] == [1 + t for t in tau_max]
    bf16 = precision == "bf16"
    accum = torch.zeros(plan.flat_elems, device="cuda")
    acc_host = [np.zeros(n, np.float32) for n in w.stage_numel()]
    versions = [list(d.versions) for d in host]                        # oldest .. newest per stage
    master = [None if d.master is None else d.master.numpy().copy() for d in host]
    updates = [0, 0, 0]
    for m in range(13):                                                # micro-steps
        mode, stale = [], []
        for j in range(3):
            if j == 1 and m % 5 == 4:                                  # stage 1 sometimes receives nothing
                mode.append(0); stale.append(0); continue
            arrivals_in_group = (m - (m // 5 if j == 1 else 0)) % ca[j]
            last = arrivals_in_group == ca[j] - 1
            mode.append(2 if last else 1)
            stale.append(min(tau_max[j], (m * 7 + j) % (tau_max[j] + 1)))
        for j in range(3):
            g = W.draw_grads(w, j, w.stage_numel()[j], amplified=True, step=m)
            g = g.to(torch.bfloat16) if bf16 else g
            st.set_flat(st.grads, j, g)
            host[j].grads = g
        write_slots = [plan.stage_write_slot(j) for j in range(3)]
        _accum_call(plan, st, accum, 1.0 / 3.0, mode, stale, w.lam, w.lr)
        norms = st.norms.cpu().numpy()
        for j in range(3):
            tag = f"micro-step {m} stage {j} mode {mode[j]}"
            got_acc = st.get_flat(accum, j).numpy()
            if mode[j] == 0:
                assert np.array_equal(got_acc, acc_host[j]), tag
                assert not norms[j].any()
                continue
            tau = min(stale[j], len(versions[j]) - 1)
            window = versions[j][len(versions[j]) - 1 - tau:]
            ref = O.accumulate_stage(window, host[j].grads, master[j], -1, np.float32(w.lam), np.float32(w.lr),
                                     np.float32(1.0 / 3.0), mode[j] == 2, acc_host[j], bf16=bf16)
            PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], tag + " g")
            PU.assert_close_f32(got_acc, ref["accum"], tag + " accum")
            acc_before, acc_host[j] = acc_host[j], got_acc.copy()
            if mode[j] == 2:
                got_new = st.get_version(j, write_slots[j])
                if bf16:
                    got_m = st.get_flat(st.master, j).numpy()
                    PU.assert_close_f32(got_m, ref["master"], tag + " master")
                    # eta multiplies scale * (running sum + this compensated gradient), scale <= 1
                    slack = PU.master_slack(ref["master"], w.lr, np.abs(acc_before) + np.abs(ref["g"]), tau + 2)
                    PU.assert_master_within_slack(got_m, ref["master"], slack, tag + " master")
                    PU.assert_bf16_within_one_ulp(PU.bits_of(got_new), ref["new"], tag + " version", abs_slack=slack)
                    PU.assert_bf16_is_rounded_master(PU.bits_of(got_new), got_m, tag)
                    master[j] = got_m.copy()
                else:
                    PU.assert_close_f32(got_new.numpy(), ref["new"], tag + " version")
                versions[j] = (versions[j] + [got_new])[-plan.stage_ring_depth(j):]
                B.ferret_push_version(plan, st.ring, None, j, None)
                updates[j] += 1
                assert not got_acc.any()
    assert updates[0] >= 3 and updates[1] >= 4 and updates[2] == 13


def test_one_arrival_groups_equal_the_plain_step_bit_for_bit():
    w = W.custom_workload("accumulate_ca1", [[60_000], [20_000], [5_000]], [3, 1, 0], 5, 2, seed=52)
    plan, st, host = PU.load_workload(w, amplified=True)
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    want = [st.get_version(j, plan.stage_write_slot(j)) for j in range(3)]
    want_norms = st.norms.cpu().clone()
    accum = torch.zeros(plan.flat_elems, device="cuda")
    _accum_call(plan, st, accum, 1.0, [2, 2, 2], None, w.lam, w.lr)
    for j in range(3):
        assert torch.equal(st.get_version(j, plan.stage_write_slot(j)), want[j])
    assert torch.equal(st.norms.cpu(), want_norms) and not accum.any()


def test_skipped_stage_is_left_alone():
    w = W.custom_workload("accumulate_skip", [[10_000], [10_000]], [1, 1], 2, -1, seed=53)
    plan, st, host = PU.load_workload(w, amplified=True)
    ring_before = st.ring.clone()
    accum = torch.full((plan.flat_elems,), 7.0, device="cuda")
    _accum_call(plan, st, accum, 1.0, [0, 1], None, w.lam, w.lr)
    n0 = plan.stage_numel(0)
    assert torch.equal(st.ring, ring_before)                           # nobody updated
    assert torch.equal(accum[:n0].cpu(), torch.full((n0,), 7.0))
    with pytest.raises(B.FerretError) as e:                            # nothing to commit either
        B.ferret_push_version(plan, st.ring, None, 1, None)
    assert e.value.status == B.FERRET_ESTATE


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_accumulation_with_self_tuned_lambda(precision, fused):
    """Per-arrival lambda block + accumulation over several groups: lambda_j, v_r, v_a, the running sum and the
    versions follow the oracle; a skipped stage keeps its lambda and averages."""
    ca, tau_max = [2, 3, 1], [2, 1, 0]
    w = W.custom_workload("accumulate_adaptive", [[25_000, 72], [8_193], [4_096]], tau_max, 3, -1,
                          precision=precision, seed=54, lam=0.3, lr=0.02)
    plan, st, host = PU.load_workload(w, amplified=True, ring_depth=B.FERRET_RING_DEPTH_MINIMAL)
    bf16 = precision == "bf16"
    st.enable_adaptive(w.lam)
    accum = torch.zeros(plan.flat_elems, device="cuda")
    n = w.stage_numel()
    acc_host = [np.zeros(k, np.float32) for k in n]
    state = [(np.zeros(k, np.float32), np.zeros(k, np.float32)) for k in n]
    lams = [np.float32(w.lam)] * 3
    versions = [list(d.versions) for d in host]
    master = [None if d.master is None else d.master.numpy().copy() for d in host]
    alpha, eta_l, scale = 0.75, 2e-3, 0.5
    count = [0, 0, 0]
    for m in range(9):
        mode, stale = [], []
        for j in range(3):
            if j == 0 and m == 4:
                mode.append(0); stale.append(0); continue
            count[j] += 1
            mode.append(2 if count[j] % ca[j] == 0 else 1)
            stale.append((m + j) % (tau_max[j] + 1))
        for j in range(3):
            g = W.draw_grads(w, j, n[j], amplified=True, step=m)
            g = g.to(torch.bfloat16) if bf16 else g
            st.set_flat(st.grads, j, g)
            host[j].grads = g
        write_slots = [plan.stage_write_slot(j) for j in range(3)]
        B.ferret_accumulate_step_adaptive(plan, st.ring, st.grads, st.master, accum, scale, mode, stale, st.lambda_dev,
                                          st.v_r, st.v_a, alpha, eta_l, w.lr, st.norms, st.grad_out, st.workspace,
                                          fused=fused)
        torch.cuda.synchronize()
        lam_gpu = st.lambda_dev.cpu().numpy()
        for j in range(3):
            tag = f"micro-step {m} stage {j} mode {mode[j]}"
            got_r, got_a = st.get_flat(st.v_r, j).numpy(), st.get_flat(st.v_a, j).numpy()
            if mode[j] == 0:
                assert lam_gpu[j] == lams[j], tag
                assert np.array_equal(got_r, state[j][0]) and np.array_equal(got_a, state[j][1]), tag
                assert np.array_equal(st.get_flat(accum, j).numpy(), acc_host[j]), tag
                continue
            tau = min(stale[j], len(versions[j]) - 1)
            window = versions[j][len(versions[j]) - 1 - tau:]
            ref = O.accumulate_stage_adaptive(window, host[j].grads, master[j], -1, lams[j], np.float32(alpha),
                                              np.float32(eta_l), np.float32(w.lr), np.float32(scale), mode[j] == 2,
                                              acc_host[j], state[j][0], state[j][1], bf16=bf16, lambda_step_last=fused)
            assert lam_gpu[j] == pytest.approx(ref["lam"], rel=1e-5), tag + " lambda"
            if tau == 0:
                assert lam_gpu[j] == lams[j], tag
            PU.assert_close_f32(got_r, ref["v_r"], tag + " v_r")
            PU.assert_close_f32(got_a, ref["v_a"], tag + " v_a")
            PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], tag + " g")
            got_acc = st.get_flat(accum, j).numpy()
            PU.assert_close_f32(got_acc, ref["accum"], tag + " accum")
            acc_before = acc_host[j]
            acc_host[j], state[j], lams[j] = got_acc.copy(), (got_r.copy(), got_a.copy()), lam_gpu[j]
            if mode[j] == 2:
                got_new = st.get_version(j, write_slots[j])
                if bf16:
                    got_m = st.get_flat(st.master, j).numpy()
                    PU.assert_close_f32(got_m, ref["master"], tag + " master")
                    # eta multiplies scale * (running sum + this compensated gradient), scale <= 1
                    # lambda_j itself is only held to 1e-5 relative, and the correction g_K' - g_0 scales with it
                    slack = PU.master_slack(ref["master"], w.lr, np.abs(acc_before) + np.abs(ref["g"]), tau + 2,
                                            extra=abs(w.lr) * 2e-5 * np.abs(ref["g"].astype(np.float64) - host[j].grads.float().numpy()))
                    PU.assert_master_within_slack(got_m, ref["master"], slack, tag + " master")
                    PU.assert_bf16_within_one_ulp(PU.bits_of(got_new), ref["new"], tag + " version", abs_slack=slack)
                    master[j] = got_m.copy()
                else:
                    PU.assert_close_f32(got_new.numpy(), ref["new"], tag + " version")
                versions[j] = (versions[j] + [got_new])[-plan.stage_ring_depth(j):]
                B.ferret_push_version(plan, st.ring, None, j, None)
    assert lams[0] != np.float32(w.lam) and lams[2] == np.float32(w.lam)


@pytest.mark.parametrize("seed", range(24))
def test_random_accumulation_schedules(seed):
    """Random stages, sizes, ring depths, iteration counts, chunk sizes and per-call (mode, staleness) patterns,
    with and without the self-tuned lambda (either ordering); every call is compared with the oracle."""
    rng = np.random.default_rng(5000 + seed)
    P = int(rng.integers(1, 5))
    tau_max = [int(rng.integers(0, 4)) for _ in range(P)]
    sizes = [[int(rng.choice([8, 63, 500, 1024, 2049, 7000]) * rng.integers(1, 4)) for _ in range(int(rng.integers(1, 3)))]
             for _ in range(P)]
    K = int(rng.choice([-1, 1, 2]))
    bf16 = bool(seed % 2)
    adaptive = (seed // 2) % 3            # 0: fixed lambda, 1: Alg. 1's order, 2: one pass
    w = W.custom_workload(f"random_accum{seed}", sizes, tau_max, max(tau_max) + 1, K,
                          precision="bf16" if bf16 else "f32", seed=6000 + seed, lam=0.3, lr=0.05)
    plan, st, host = PU.load_workload(w, amplified=True, ring_depth=B.FERRET_RING_DEPTH_MINIMAL,
                                      chunk_elems=int(rng.choice([0, 1024, 4096])))
    if adaptive:
        st.enable_adaptive(w.lam)
    n = w.stage_numel()
    accum = torch.zeros(plan.flat_elems, device="cuda")
    acc_host = [np.zeros(k, np.float32) for k in n]
    state = [(np.zeros(k, np.float32), np.zeros(k, np.float32)) for k in n]
    lams = [np.float32(w.lam)] * P
    versions = [list(d.versions) for d in host]
    master = [None if d.master is None else d.master.numpy().copy() for d in host]
    alpha, eta_l, scale = 0.5, 1e-3, float(rng.choice([1.0, 0.5]))
    for m in range(6):
        mode = [int(rng.choice([0, 1, 1, 2])) for _ in range(P)]
        stale = [int(rng.integers(0, tau_max[j] + 1)) for j in range(P)]
        for j in range(P):
            g = W.draw_grads(w, j, n[j], amplified=True, step=m)
            g = g.to(torch.bfloat16) if bf16 else g
            st.set_flat(st.grads, j, g)
            host[j].grads = g
        write_slots = [plan.stage_write_slot(j) for j in range(P)]
        if adaptive:
            B.ferret_accumulate_step_adaptive(plan, st.ring, st.grads, st.master, accum, scale, mode, stale,
                                              st.lambda_dev, st.v_r, st.v_a, alpha, eta_l, w.lr, st.norms, st.grad_out,
                                              st.workspace, fused=adaptive == 2)
        else:
            B.ferret_accumulate_step(plan, st.ring, st.grads, st.master, accum, scale, mode, stale, w.lam, w.lr,
                                     st.norms, st.grad_out, st.workspace)
        torch.cuda.synchronize()
        lam_gpu = st.lambda_dev.cpu().numpy() if adaptive else None
        for j in range(P):
            tag = f"seed {seed} call {m} stage {j} mode {mode[j]}"
            got_acc = st.get_flat(accum, j).numpy()
            if mode[j] == 0:
                assert np.array_equal(got_acc, acc_host[j]), tag
                continue
            tau = min(stale[j], len(versions[j]) - 1)
            window = versions[j][len(versions[j]) - 1 - tau:]
            if adaptive:
                ref = O.accumulate_stage_adaptive(window, host[j].grads, master[j], K, lams[j], np.float32(alpha),
                                                  np.float32(eta_l), np.float32(w.lr), np.float32(scale), mode[j] == 2,
                                                  acc_host[j], state[j][0], state[j][1], bf16=bf16,
                                                  lambda_step_last=adaptive == 2)
                assert lam_gpu[j] == pytest.approx(ref["lam"], rel=1e-5), tag + " lambda"
                got_r, got_a = st.get_flat(st.v_r, j).numpy(), st.get_flat(st.v_a, j).numpy()
                PU.assert_close_f32(got_r, ref["v_r"], tag + " v_r")
                PU.assert_close_f32(got_a, ref["v_a"], tag + " v_a")
                state[j], lams[j] = (got_r.copy(), got_a.copy()), lam_gpu[j]
            else:
                ref = O.accumulate_stage(window, host[j].grads, master[j], K, np.float32(w.lam), np.float32(w.lr),
                                         np.float32(scale), mode[j] == 2, acc_host[j], bf16=bf16)
            PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], tag + " g")
            PU.assert_close_f32(got_acc, ref["accum"], tag + " accum")
            acc_before, acc_host[j] = acc_host[j], got_acc.copy()
            if mode[j] == 2:
                got_new = st.get_version(j, write_slots[j])
                if bf16:
                    got_m = st.get_flat(st.master, j).numpy()
                    PU.assert_close_f32(got_m, ref["master"], tag + " master")
                    # eta multiplies scale * (running sum + this compensated gradient), scale <= 1
                    slack = PU.master_slack(ref["master"], w.lr, np.abs(acc_before) + np.abs(ref["g"]), O.effective_iters(K, tau) + 2,
                                            extra=abs(w.lr) * 2e-5 * np.abs(ref["g"].astype(np.float64) - host[j].grads.float().numpy()) if adaptive else 0.0)
                    PU.assert_master_within_slack(got_m, ref["master"], slack, tag + " master")
                    PU.assert_bf16_within_one_ulp(PU.bits_of(got_new), ref["new"], tag + " version", abs_slack=slack)
                    master[j] = got_m.copy()
                else:
                    PU.assert_close_f32(got_new.numpy(), ref["new"], tag + " version")
                versions[j] = (versions[j] + [got_new])[-plan.stage_ring_depth(j):]
                B.ferret_push_version(plan, st.ring, None, j, None)
