"""GPU parity at the full benchmark shapes for every mode bench.py times, in the launch configuration it times
(default chunking, grid and resident-workgroup cap), element by element against the CPU oracle:

  ViT-B-sized, fp32 (86.6 M parameters, 8 stages)
      one iteration per version step (Alg. 1 literally; the K' <= 8 kernels under the cap)
      the same with the self-tuned lambda: Alg. 1 as printed, and its block fused into the step (one pass)
      gradient accumulation with c^a = 2 (T2 in Sec. "Fine-grained Pipeline Parallelism")
  350 M parameters, bf16 versions + fp32 master, 16 stages
      one iteration per version step (K' up to 15: the streamed kernels under the cap), amplified inputs
      the newest version recomputed from the master
      self-tuned lambda, Alg. 1's order and the one-pass order

The default-K steps of both shapes, the self-tuned step at the ViT-B shape and the penalised steps are covered at
full size in test_gpu_parity.py, test_gpu_adaptive.py and test_gpu_penalized.py.  One set of device buffers is loaded
per shape and reused: after a check, the slot the step wrote and the master are put back from the host copy.
"""
import numpy as np
import pytest
import torch

from oracle import ferret_oracle as O
from paper_2503_12053_amd import binding as B
from paper_2503_12053_amd import workloads as W

import parity_util as PU
from test_gpu_adaptive import _check as check_adaptive, _state as adaptive_state

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    B.load()


class Loaded:
    """A workload resident on the device with every ring slot valid, plus the host copy for the oracle."""

    def __init__(self, idx, amplified):
        self.w = W.make_workload(idx)
        print(f"[load] {self.w.name} amplified={amplified}", flush=True)
        self.plan, self.st, self.host = PU.load_workload(self.w, amplified=amplified)
        self.heads, self.valid = self.plan.get_state()

    def plan_like(self, **kw):
        """Another plan over the same buffers (same layout; chunking, iteration count or tuning differ)."""
        plan = B.plan_for_workload(self.w, **kw)
        assert plan.ring_elems == self.plan.ring_elems and plan.flat_elems == self.plan.flat_elems
        assert [plan.stage_slot_stride(j) for j in range(self.w.n_stages)] == \
               [self.plan.stage_slot_stride(j) for j in range(self.w.n_stages)]
        plan.set_state(self.heads, self.valid)
        return plan

    def restore(self, plan):
        """Undo a step: the slot it wrote held the oldest version (the ring is full), the master was replaced."""
        for j in range(self.w.n_stages):
            self.st.set_version(j, plan.stage_write_slot(j), self.host[j].versions[0])
            if self.host[j].master is not None:
                self.st.set_flat(self.st.master, j, self.host[j].master)
        torch.cuda.synchronize()

    def state_for(self, plan):
        """The device buffers seen through another plan (DeviceState does no arithmetic; it only holds buffers)."""
        st = B.DeviceState.__new__(B.DeviceState)
        st.__dict__.update(self.st.__dict__)
        st.plan = plan
        need = max(plan.workspace_bytes // 4, 4)
        if st.workspace.numel() < need:
            st.workspace = torch.zeros(need, dtype=torch.float32, device=st.device)
        return st


@pytest.fixture(scope="module")
def vit_amplified():
    return Loaded(4, True)


@pytest.fixture(scope="module")
def mixed_nominal():
    return Loaded(5, False)


# ---- ViT-B-sized, fp32 ---------------------------------------------------------------------------------
def test_vit_b_one_iteration_per_version_step(vit_amplified):
    L = vit_amplified
    plan = L.plan_like(n_iters=B.FERRET_ITERS_FULL)
    assert [plan.stage_effective_iters(j) for j in range(8)] == [7, 6, 5, 4, 3, 2, 1, 0]
    assert [plan.stage_chunk_elems(j) for j in range(8)] == [1024, 1024, 2048, 2048, 2048, 2048, 3072, 4096]
    st = L.state_for(plan)
    st.step(L.w.lam, L.w.lr)
    torch.cuda.synchronize()
    PU.check_step_against_oracle(L.w, plan, st, L.host, K=-1, n_threads=8, label="full iterations ")
    L.restore(plan)


@pytest.mark.parametrize("fused", [False, True])
def test_vit_b_self_tuned_lambda_with_one_iteration_per_version_step(vit_amplified, fused):
    """bench.py --adaptive / --adaptive-fused with --iters -1: Alg. 1 as printed (the lambda block, then one iteration
    per version step, stages with K' = 7 ... 0), and the same with the block fused into the step."""
    L = vit_amplified
    w = L.w
    plan = L.plan_like(n_iters=B.FERRET_ITERS_FULL)
    st = L.state_for(plan)
    state = adaptive_state(w, st, 36, w.lam)
    st.step_adaptive(0.9, 1e-5, w.lr, fused=fused)
    torch.cuda.synchronize()
    check_adaptive(w, plan, st, L.host, state, [w.lam] * w.n_stages, 0.9, 1e-5, -1, "vit full iterations", fused,
                   n_threads=8)
    L.restore(plan)         # the averages and lambda live on `st`, a view of the buffers that ends here


def test_vit_b_accumulation_of_two_gradients(vit_amplified):
    """bench.py --accumulate 2: two arrivals per stage with the plan's staleness, the second one updates."""
    L = vit_amplified
    w, plan, st = L.w, L.plan, L.st
    accum = torch.zeros(plan.flat_elems, device="cuda")
    acc_host = [np.zeros(n, np.float32) for n in w.stage_numel()]
    slots = [plan.stage_write_slot(j) for j in range(w.n_stages)]
    for arrival, mode in enumerate([1, 2]):
        grads = []
        for j in range(w.n_stages):
            g = W.draw_grads(w, j, w.stage_numel()[j], amplified=True, step=200 + arrival)
            st.set_flat(st.grads, j, g)
            grads.append(g)
        B.ferret_accumulate_step(plan, st.ring, st.grads, None, accum, 0.5, [mode] * w.n_stages, None, w.lam, w.lr,
                                 st.norms, st.grad_out, st.workspace)
        torch.cuda.synchronize()
        norms = st.norms.cpu().numpy().astype(np.float64)
        for j in range(w.n_stages):
            tau = plan.stage_effective_staleness(j)
            window = L.host[j].versions[len(L.host[j].versions) - 1 - tau:]
            ref = O.accumulate_stage(window, grads[j], None, w.n_iters, np.float32(w.lam), np.float32(w.lr),
                                     np.float32(0.5), mode == 2, acc_host[j], bf16=False)
            tag = f"arrival {arrival} stage {j}"
            PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], tag + " g_K'")
            got_acc = st.get_flat(accum, j).numpy()
            PU.assert_close_f32(got_acc, ref["accum"], tag + " running sum")
            acc_host[j] = got_acc.copy()
            want_norms = [float((grads[j].double() ** 2).sum()), float((ref["g"] ** 2).sum()),
                          float(((window[-1].double() - window[0].double()) ** 2).sum())]
            np.testing.assert_allclose(norms[j], want_norms, rtol=PU.RTOL, atol=1e-30, err_msg=tag + " norms")
            if mode == 2:
                PU.assert_close_f32(st.get_version(j, slots[j]).numpy(), ref["new"], tag + " new version")
                assert not got_acc.any(), tag + ": the sum is cleared by the update"
            else:       # an arrival that only accumulates writes no version
                assert torch.equal(st.get_version(j, slots[j]), L.host[j].versions[0]), tag
        print(f"  checked arrival {arrival}", flush=True)
    for j in range(w.n_stages):
        st.set_flat(st.grads, j, L.host[j].grads)
    L.restore(plan)


# ---- 350 M parameters, bf16 + fp32 master ----------------------------------------------------------------
@pytest.mark.timeout(900)
def test_mixed_350m_newest_version_from_master(mixed_nominal):
    L = mixed_nominal
    plan = L.plan_like(tuning=dict(newest_from_master=1))
    st = L.state_for(plan)
    st.step(L.w.lam, L.w.lr)
    torch.cuda.synchronize()
    PU.check_step_against_oracle(L.w, plan, st, L.host, n_threads=8, label="newest from master ")
    L.restore(plan)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("fused", [False, True])
def test_mixed_350m_self_tuned_lambda(mixed_nominal, fused):
    L = mixed_nominal
    w, plan, st = L.w, L.plan, L.st
    state = adaptive_state(w, st, 35, w.lam)
    st.step_adaptive(0.9, 1e-5, w.lr, fused=fused)
    torch.cuda.synchronize()
    check_adaptive(w, plan, st, L.host, state, [w.lam] * w.n_stages, 0.9, 1e-5, w.n_iters, "350m", fused, n_threads=8)
    del st.v_r, st.v_a, st.lambda_dev
    L.restore(plan)


@pytest.mark.timeout(900)
def test_mixed_350m_one_iteration_per_version_step_amplified(mixed_nominal):
    """All 16 stages at full size with the compensation term at a few per cent of the gradient, so that a wrong K' or
    boundary table in any stage shows; the inputs are swapped for amplified ones stage by stage (the host copy of the
    nominal ones is dropped first to bound memory).  Amplified here means g ~ N(0, 1) without the x100 tail and
    drift ~ N(0, 0.05) with lambda = 0.05: each of up to 15 iterations then moves g by about 0.25 % (4 % in all),
    and no element comes near the point where the recurrence g <- g + lambda g^2 delta runs away, which fp32 and
    fp64 would do at different speeds (with the x100 tail it overflows fp32 within 15 iterations)."""
    import dataclasses
    L = mixed_nominal
    w = dataclasses.replace(L.w, heavy_tail=None, lam=0.05)
    plan = L.plan_like(n_iters=B.FERRET_ITERS_FULL)
    assert [plan.stage_effective_iters(j) for j in range(16)] == list(range(15, -1, -1))
    st = L.state_for(plan)
    L.host.clear()
    host = []
    generated = PU.map_stages(lambda j: W.generate_stage(w, j, True, n_versions=w.ring_depth), w.n_stages, True)
    for j in range(w.n_stages):
        d = generated[j]
        assert st.load_versions(j, d.versions, L.heads[j]) == L.heads[j]
        st.set_flat(st.grads, j, d.grads)
        st.set_flat(st.master, j, d.master)
        host.append(d)
        print(f"  loaded amplified stage {j}", flush=True)
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    PU.check_step_against_oracle(w, plan, st, host, K=-1, n_threads=8, label="full iterations amplified ")
