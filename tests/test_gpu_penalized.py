"""GPU parity of the step-size-penalising comparison methods against the oracle."""
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


@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("method", ["step-aware", "gap-aware", "both"])
def test_penalized_step(precision, method):
    tau = [5, 2, 1, 0]
    w = W.custom_workload("penalized", [[40_000, 24], [15_001], [9_000], [2_048]], tau, 6, 3, precision=precision,
                          seed=95, lr=0.05)
    plan, st, host = PU.load_workload(w, amplified=True)
    C = [0.05, 0.02, 0.1, 0.3]
    scale = None if method == "step-aware" else ([1.0] * 4 if method == "gap-aware" else [0.5, 2.0, 1.0, 0.25])
    inv_c = None if method == "step-aware" else [1.0 / c for c in C]
    B.ferret_penalized_step(plan, st.ring, st.grads, st.master, scale, inv_c, w.lr, st.norms, st.grad_out, st.workspace)
    torch.cuda.synchronize()
    norms = st.norms.cpu().numpy()
    bf16 = precision == "bf16"
    for j in range(4):
        d = host[j]
        t = plan.stage_effective_staleness(j)
        sc = np.float32(1.0) / np.float32(max(t, 1)) if scale is None else np.float32(scale[j])
        ic = np.float32(0.0) if inv_c is None else np.float32(inv_c[j])
        ref = O.penalized_stage(d.versions[len(d.versions) - 1 - t], d.versions[-1], d.grads, d.master, np.float32(w.lr),
                                sc, ic, bf16=bf16)
        tag = f"{method} stage {j}"
        PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], tag + " penalised gradient")
        slot = plan.stage_write_slot(j)
        if bf16:
            got_m = st.get_flat(st.master, j).numpy()
            PU.assert_close_f32(got_m, ref["master"], tag + " master")
            slack = PU.master_slack(ref["master"], w.lr, np.abs(ref["g"]), 1)      # one division instead of iterations
            PU.assert_master_within_slack(got_m, ref["master"], slack, tag + " master")
            bits = PU.bits_of(st.get_version(j, slot))
            PU.assert_bf16_within_one_ulp(bits, ref["new"], tag + " version", abs_slack=slack)
            PU.assert_bf16_is_rounded_master(bits, got_m, tag)
        else:
            PU.assert_close_f32(st.get_version(j, slot).numpy(), ref["new"], tag + " version")
        g64 = d.grads.double().numpy()
        assert norms[j][0] == pytest.approx(float(g64 @ g64), rel=1e-5) and norms[j][1] == norms[j][0]
    st.commit()


def test_unit_penalty_is_the_uncompensated_step_bit_for_bit():
    w = W.custom_workload("penalized_none", [[50_000], [10_000]], [3, 1], 5, 0, seed=96)      # K = 0: "None"
    plan, st, host = PU.load_workload(w, amplified=True, n_iters=0)
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    want = [st.get_version(j, plan.stage_write_slot(j)) for j in range(2)]
    B.ferret_penalized_step(plan, st.ring, st.grads, None, [1.0, 1.0], [0.0, 0.0], w.lr, None, None, None)
    torch.cuda.synchronize()
    for j in range(2):
        assert torch.equal(st.get_version(j, plan.stage_write_slot(j)), want[j])


@pytest.mark.parametrize("method", ["step-aware", "gap-aware"])
def test_penalized_step_at_benchmark_shape(method):
    """ViT-B-sized workload, the launch configuration bench.py --compensator step-aware / gap-aware times."""
    w = W.make_workload(4)
    plan, st, host = PU.load_workload(w, amplified=True)
    gap = method == "gap-aware"
    scale = [1.0] * w.n_stages if gap else None
    inv_c = [1.0 / (w.lr * w.grad_std)] * w.n_stages if gap else None
    B.ferret_penalized_step(plan, st.ring, st.grads, st.master, scale, inv_c, w.lr, st.norms, st.grad_out, st.workspace)
    torch.cuda.synchronize()
    for j in range(w.n_stages):
        d = host[j]
        t = plan.stage_effective_staleness(j)
        sc = np.float32(1.0) / np.float32(max(t, 1)) if scale is None else np.float32(scale[j])
        ic = np.float32(0.0) if inv_c is None else np.float32(inv_c[j])
        ref = O.penalized_stage(d.versions[len(d.versions) - 1 - t], d.versions[-1], d.grads, None, np.float32(w.lr),
                                sc, ic)
        tag = f"{method} stage {j}"
        PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], tag + " penalised gradient")
        PU.assert_close_f32(st.get_version(j, plan.stage_write_slot(j)).numpy(), ref["new"], tag + " version")
