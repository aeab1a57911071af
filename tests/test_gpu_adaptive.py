"""GPU parity of the self-tuned-lambda step (all of Alg. 1) against the oracle."""
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


def _state(w, st, seed, lam0):
    """Random non-trivial averages so that the first step already moves lambda."""
    st.enable_adaptive(lam0)

    def draw(j):
        g = torch.Generator().manual_seed(seed * 100 + j)
        n = w.stage_numel()[j]
        return torch.randn(n, generator=g), torch.randn(n, generator=g) * 0.05

    host = []
    for j, (vr, va) in enumerate(PU.map_stages(draw, w.n_stages, w.numel > PU.BIG)):
        st.set_flat(st.v_r, j, vr)
        st.set_flat(st.v_a, j, va)
        host.append((vr.numpy().copy(), va.numpy().copy()))
    return host


def _check(w, plan, st, host, state, lams, alpha, eta_l, K, tag, fused=False, n_threads=1):
    norms = st.norms.cpu().numpy().astype(np.float64)
    lam_gpu = st.lambda_dev.cpu().numpy()
    bf16 = w.precision == "bf16"

    def check_stage(j):
        tau = plan.stage_effective_staleness(j)
        d = host[j]
        window = d.versions[len(d.versions) - 1 - tau:]
        ref = O.compensate_stage_adaptive(window, d.grads, d.master, K, lams[j], np.float32(alpha), np.float32(eta_l),
                                          np.float32(w.lr), state[j][0], state[j][1], bf16=bf16,
                                          lambda_step_last=fused, n_threads=n_threads)
        t = f"{tag} stage {j}"
        assert lam_gpu[j] == pytest.approx(ref["lam"], rel=1e-5), t + " lambda"
        if tau == 0:
            assert lam_gpu[j] == np.float32(lams[j])
        got_r, got_a = st.get_flat(st.v_r, j).numpy(), st.get_flat(st.v_a, j).numpy()
        PU.assert_close_f32(got_r, ref["v_r"], t + " v_r")
        PU.assert_close_f32(got_a, ref["v_a"], t + " v_a")
        PU.assert_close_f32(st.get_flat(st.grad_out, j).numpy(), ref["g"], t + " g_K'")
        slot = plan.stage_write_slot(j)
        if bf16:
            got_m = st.get_flat(st.master, j).numpy()
            PU.assert_close_f32(got_m, ref["master"], t + " master")
            # lambda_j itself is only held to 1e-5 relative (above), and the correction g_K' - g_0 scales with it
            g0 = d.grads.float().numpy().astype(np.float64)
            slack = PU.master_slack(ref["master"], w.lr, np.maximum(np.abs(ref["g"]), np.abs(g0)), plan.stage_effective_iters(j),
                                    extra=abs(w.lr) * 2e-5 * np.abs(ref["g"].astype(np.float64) - g0))
            PU.assert_master_within_slack(got_m, ref["master"], slack, t + " master")
            bits = PU.bits_of(st.get_version(j, slot))
            PU.assert_bf16_within_one_ulp(bits, ref["new"], t + " version", abs_slack=slack)
            PU.assert_bf16_is_rounded_master(bits, got_m, t + " version vs own master")
        else:
            PU.assert_close_f32(st.get_version(j, slot).numpy(), ref["new"], t + " version")
        np.testing.assert_allclose(norms[j], ref["norms"], rtol=PU.RTOL, atol=1e-30, err_msg=t + " norms")
        return (got_r.copy(), got_a.copy()), float(lam_gpu[j])

    results = PU.map_stages(check_stage, w.n_stages, w.numel > PU.BIG)
    return [r[0] for r in results], [r[1] for r in results]


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("precision", ["f32", "bf16"])
@pytest.mark.parametrize("K", [-1, 2, 1])
def test_one_adaptive_step(precision, K, fused):
    w = W.custom_workload("adaptive", [[50_000, 24], [33_001], [20_000], [8_192]], [5, 3, 1, 0], 6, K,
                          precision=precision, seed=31, lam=0.4)
    plan, st, host = PU.load_workload(w, amplified=True)
    state = _state(w, st, 31, w.lam)
    alpha, eta_l = 0.9, 1e-3
    st.step_adaptive(alpha, eta_l, w.lr, fused=fused)
    torch.cuda.synchronize()
    _, lams = _check(w, plan, st, host, state, [w.lam] * 4, alpha, eta_l, K, f"K={K}", fused)
    assert abs(lams[0] - w.lam) > 1e-3           # lambda really moved
    assert lams[3] == np.float32(w.lam)          # the stage without staleness is left alone


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_fused_lambda_block_on_the_streamed_path(precision):
    """K' beyond the unrolled variants (9 and 12 iterations) and one stage in between, ragged sizes."""
    w = W.custom_workload("adaptive_deep", [[21_001], [9_000, 40], [5_000]], [12, 9, 6], 13, -1,
                          precision=precision, seed=35, lam=0.3)
    plan, st, host = PU.load_workload(w, amplified=True)
    state = _state(w, st, 35, w.lam)
    st.step_adaptive(0.8, 1e-3, w.lr, fused=True)
    torch.cuda.synchronize()
    _check(w, plan, st, host, state, [w.lam] * 3, 0.8, 1e-3, -1, "deep", True)


def test_fused_and_two_pass_agree_on_the_lambda_block():
    """Both orderings leave the same lambda and averages behind (bit for bit: same per-chunk sums in the same
    order) when they start from the same state; only the compensated gradient differs."""
    w = W.custom_workload("adaptive_both", [[30_000], [12_345]], [3, 2], 5, 2, seed=36, lam=0.25)
    results = []
    for fused in (False, True):
        plan, st, host = PU.load_workload(w, amplified=True)
        _state(w, st, 36, w.lam)
        st.step_adaptive(0.9, 1e-3, w.lr, fused=fused)
        torch.cuda.synchronize()
        results.append((st.lambda_dev.cpu().clone(), st.v_r.cpu().clone(), st.v_a.cpu().clone(),
                        st.grad_out.cpu().clone()))
    assert torch.equal(results[0][0], results[1][0])
    assert torch.equal(results[0][1], results[1][1]) and torch.equal(results[0][2], results[1][2])
    assert not torch.equal(results[0][3], results[1][3])


@pytest.mark.parametrize("fused", [False, True])
def test_adaptive_trajectory_over_several_steps(fused):
    tau = [2, 1, 0]
    w = W.custom_workload("adaptive_steps", [[30_000], [12_345], [4_096]], tau, 3, -1, seed=32, lam=0.2)
    plan, st, host = PU.load_workload(w, amplified=True)
    st.enable_adaptive(w.lam)                    # the paper's start: lambda = lambda0, v_r = v_a = 0
    state = [(np.zeros(n, np.float32), np.zeros(n, np.float32)) for n in w.stage_numel()]
    lams = [w.lam] * 3
    alpha, eta_l = 0.5, 2e-3
    for step in range(6):
        for j in range(3):
            g = W.draw_grads(w, j, w.stage_numel()[j], amplified=True, step=step)
            st.set_flat(st.grads, j, g)
            host[j].grads = g
        st.step_adaptive(alpha, eta_l, w.lr, fused=fused)
        torch.cuda.synchronize()
        state, lams = _check(w, plan, st, host, state, lams, alpha, eta_l, -1, f"step {step}", fused)
        # adopt the device's new version on the host side, then commit
        for j in range(3):
            new = st.get_version(j, plan.stage_write_slot(j))
            host[j].versions = host[j].versions[1:] + [new]
        st.commit()
    assert lams[0] != np.float32(w.lam) and lams[2] == np.float32(w.lam)


def test_zero_eta_lambda_is_the_fixed_lambda_step():
    w = W.custom_workload("adaptive_off", [[40_000], [10_000]], [3, 1], 5, -1, seed=33, lam=0.3)   # depth > tau+1: re-running a step is idempotent
    plan, st, host = PU.load_workload(w, amplified=True)
    st.step(w.lam, w.lr)
    torch.cuda.synchronize()
    want = [st.get_version(j, plan.stage_write_slot(j)) for j in range(2)]
    want_g = [st.get_flat(st.grad_out, j) for j in range(2)]
    state = _state(w, st, 33, w.lam)
    st.step_adaptive(0.9, 0.0, w.lr)
    torch.cuda.synchronize()
    for j in range(2):
        assert torch.equal(st.get_version(j, plan.stage_write_slot(j)), want[j])
        assert torch.equal(st.get_flat(st.grad_out, j), want_g[j])
        assert np.array_equal(st.get_flat(st.v_r, j).numpy(), state[j][0])
        assert np.array_equal(st.get_flat(st.v_a, j).numpy(), state[j][1])
    assert torch.equal(st.lambda_dev.cpu(), torch.full((2,), w.lam))


@pytest.mark.parametrize("fused", [False, True])
def test_adaptive_step_at_benchmark_shape(fused):
    """ViT-B-sized workload, the launch configurations bench.py --adaptive / --adaptive-fused time."""
    w = W.make_workload(4)
    plan, st, host = PU.load_workload(w, amplified=True)
    state = _state(w, st, 34, w.lam)
    st.step_adaptive(0.9, 1e-5, w.lr, fused=fused)
    torch.cuda.synchronize()
    _check(w, plan, st, host, state, [w.lam] * w.n_stages, 0.9, 1e-5, w.n_iters, "vit", fused)


@pytest.mark.parametrize("seed", range(40))
def test_random_adaptive_configurations(seed):
    """Random stages, ragged sizes, staleness, ring depth, iteration count, storage type, chunk size, moving-average
    and lambda rates, either ordering of the lambda block, random head positions."""
    rng = np.random.default_rng(3000 + seed)
    n_stages = int(rng.integers(1, 6))
    R = int(rng.integers(2, 12))
    tau = [int(rng.integers(0, R)) for _ in range(n_stages)]
    sizes = [[int(rng.choice([8, 9, 63, 500, 1024, 2047, 2049, 5000, 30_000]) * rng.integers(1, 4))
              for _ in range(int(rng.integers(1, 4)))] for _ in range(n_stages)]
    K = int(rng.choice([-1, 1, 2, 3, 5, 9]))
    precision = "bf16" if seed % 2 else "f32"
    fused = bool((seed // 2) % 2)
    chunk = int(rng.choice([0, 1024, 4096]))
    w = W.custom_workload(f"random_adaptive{seed}", sizes, tau, R, K, precision=precision, seed=4000 + seed,
                          lam=float(rng.choice([0.1, 0.5, -0.3])), lr=float(rng.choice([0.01, 0.2])))
    heads = [int(rng.integers(0, 16)) for _ in range(n_stages)]
    plan, st, host = PU.load_workload(w, amplified=True, chunk_elems=chunk, heads=heads)
    state = _state(w, st, 4000 + seed, w.lam)
    alpha, eta_l = float(rng.choice([0.0, 0.5, 0.9])), float(rng.choice([1e-5, 1e-3]))
    st.step_adaptive(alpha, eta_l, w.lr, fused=fused)
    torch.cuda.synchronize()
    _check(w, plan, st, host, state, [w.lam] * n_stages, alpha, eta_l, K, f"seed {seed} fused={fused}", fused)


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("active", [[1, 0, 1, 0], [0, 1, 0, 0], [0, 0, 0, 0]])
def test_adaptive_step_for_a_subset_of_stages(fused, active):
    """Stages that take part end up exactly as after the full self-tuned step; the others keep weights, lambda
    and averages."""
    w = W.custom_workload("adaptive_subset", [[30_000, 8], [12_345], [9_000], [4_096]], [3, 2, 1, 1], 4, 2, seed=37,
                          lam=0.3)
    plan, st, host = PU.load_workload(w, amplified=True)
    _state(w, st, 37, w.lam)
    st.step_adaptive(0.8, 1e-3, w.lr, fused=fused)
    torch.cuda.synchronize()
    full = dict(ring=st.ring.clone(), lam=st.lambda_dev.clone(), vr=st.v_r.clone(), va=st.v_a.clone(),
                norms=st.norms.clone(), g=st.grad_out.clone())
    plan2, st2, _ = PU.load_workload(w, amplified=True)
    _state(w, st2, 37, w.lam)
    before = dict(ring=st2.ring.clone(), lam=st2.lambda_dev.clone(), vr=st2.v_r.clone(), va=st2.v_a.clone())
    B.ferret_compensate_stages_adaptive(plan2, st2.ring, st2.grads, st2.master, active, st2.lambda_dev, st2.v_r, st2.v_a,
                                        0.8, 1e-3, w.lr, st2.norms, st2.grad_out, st2.workspace, fused=fused)
    torch.cuda.synchronize()
    for j in range(4):
        lo = plan2.stage_ring_offset(j)
        hi = lo + plan2.stage_slot_stride(j) * plan2.stage_ring_depth(j)
        f0, f1 = plan2.stage_flat_offset(j), plan2.stage_flat_offset(j) + plan2.stage_numel(j)
        ref = full if active[j] else before
        assert torch.equal(st2.ring[lo:hi], ref["ring"][lo:hi]), f"stage {j} ring"
        assert torch.equal(st2.lambda_dev[j], ref["lam"][j]), f"stage {j} lambda"
        assert torch.equal(st2.v_r[f0:f1], ref["vr"][f0:f1]) and torch.equal(st2.v_a[f0:f1], ref["va"][f0:f1])
        if active[j]:
            assert torch.equal(st2.norms[j], full["norms"][j]) and torch.equal(st2.grad_out[f0:f1], full["g"][f0:f1])
        else:
            assert not st2.norms[j].any()
