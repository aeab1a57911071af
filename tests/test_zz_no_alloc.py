"""GPU test of ferret_compensate_step_noalloc, the entry point for callers that cannot allocate: its
outputs (new version, master, compensated gradient, norms) must equal those of ferret_compensate_step on the
same inputs.  Both run the same kernels, so the comparison is bit for bit, which is within every tolerance of
tests/parity_util.py; the first case is also compared with the CPU oracle.  Two calls in a row share the
library's one scratch array, the second with a smaller input, so stale partial sums of the first call lie
behind the second call's.

Collected last (file name) so that a failure here cannot hide another test's result under `pytest -x`.
"""
import numpy as np
import pytest
import torch

from paper_2503_12053_amd import binding as B
from paper_2503_12053_amd import workloads as W

import parity_util as PU

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m 'not gpu' elsewhere)")
    B.load()


def _pair(w, **kw):
    """Two device states with identical contents: one for each entry point."""
    plan_a, st_a, host = PU.load_workload(w, amplified=True, **kw)
    plan_b, st_b, _ = PU.load_workload(w, amplified=True, **kw)
    return (plan_a, st_a), (plan_b, st_b), host


def _step_both(w, a, b):
    (plan_a, st_a), (plan_b, st_b) = a, b
    st_a.step(w.lam, w.lr)                                                     # caller's workspace
    B.ferret_compensate_step_noalloc(plan_b, st_b.ring, st_b.grads, st_b.master, w.lam, w.lr,
                                     st_b.norms, st_b.grad_out)               # library's own scratch
    torch.cuda.synchronize()
    assert torch.equal(st_a.ring, st_b.ring), "ring differs"
    assert torch.equal(st_a.grad_out, st_b.grad_out), "compensated gradient differs"
    assert torch.equal(st_a.norms, st_b.norms), "norms differ"
    if st_a.master is not None:
        assert torch.equal(st_a.master, st_b.master), "master differs"
    assert float(st_b.norms[0, 0]) > 0.0


@pytest.mark.parametrize("precision", ["f32", "bf16"])
def test_noalloc_matches_step_on_two_calls_the_second_smaller(precision):
    big = W.custom_workload("noalloc_big", [[300_000, 17, 40_001], [123_457], [9_000]], [3, 1, 0], 4, 2,
                            precision=precision, seed=71)
    small = W.custom_workload("noalloc_small", [[20_000, 5], [3_001]], [2, 1], 3, -1, precision=precision, seed=72)
    for w in (big, small):
        print(f"[case] {w.name} {precision}", flush=True)
        a, b, host = _pair(w)
        _step_both(w, a, b)
        PU.check_step_against_oracle(w, b[0], b[1], host, label="noalloc ")
        # a committed second step on the same plans: the scratch holds the first step's partial sums
        for plan, st in (a, b):
            st.commit()
        _step_both(w, a, b)


def test_noalloc_without_norms_and_on_a_side_stream():
    w = W.custom_workload("noalloc_stream", [[150_000], [50_000]], [1, 0], 2, 1, seed=73)
    a, b, host = _pair(w)
    (plan_a, st_a), (plan_b, st_b) = a, b
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    st_a.step(w.lam, w.lr, norms=False, stream=s)
    B.ferret_compensate_step_noalloc(plan_b, st_b.ring, st_b.grads, None, w.lam, w.lr, None, st_b.grad_out, s)
    s.synchronize()
    assert torch.equal(st_a.ring, st_b.ring) and torch.equal(st_a.grad_out, st_b.grad_out)
    st_b.commit()
    with pytest.raises(B.FerretError) as e:       # nothing to commit twice: same protocol as the plain step
        st_b.commit()
    assert e.value.status == B.FERRET_ESTATE
