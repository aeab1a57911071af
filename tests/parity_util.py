"""Helpers shared by the GPU parity tests: run one step through the C ABI on the device and
the same step through the CPU oracle, and compare element by element.

Tolerances (written here once, used by every parity test):
  fp32 outputs (new version, g_K', master):  |gpu - ref| <= 1e-5 * |ref| + 1e-5 * rms(ref)
      The device computes in fp32 with fused multiply-adds (a few 1e-7 relative per
      iteration), the oracle in fp64 rounded once; the rms term only matters for elements
      that cancel to (almost) zero, where a relative bound has no meaning.
  bf16 outputs (new version):                bit-exact round-to-nearest-even of the device's own
      fp32 master, and at most 1 bf16 ulp from the oracle's value: both sides round their fp32
      master, so they differ only when the two masters straddle a rounding boundary.  The two
      masters themselves differ by the fp32 arithmetic of the update, bounded per element by
          d = 8 * 2^-24 * (|m'| + |eta| * (K'+1) * |step|)         (master_slack below)
      (oracle: fp64 rounded once, 2^-25 |m'|; device: one fused multiply-add m - eta*step, 2^-24 |m'|,
      on a step that went through K' iterations of three to four fp32 roundings each, i.e. at most
      about 4 (K'+1) 2^-24 |step|; the factor 8 leaves a margin of two).  An element whose update
      cancels to almost zero can sit many bf16 steps of its own tiny magnitude away and still be
      within d, so the bound is  |gpu - ref| <= ulp_bf16(ref) + d;  the device master is held to
      |gpu - ref| <= d as well.  Every check reports how many elements differ at all and how many
      needed d (were further than one bf16 ulp from the oracle).
  norms:                                     relative 1e-5 against the oracle's fp64 sums
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import ferret_oracle as O
from paper_2503_12053_amd import binding as B
from paper_2503_12053_amd import workloads as W

RTOL = 1e-5
BIG = 50_000_000          # workloads beyond this many parameters: stages are generated and checked on a few host threads


def map_stages(fn, n_stages, big):
    """[fn(j) for j in range(n_stages)]; for big workloads on four host threads (the generator, the oracle and
    numpy release the interpreter lock), in stage order either way."""
    if not big or n_stages == 1:
        return [fn(j) for j in range(n_stages)]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=4) as pool:
        return list(pool.map(fn, range(n_stages)))


def assert_close_f32(got, ref, what):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, what
    both_nan = np.isnan(got) & np.isnan(ref)
    same_inf = np.isinf(ref) & (got == ref)
    finite = np.isfinite(ref) & np.isfinite(got)
    assert np.all(both_nan | same_inf | finite), f"{what}: non-finite mismatch"
    if not finite.any():
        return 0.0
    rms = float(np.sqrt(np.mean(ref[finite] ** 2)))
    err = np.abs(got[finite] - ref[finite])
    bound = RTOL * np.abs(ref[finite]) + RTOL * rms
    worst = int(np.argmax(err - bound))
    assert np.all(err <= bound), (f"{what}: {int((err > bound).sum())} of {err.size} elements out of tolerance; "
                                  f"worst got {got[finite][worst]!r} ref {ref[finite][worst]!r}")
    den = np.maximum(np.abs(ref[finite]), rms)
    return float((err / np.where(den > 0, den, 1.0)).max())       # an all-zero reference has err = 0 as well


def bf16_ulp_distance(a_bits, b_bits):
    """Distance in representable bf16 steps between two arrays of bit patterns."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, 0x8000 - (x & 0x7FFF) - 1 + 0, 0x8000 + (x & 0x7FFF))
    return np.abs(key(np.asarray(a_bits, dtype=np.uint16)) - key(np.asarray(b_bits, dtype=np.uint16)))


def bf16_bits_to_f64(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


EPS32 = 2.0 ** -24
BF16_REPORT = []        # (what, elements, differing bit patterns, elements beyond one bf16 ulp): filled by every check


def master_slack(ref_master, lr, step_mag, kp, extra=0.0):
    """Per-element bound on |device fp32 master - oracle fp32 master| from the arithmetic of the update
    (module docstring).  step_mag: magnitude of what eta multiplies (the compensated gradient, or the scaled
    running sum); kp: iterations it went through; extra: further per-element terms a caller can justify."""
    m = np.abs(np.asarray(ref_master, dtype=np.float64))
    m = np.where(np.isfinite(m), m, 0.0)
    g = np.abs(np.asarray(step_mag, dtype=np.float64))
    g = np.where(np.isfinite(g), g, 0.0)
    return 8.0 * EPS32 * (m + abs(float(lr)) * (kp + 1) * g) + extra


def assert_master_within_slack(got_master, ref_master, slack, what):
    got = np.asarray(got_master, dtype=np.float64)
    ref = np.asarray(ref_master, dtype=np.float64)
    finite = np.isfinite(ref) & np.isfinite(got)
    err = np.abs(got - ref)[finite]
    lim = np.broadcast_to(slack, ref.shape)[finite]
    bad = err > lim
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {err.size} master elements beyond the derived fp32 bound; worst "
                           f"error {err[np.argmax(err - lim)]:.3g} against {lim[np.argmax(err - lim)]:.3g}")


def assert_bf16_within_one_ulp(got_bits, ref_bits, what, abs_slack=0.0):
    """|gpu - ref| <= one bf16 step at ref's magnitude + abs_slack (scalar or per element; see the module
    docstring).  Records and returns how many elements needed the slack."""
    got_bits = np.asarray(got_bits, dtype=np.uint16)
    ref_bits = np.asarray(ref_bits, dtype=np.uint16)
    def isnan(b):
        return ((b & 0x7F80) == 0x7F80) & ((b & 0x007F) != 0)
    nan_g, nan_r = isnan(got_bits), isnan(ref_bits)
    assert np.array_equal(nan_g, nan_r), f"{what}: NaN pattern differs"
    ok = ~nan_r
    got, ref = bf16_bits_to_f64(got_bits[ok]), bf16_bits_to_f64(ref_bits[ok])
    inf = np.isinf(ref)
    assert np.array_equal(got[inf], ref[inf]), f"{what}: infinities differ"
    got, ref = got[~inf], ref[~inf]
    assert np.all(np.isfinite(got)), f"{what}: device produced an infinity the oracle did not"
    # one bf16 step at |ref|: 2^(exponent - 7); subnormals and zero step by 2^-133
    expo = np.floor(np.log2(np.maximum(np.abs(ref), 2.0 ** -126)))
    ulp = 2.0 ** (expo - 7)
    err = np.abs(got - ref)
    slack = np.broadcast_to(np.asarray(abs_slack, dtype=np.float64), got_bits.shape)[ok][~inf]
    bad = err > ulp + slack
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {err.size} elements beyond 1 bf16 ulp + the derived slack; "
                           f"worst got {got[np.argmax(err - ulp - slack)]!r} ref {ref[np.argmax(err - ulp - slack)]!r} "
                           f"slack {slack[np.argmax(err - ulp - slack)]:.3g}")
    n_diff, n_beyond = int((got_bits != ref_bits).sum()), int((err > ulp).sum())
    BF16_REPORT.append((what, int(got_bits.size), n_diff, n_beyond))
    if got_bits.size >= 1_000_000 or n_beyond:
        print(f"  [bf16] {what}: {got_bits.size} elements, {n_diff} differ from the oracle, {n_beyond} by more than 1 bf16 ulp "
              f"(within the derived slack)", flush=True)
    return float(n_diff / got_bits.size) if got_bits.size else 0.0


def assert_bf16_is_rounded_master(got_bits, got_master, what):
    """Integer work: the stored bf16 version must be exactly RNE(bf16) of the device's fp32 master."""
    want = torch.from_numpy(np.ascontiguousarray(got_master)).to(torch.bfloat16)
    want_bits = bits_of(want)
    got_bits = np.asarray(got_bits, dtype=np.uint16)
    nan = np.isnan(got_master)
    assert np.array_equal(got_bits[~nan], want_bits[~nan]), f"{what}: stored bf16 is not RNE of the master"
    assert np.all((got_bits[nan] & 0x7F80) == 0x7F80) and np.all((got_bits[nan] & 0x7F) != 0), what


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def tensors_of(w: W.Workload):
    return [(n, s) for _, n, s in w.tensors]


def load_workload(w: W.Workload, amplified=False, chunk_elems=0, tuning=None, heads=None, n_iters=None,
                  ring_depth=None, device="cuda"):
    """Plan + device state with every ring slot valid, filled from the seeded generator.
    Returns (plan, state, host_data) where host_data[j] is the StageData kept for the oracle."""
    plan = B.plan_for_workload(w, chunk_elems=chunk_elems, tuning=tuning, n_iters=n_iters,
                               ring_depth=ring_depth)
    st = B.DeviceState(plan, tensors_of(w), device=device)
    host, hd, valid = [], [], []
    generated = map_stages(lambda j: W.generate_stage(w, j, amplified, n_versions=plan.stage_ring_depth(j)),
                           w.n_stages, w.numel > BIG)
    for j in range(w.n_stages):
        R = plan.stage_ring_depth(j)
        data = generated[j]
        h = st.load_versions(j, data.versions, None if heads is None else heads[j] % R)
        st.set_flat(st.grads, j, data.grads)
        if data.master is not None:
            st.set_flat(st.master, j, data.master)
        hd.append(h)
        valid.append(R)
        host.append(data)
        if w.numel > BIG:
            print(f"  loaded stage {j} of {w.name}", flush=True)
    plan.set_state(hd, valid)
    return plan, st, host


def oracle_stage(w: W.Workload, data: W.StageData, tau: int, K: int, lam=None, lr=None, n_threads=1):
    """Oracle result of one stage given its newest tau+1 versions."""
    lam = w.lam if lam is None else lam
    lr = w.lr if lr is None else lr
    window = data.versions[len(data.versions) - 1 - tau:]
    if w.precision == "f32":
        new, g_out, norms = O.compensate_stage_f32(window, data.grads, K, np.float32(lam), np.float32(lr),
                                                   n_threads=n_threads)
        return dict(new=new, g=g_out, norms=norms)
    new, m_new, g_out, norms = O.compensate_stage_bf16(window, data.grads, data.master, K, np.float32(lam),
                                                       np.float32(lr), n_threads=n_threads)
    return dict(new=new, master=m_new, g=g_out, norms=norms)


def check_step_against_oracle(w, plan, st, host, K=None, lam=None, lr=None, n_threads=1, label=""):
    """After st.step(...) + synchronize: compare every stage with the oracle.  Returns stats."""
    K = w.n_iters if K is None else K
    norms = st.norms.cpu().numpy().astype(np.float64)
    stats = {}

    def check_stage(j):
        tau = plan.stage_effective_staleness(j)
        ref = oracle_stage(w, host[j], tau, K, lam, lr, n_threads)
        slot = plan.stage_write_slot(j)
        tag = f"{label}{w.name} stage {j}"
        got_g = st.get_flat(st.grad_out, j).numpy()
        stats[f"g{j}"] = assert_close_f32(got_g, ref["g"], tag + " g_K'")
        if w.precision == "f32":
            got_new = st.get_version(j, slot).numpy()
            stats[f"w{j}"] = assert_close_f32(got_new, ref["new"], tag + " new version")
        else:
            got_new = bits_of(st.get_version(j, slot))
            got_m = st.get_flat(st.master, j).numpy()
            stats[f"m{j}"] = assert_close_f32(got_m, ref["master"], tag + " master")
            slack = master_slack(ref["master"], w.lr if lr is None else lr, np.maximum(np.abs(ref["g"]), np.abs(host[j].grads.float().numpy())),
                                 plan.stage_effective_iters(j))
            assert_master_within_slack(got_m, ref["master"], slack, tag + " master")
            stats[f"w{j}"] = assert_bf16_within_one_ulp(got_new, ref["new"], tag + " new version (bf16)",
                                                        abs_slack=slack)
            assert_bf16_is_rounded_master(got_new, got_m, tag + " new version vs own master")
        np.testing.assert_allclose(norms[j], ref["norms"], rtol=RTOL, atol=1e-30, err_msg=tag + " norms")
        if w.numel > BIG:
            print(f"  checked stage {j} of {w.name}", flush=True)

    map_stages(check_stage, w.n_stages, w.numel > BIG)
    return stats
