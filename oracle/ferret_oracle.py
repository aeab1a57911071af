"""Python face of the CPU oracle (oracle/ferret_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
It compiles the C file with gcc on first use and calls it through ctypes.  Nothing here
touches the HIP library or shares code with it.

The oracle works on one pipeline stage at a time, on the plain problem statement of
Alg. 1 (paper, appendix "Algorithm Details"): the stale gradient, the tau+1 stored
versions oldest first, lambda, eta.  `OracleRing` adds the bookkeeping of a version store
across several optimisation steps (Sec. "Fine-grained Pipeline Parallelism", T2: a stage
keeps a bounded number of versions) so that multi-step behaviour can be checked.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ferret_oracle.c")
_LIB = os.path.join(_HERE, "libferret_oracle.so")
_lib = None

ITERS_FULL = -1


def build(force: bool = False) -> str:
    """Compile the oracle (gcc, -O2, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        override = os.environ.get("FERRET_ORACLE_LIB")      # tests of the pins load a deliberately broken build
        if override:
            lib = ctypes.CDLL(override)
        else:
            build()
            lib = ctypes.CDLL(_LIB)
        pp = ctypes.POINTER(ctypes.c_void_p)
        lib.ferret_oracle_effective_iters.restype = ctypes.c_int32
        lib.ferret_oracle_effective_iters.argtypes = [ctypes.c_int32, ctypes.c_int32]
        lib.ferret_oracle_segment_boundary.restype = ctypes.c_int32
        lib.ferret_oracle_segment_boundary.argtypes = [ctypes.c_int32] * 3
        lib.ferret_oracle_bf16_to_f32.restype = ctypes.c_float
        lib.ferret_oracle_bf16_to_f32.argtypes = [ctypes.c_uint16]
        lib.ferret_oracle_f32_to_bf16.restype = ctypes.c_uint16
        lib.ferret_oracle_f32_to_bf16.argtypes = [ctypes.c_float]
        lib.ferret_oracle_stage_f32.restype = ctypes.c_int
        lib.ferret_oracle_stage_f32.argtypes = [
            ctypes.c_int64, ctypes.c_int32, pp, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_int32]
        lib.ferret_oracle_stage_bf16.restype = ctypes.c_int
        lib.ferret_oracle_stage_bf16.argtypes = [
            ctypes.c_int64, ctypes.c_int32, pp, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int32, ctypes.c_double, ctypes.c_double, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32]
        lib.ferret_oracle_lambda_update.restype = ctypes.c_double
        lib.ferret_oracle_lambda_update.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.ferret_oracle_accumulate.restype = ctypes.c_int
        lib.ferret_oracle_accumulate.argtypes = [
            ctypes.c_int64, ctypes.c_int32, pp, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
            ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.ferret_oracle_penalized.restype = ctypes.c_int
        lib.ferret_oracle_penalized.argtypes = [
            ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
            ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


# ---- small scalar helpers ---------------------------------------------------------------
def effective_iters(K: int, tau: int) -> int:
    return int(_load().ferret_oracle_effective_iters(K, tau))


def segment_boundaries(tau: int, K: int) -> List[int]:
    """[s_0 .. s_K'] for staleness tau and iteration count K (empty loop -> [0] or [tau])."""
    Kp = effective_iters(K, tau)
    if Kp == 0:
        return [tau]
    return [int(_load().ferret_oracle_segment_boundary(i, tau, Kp)) for i in range(Kp + 1)]


def bf16_bits_to_f32(bits: int) -> float:
    return float(_load().ferret_oracle_bf16_to_f32(bits))


def f32_to_bf16_bits(x: float) -> int:
    return int(_load().ferret_oracle_f32_to_bf16(np.float32(x)))


# ---- array plumbing ---------------------------------------------------------------------
def _as_np(a, dtype) -> np.ndarray:
    """torch tensor / numpy array -> contiguous numpy array of `dtype` (no value change)."""
    if hasattr(a, "detach"):               # torch tensor
        import torch
        t = a.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            t = t.view(torch.int16)
        a = t.numpy()
    a = np.ascontiguousarray(a)
    if dtype == np.uint16 and a.dtype == np.int16:
        a = a.view(np.uint16)
    if a.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {a.dtype}")
    return a


def _ptr_array(arrs: Sequence[np.ndarray]):
    P = (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
    return P


def compensate_stage_f32(versions, g0, K: int, lam: float, eta: float, n_threads: int = 1,
                         want_g: bool = True):
    """One stage, fp32 storage.  versions: tau+1 arrays oldest first.
    Returns (theta_new float32[n], g_K' float64[n] or None, norms float64[3])."""
    V = [_as_np(v, np.float32) for v in versions]
    g = _as_np(g0, np.float32)
    n = g.size
    for v in V:
        if v.size != n:
            raise ValueError("version/gradient size mismatch")
    out = np.empty(n, np.float32)
    g_out = np.empty(n, np.float64) if want_g else None
    norms = np.zeros(3, np.float64)
    rc = _load().ferret_oracle_stage_f32(
        n, len(V), _ptr_array(V), g.ctypes.data, K, float(lam), float(eta), out.ctypes.data,
        g_out.ctypes.data if want_g else None, norms.ctypes.data, n_threads)
    if rc != 0:
        raise ValueError("ferret_oracle_stage_f32: bad arguments")
    return out, g_out, norms


def compensate_stage_bf16(versions, g0, master, K: int, lam: float, eta: float,
                          n_threads: int = 1, want_g: bool = True):
    """One stage, bf16 versions/gradient (uint16 bit patterns or torch.bfloat16) + fp32 master.
    Returns (theta_new uint16[n], master_new float32[n], g_K' float64[n] or None, norms)."""
    V = [_as_np(v, np.uint16) for v in versions]
    g = _as_np(g0, np.uint16)
    m = _as_np(master, np.float32)
    n = g.size
    for v in V + [m]:
        if v.size != n:
            raise ValueError("size mismatch")
    out = np.empty(n, np.uint16)
    m_out = np.empty(n, np.float32)
    g_out = np.empty(n, np.float64) if want_g else None
    norms = np.zeros(3, np.float64)
    rc = _load().ferret_oracle_stage_bf16(
        n, len(V), _ptr_array(V), g.ctypes.data, m.ctypes.data, K, float(lam), float(eta),
        out.ctypes.data, m_out.ctypes.data, g_out.ctypes.data if want_g else None,
        norms.ctypes.data, n_threads)
    if rc != 0:
        raise ValueError("ferret_oracle_stage_bf16: bad arguments")
    return out, m_out, g_out, norms


# ---- adaptive lambda (Alg. 1 with eta_lambda > 0) ------------------------------------------
def lambda_update(g0, V0, V1, lam: float, alpha: float, eta_lambda: float, v_r, v_a, bf16: bool = False):
    """The "update lambda" block of Alg. 1 on one stage.  Returns (lambda_new, v_r_new, v_a_new, sums)
    with sums = (<v_a, dv_r>, <v_a, v_a>) taken on the state before the call."""
    dt = np.uint16 if bf16 else np.float32
    g, a0, a1 = _as_np(g0, dt), _as_np(V0, dt), _as_np(V1, dt)
    r, a = _as_np(v_r, np.float32), _as_np(v_a, np.float32)
    n = g.size
    if not (a0.size == a1.size == r.size == a.size == n):
        raise ValueError("size mismatch")
    r_new, a_new = np.empty(n, np.float32), np.empty(n, np.float32)
    sums = np.zeros(2, np.float64)
    lam_new = _load().ferret_oracle_lambda_update(
        n, g.ctypes.data, a0.ctypes.data, a1.ctypes.data, int(bf16), float(lam), float(alpha),
        float(eta_lambda), r.ctypes.data, a.ctypes.data, r_new.ctypes.data, a_new.ctypes.data,
        sums.ctypes.data)
    return float(lam_new), r_new, a_new, sums


def compensate_stage_adaptive(versions, g0, master, K: int, lam: float, alpha: float, eta_lambda: float,
                              eta: float, v_r, v_a, bf16: bool = False, n_threads: int = 1,
                              lambda_step_last: bool = False):
    """All of Alg. 1 for one stage: lambda block (skipped when eta_lambda = 0 or tau = 0), then the
    iterations with the NEW lambda, then the update.  Returns a dict.

    lambda_step_last = True is the one-pass ordering the library offers beside Alg. 1's: the same lambda
    block on the same inputs, but the iterations of this call still use the lambda passed in, so that each
    lambda step takes effect one call later."""
    tau = len(versions) - 1
    if eta_lambda > 0 and tau >= 1:
        lam_new, r_new, a_new, sums = lambda_update(g0, versions[0], versions[1], lam, alpha, eta_lambda,
                                                    v_r, v_a, bf16)
    else:
        lam_new, sums = float(lam), np.zeros(2)
        r_new, a_new = _as_np(v_r, np.float32).copy(), _as_np(v_a, np.float32).copy()
    out = dict(lam=lam_new, v_r=r_new, v_a=a_new, sums=sums)
    lam_used = float(lam) if lambda_step_last else lam_new
    if bf16:
        new, m_new, g_out, norms = compensate_stage_bf16(versions, g0, master, K, lam_used, eta, n_threads)
        out.update(new=new, master=m_new, g=g_out, norms=norms)
    else:
        new, g_out, norms = compensate_stage_f32(versions, g0, K, lam_used, eta, n_threads)
        out.update(new=new, g=g_out, norms=norms)
    return out


# ---- gradient accumulation (T2) --------------------------------------------------------------
def accumulate_stage(versions, g0, master, K: int, lam: float, eta: float, scale: float, do_update: bool,
                     accum, bf16: bool = False):
    """Compensate one arriving gradient to the current version, add it to the running sum and, when
    do_update, apply theta_next = V[tau] - eta*scale*sum and clear the sum.
    Returns dict(accum=float32[n], g=float64[n], new=..., master=...) (new/master only when do_update)."""
    dt = np.uint16 if bf16 else np.float32
    V = [_as_np(v, dt) for v in versions]
    g = _as_np(g0, dt)
    acc = _as_np(accum, np.float32)
    n = g.size
    m = _as_np(master, np.float32) if bf16 else None
    acc_out = np.empty(n, np.float32)
    g_out = np.empty(n, np.float64)
    new = np.zeros(n, dt)
    m_new = np.zeros(n, np.float32) if bf16 else None
    rc = _load().ferret_oracle_accumulate(
        n, len(V), _ptr_array(V), g.ctypes.data, int(bf16), m.ctypes.data if bf16 else None, K, float(lam),
        float(eta), float(scale), int(bool(do_update)), acc.ctypes.data, acc_out.ctypes.data, new.ctypes.data,
        m_new.ctypes.data if bf16 else None, g_out.ctypes.data)
    if rc != 0:
        raise ValueError("ferret_oracle_accumulate: bad arguments")
    out = dict(accum=acc_out, g=g_out)
    if do_update:
        out["new"] = new
        if bf16:
            out["master"] = m_new
    return out


def accumulate_stage_adaptive(versions, g0, master, K: int, lam: float, alpha: float, eta_lambda: float, eta: float,
                              scale: float, do_update: bool, accum, v_r, v_a, bf16: bool = False,
                              lambda_step_last: bool = False):
    """One arriving gradient under accumulation with self-tuned lambda: Alg. 1 runs per gradient, so the
    lambda block comes first (on the version this gradient was taken on and the one after it; skipped when
    eta_lambda = 0 or the arrival has no staleness), then accumulate_stage with the new lambda
    (lambda_step_last: with the lambda that was passed in, as in compensate_stage_adaptive)."""
    tau = len(versions) - 1
    if eta_lambda > 0 and tau >= 1:
        lam_new, r_new, a_new, _ = lambda_update(g0, versions[0], versions[1], lam, alpha, eta_lambda, v_r, v_a, bf16)
    else:
        lam_new = float(lam)
        r_new, a_new = _as_np(v_r, np.float32).copy(), _as_np(v_a, np.float32).copy()
    lam_used = float(lam) if lambda_step_last else lam_new
    out = accumulate_stage(versions, g0, master, K, lam_used, eta, scale, do_update, accum, bf16)
    out.update(lam=lam_new, v_r=r_new, v_a=a_new)
    return out


# ---- step-size-penalising comparison methods ------------------------------------------------
def penalized_stage(V0, Vtau, g0, master, eta: float, scale: float, inv_c: float, bf16: bool = False):
    """theta_next = V[tau] - eta*scale*g0 / (|V[tau]-V[0]|*inv_c + 1).  Returns dict(new, g[, master])."""
    dt = np.uint16 if bf16 else np.float32
    a0, a1, g = _as_np(V0, dt), _as_np(Vtau, dt), _as_np(g0, dt)
    n = g.size
    m = _as_np(master, np.float32) if bf16 else None
    new = np.zeros(n, dt)
    m_new = np.zeros(n, np.float32) if bf16 else None
    g_out = np.empty(n, np.float64)
    rc = _load().ferret_oracle_penalized(n, a0.ctypes.data, a1.ctypes.data, g.ctypes.data, int(bf16),
                                         m.ctypes.data if bf16 else None, float(eta), float(scale), float(inv_c),
                                         new.ctypes.data, m_new.ctypes.data if bf16 else None, g_out.ctypes.data)
    if rc != 0:
        raise ValueError("ferret_oracle_penalized: bad arguments")
    out = dict(new=new, g=g_out)
    if bf16:
        out["master"] = m_new
    return out


# ---- version store across steps ---------------------------------------------------------
class OracleRing:
    """Per-stage store of the last R weight versions, plain Python lists.

    step(j, g) applies Alg. 1 to stage j with effective staleness
    min(tau_j, versions_held - 1) (during warm-up fewer than tau_j + 1 versions exist),
    appends the new version and drops the oldest beyond R.
    """

    def __init__(self, staleness: Sequence[int], ring_depth: int, K: int, precision: str = "f32"):
        self.tau = list(staleness)
        self.R = int(ring_depth)
        self.K = int(K)
        self.precision = precision
        self.versions: List[List[np.ndarray]] = [[] for _ in self.tau]
        self.master: List[Optional[np.ndarray]] = [None for _ in self.tau]

    def push(self, j: int, version, master=None) -> None:
        dt = np.float32 if self.precision == "f32" else np.uint16
        self.versions[j].append(_as_np(version, dt).copy())
        if len(self.versions[j]) > self.R:
            self.versions[j].pop(0)
        if master is not None:
            self.master[j] = _as_np(master, np.float32).copy()

    def effective_tau(self, j: int) -> int:
        return min(self.tau[j], len(self.versions[j]) - 1)

    def step(self, j: int, g, lam: float, eta: float):
        held = self.versions[j]
        if not held:
            raise RuntimeError("stage has no version yet")
        tau = self.effective_tau(j)
        window = held[len(held) - 1 - tau:]
        if self.precision == "f32":
            new, g_out, norms = compensate_stage_f32(window, g, self.K, lam, eta)
            self.push(j, new)
        else:
            new, m_new, g_out, norms = compensate_stage_bf16(window, g, self.master[j], self.K,
                                                              lam, eta)
            self.push(j, new, m_new)
        return new, g_out, norms
