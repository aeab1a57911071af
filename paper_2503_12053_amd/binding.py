"""ctypes binding of libferret.so -- same names as include/ferret.h, argument marshalling only.

`load()` returns the library handle and raises RuntimeError if it has not been built: there is
no fallback path.  torch is imported first so that libferret resolves the same HIP runtime
that owns torch's device memory and streams.

Besides the raw functions (`ferret_plan_buckets`, `ferret_push_version`,
`ferret_compensate_step`, the plan queries) this module has `DeviceState`, a small holder of
the device buffers a plan needs (ring, gradients, master, workspace) that tests and the
benchmark use to move workload data in and results out.  It does no arithmetic.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, byref, c_char_p, c_float, c_int32, c_int64, c_size_t, c_void_p
from typing import List, Optional, Sequence

import torch  # noqa: F401  (must precede loading libferret: fixes which libamdhip64 is used)

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libferret.so")

FERRET_OK, FERRET_EINVAL, FERRET_ESTATE, FERRET_ENOMEM, FERRET_EDEVICE = range(5)
FERRET_F32, FERRET_BF16_MASTER_F32 = 0, 1
FERRET_ITERS_FULL = -1
FERRET_RING_DEPTH_MINIMAL = 0
FERRET_MAX_STAGES = 64
FERRET_ALIGN_ELEMS = 8
FERRET_NOALLOC_MAX_CHUNKS = 262144

STATUS_NAMES = {0: "FERRET_OK", 1: "FERRET_EINVAL", 2: "FERRET_ESTATE", 3: "FERRET_ENOMEM",
                4: "FERRET_EDEVICE"}


class ferret_tensor(ctypes.Structure):
    _fields_ = [("numel", c_int64), ("stage", c_int32), ("reserved", c_int32)]


class ferret_tuning(ctypes.Structure):
    _fields_ = [("slot_align_elems", c_int64), ("slot_skew_elems", c_int64), ("chunk_bytes", c_int64),
                ("blocks_per_cu", c_int32), ("resident_cap", c_int32), ("newest_from_master", c_int32),
                ("cache_policy", c_int32), ("xcd_group", c_int32), ("reserved", c_int32)]


class ferret_adaptive(ctypes.Structure):
    _fields_ = [("lambda_", c_void_p), ("v_r", c_void_p), ("v_a", c_void_p), ("alpha", c_float),
                ("eta_lambda", c_float), ("fused", c_int32), ("reserved", c_int32)]


class ferret_accumulate(ctypes.Structure):
    _fields_ = [("accum", c_void_p), ("scale", c_float), ("mode", POINTER(c_int32)),
                ("staleness", POINTER(c_int32))]


class ferret_layer(ctypes.Structure):
    _fields_ = [("t_f", ctypes.c_double), ("t_b", ctypes.c_double), ("n_params", ctypes.c_double),
                ("n_acts", ctypes.c_double)]


class FerretError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


# every symbol include/ferret.h declares: name -> (restype, argtypes)
_P = c_void_p
SIGNATURES = {
    "ferret_plan_buckets": (c_int32, [POINTER(ferret_tensor), c_int32, c_int32, POINTER(c_int32), c_int32,
                                      c_int32, c_int32, c_int64, POINTER(_P)]),
    "ferret_plan_buckets_tuned": (c_int32, [POINTER(ferret_tensor), c_int32, c_int32, POINTER(c_int32),
                                            c_int32, c_int32, c_int32, c_int64, POINTER(ferret_tuning),
                                            POINTER(_P)]),
    "ferret_plan_destroy": (None, [_P]),
    "ferret_plan_n_stages": (c_int32, [_P]),
    "ferret_plan_n_tensors": (c_int32, [_P]),
    "ferret_plan_precision": (c_int32, [_P]),
    "ferret_plan_n_iters": (c_int32, [_P]),
    "ferret_plan_chunk_elems": (c_int64, [_P]),
    "ferret_plan_n_chunks": (c_int64, [_P]),
    "ferret_plan_flat_elems": (c_int64, [_P]),
    "ferret_plan_ring_elems": (c_int64, [_P]),
    "ferret_plan_ring_bytes": (c_size_t, [_P]),
    "ferret_plan_grad_bytes": (c_size_t, [_P]),
    "ferret_plan_master_bytes": (c_size_t, [_P]),
    "ferret_plan_workspace_bytes": (c_size_t, [_P]),
    "ferret_plan_total_params": (c_int64, [_P]),
    "ferret_plan_stage_params": (c_int64, [_P, c_int32]),
    "ferret_plan_stage_numel": (c_int64, [_P, c_int32]),
    "ferret_plan_stage_flat_offset": (c_int64, [_P, c_int32]),
    "ferret_plan_stage_ring_offset": (c_int64, [_P, c_int32]),
    "ferret_plan_stage_slot_stride": (c_int64, [_P, c_int32]),
    "ferret_plan_stage_ring_depth": (c_int32, [_P, c_int32]),
    "ferret_plan_stage_staleness": (c_int32, [_P, c_int32]),
    "ferret_plan_stage_chunk_elems": (c_int64, [_P, c_int32]),
    "ferret_plan_stage_n_chunks": (c_int64, [_P, c_int32]),
    "ferret_plan_tensor_offset": (c_int64, [_P, c_int32]),
    "ferret_plan_get_state": (c_int32, [_P, POINTER(c_int32), POINTER(c_int32)]),
    "ferret_plan_set_state": (c_int32, [_P, POINTER(c_int32), POINTER(c_int32)]),
    "ferret_plan_stage_effective_staleness": (c_int32, [_P, c_int32]),
    "ferret_plan_stage_effective_iters": (c_int32, [_P, c_int32]),
    "ferret_plan_stage_read_slots": (c_int32, [_P, c_int32, POINTER(c_int32), c_int32]),
    "ferret_plan_stage_write_slot": (c_int32, [_P, c_int32]),
    "ferret_plan_step_bytes": (c_int64, [_P]),
    "ferret_push_version": (c_int32, [_P, _P, _P, c_int32, _P, _P]),
    "ferret_compensate_step": (c_int32, [_P, _P, _P, _P, c_float, c_float, _P, _P, _P, _P]),
    "ferret_compensate_step_noalloc": (c_int32, [_P, _P, _P, _P, c_float, c_float, _P, _P, _P]),
    "ferret_compensate_step_adaptive": (c_int32, [_P, _P, _P, _P, POINTER(ferret_adaptive), c_float, _P, _P, _P, _P]),
    "ferret_compensate_stages_adaptive": (c_int32, [_P, _P, _P, _P, POINTER(c_int32), POINTER(ferret_adaptive), c_float,
                                                    _P, _P, _P, _P]),
    "ferret_compensate_stages": (c_int32, [_P, _P, _P, _P, POINTER(c_int32), c_float, c_float, _P, _P, _P, _P]),
    "ferret_accumulate_step": (c_int32, [_P, _P, _P, _P, POINTER(ferret_accumulate), c_float, c_float, _P, _P, _P, _P]),
    "ferret_accumulate_step_adaptive": (c_int32, [_P, _P, _P, _P, POINTER(ferret_accumulate), POINTER(ferret_adaptive),
                                                  c_float, _P, _P, _P, _P]),
    "ferret_pipeline_evaluate": (c_int32, [POINTER(ferret_layer), c_int32, POINTER(c_int32), c_int32, c_int32,
                                           POINTER(c_int32), POINTER(c_int32), POINTER(c_int32), POINTER(c_int32),
                                           ctypes.c_double, ctypes.c_double, POINTER(ctypes.c_double),
                                           POINTER(ctypes.c_double)]),
    "ferret_pipeline_search": (c_int32, [POINTER(ferret_layer), c_int32, POINTER(c_int32), c_int32, ctypes.c_double,
                                         ctypes.c_double, ctypes.c_double, ctypes.c_double, POINTER(_P)]),
    "ferret_pipeline_plan": (c_int32, [POINTER(ferret_layer), c_int32, ctypes.c_double, ctypes.c_double,
                                       ctypes.c_double, ctypes.c_double, POINTER(_P)]),
    "ferret_pipeline_destroy": (None, [_P]),
    "ferret_pipeline_feasible": (c_int32, [_P]),
    "ferret_pipeline_n_stages": (c_int32, [_P]),
    "ferret_pipeline_n_workers": (c_int32, [_P]),
    "ferret_pipeline_stage_begin": (c_int32, [_P, c_int32]),
    "ferret_pipeline_rate": (ctypes.c_double, [_P]),
    "ferret_pipeline_memory": (ctypes.c_double, [_P]),
    "ferret_pipeline_stage_bound": (ctypes.c_double, [_P]),
    "ferret_pipeline_worker_delay": (c_int32, [_P, c_int32]),
    "ferret_pipeline_worker_recompute": (c_int32, [_P, c_int32]),
    "ferret_pipeline_worker_accum": (c_int32, [_P, c_int32, c_int32]),
    "ferret_pipeline_worker_omit": (c_int32, [_P, c_int32, c_int32]),
    "ferret_pipeline_stage_versions": (c_int32, [_P, c_int32, c_int32]),
    "ferret_pipeline_n_moves": (c_int32, [_P]),
    "ferret_pipeline_move": (c_int32, [_P, c_int32, POINTER(c_int32), POINTER(c_int32), POINTER(c_int32)]),
    "ferret_penalized_step": (c_int32, [_P, _P, _P, _P, POINTER(c_float), POINTER(c_float), c_float, _P, _P, _P, _P]),
    "ferret_last_error": (c_char_p, []),
    "ferret_version": (c_char_p, []),
    "ferret_copy_bytes": (c_int32, [_P, _P, c_size_t, _P]),
    "ferret_stream_mix": (c_int32, [_P, _P, c_size_t, c_int32, c_size_t, c_int32, _P]),
    "ferret_read_bytes": (c_int32, [_P, c_size_t, _P, _P]),
    "ferret_profile_begin": (c_int32, [c_int32]),
    "ferret_profile_end": (c_int32, [POINTER(c_float), c_int32, POINTER(c_int32)]),
}

_lib = None


def load():
    """Load libferret.so (built by paper_2503_12053_amd.build); raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_12053_amd.build` "
                               "(there is no fallback implementation)")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)      # AttributeError if the library does not export it
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def last_error() -> str:
    return load().ferret_last_error().decode()


def _check(status: int) -> None:
    if status != FERRET_OK:
        raise FerretError(status, last_error())


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor, an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- the three entry points, named as in the header ---------------------------------------------
def ferret_plan_buckets(tensors: Sequence, n_stages: int, staleness: Sequence[int], n_iters: int,
                        ring_depth: int, prec: int = FERRET_F32, chunk_elems: int = 0,
                        tuning: Optional[dict] = None) -> "Plan":
    """tensors: sequence of (numel, stage).  Returns a Plan (owns the C plan)."""
    lib = load()
    arr = (ferret_tensor * max(len(tensors), 1))()
    for i, (numel, stage) in enumerate(tensors):
        arr[i].numel, arr[i].stage, arr[i].reserved = int(numel), int(stage), 0
    st = (c_int32 * max(len(staleness), 1))(*[int(x) for x in staleness])
    out = _P()
    if tuning is None:
        rc = lib.ferret_plan_buckets(arr, len(tensors), n_stages, st, n_iters, ring_depth, prec,
                                     chunk_elems, byref(out))
    else:
        unknown = set(tuning) - {n for n, _ in ferret_tuning._fields_}
        if unknown:
            raise ValueError(f"unknown tuning fields {sorted(unknown)}")
        tn = ferret_tuning(int(tuning.get("slot_align_elems", 0)), int(tuning.get("slot_skew_elems", 0)),
                           int(tuning.get("chunk_bytes", 0)),
                           int(tuning.get("blocks_per_cu", 0)), int(tuning.get("resident_cap", 0)),
                           int(tuning.get("newest_from_master", 0)), int(tuning.get("cache_policy", 0)),
                           int(tuning.get("xcd_group", 0)), int(tuning.get("reserved", 0)))
        rc = lib.ferret_plan_buckets_tuned(arr, len(tensors), n_stages, st, n_iters, ring_depth, prec,
                                           chunk_elems, byref(tn), byref(out))
    _check(rc)
    return Plan(out)


def ferret_push_version(plan: "Plan", ring, master, stage: int, src, stream=None) -> None:
    _check(load().ferret_push_version(plan.handle, _ptr(ring), _ptr(master), stage, _ptr(src),
                                      _stream(stream)))


def ferret_compensate_step(plan: "Plan", ring, grads, master, lam: float, lr: float, norms_out=None,
                           grad_out=None, workspace=None, stream=None) -> None:
    _check(load().ferret_compensate_step(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), lam, lr,
                                         _ptr(norms_out), _ptr(grad_out), _ptr(workspace),
                                         _stream(stream)))


def ferret_compensate_step_noalloc(plan: "Plan", ring, grads, master, lam: float, lr: float, norms_out=None,
                                   grad_out=None, stream=None) -> None:
    _check(load().ferret_compensate_step_noalloc(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), lam, lr,
                                                 _ptr(norms_out), _ptr(grad_out), _stream(stream)))


def ferret_compensate_step_adaptive(plan: "Plan", ring, grads, master, lambda_dev, v_r, v_a, alpha: float,
                                    eta_lambda: float, lr: float, norms_out=None, grad_out=None,
                                    workspace=None, stream=None, fused: bool = False) -> None:
    ad = ferret_adaptive(_ptr(lambda_dev), _ptr(v_r), _ptr(v_a), alpha, eta_lambda, int(fused), 0)
    _check(load().ferret_compensate_step_adaptive(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), byref(ad), lr,
                                                  _ptr(norms_out), _ptr(grad_out), _ptr(workspace),
                                                  _stream(stream)))


def ferret_compensate_stages(plan: "Plan", ring, grads, master, active: Sequence[int], lam: float, lr: float,
                             norms_out=None, grad_out=None, workspace=None, stream=None) -> None:
    arr = (c_int32 * plan.n_stages)(*[int(bool(x)) for x in active])
    _check(load().ferret_compensate_stages(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), arr, lam, lr,
                                           _ptr(norms_out), _ptr(grad_out), _ptr(workspace), _stream(stream)))


def ferret_compensate_stages_adaptive(plan: "Plan", ring, grads, master, active: Sequence[int], lambda_dev, v_r, v_a,
                                      alpha: float, eta_lambda: float, lr: float, norms_out=None, grad_out=None,
                                      workspace=None, stream=None, fused: bool = False) -> None:
    arr = (c_int32 * plan.n_stages)(*[int(bool(x)) for x in active])
    ad = ferret_adaptive(_ptr(lambda_dev), _ptr(v_r), _ptr(v_a), alpha, eta_lambda, int(fused), 0)
    _check(load().ferret_compensate_stages_adaptive(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), arr, byref(ad),
                                                    lr, _ptr(norms_out), _ptr(grad_out), _ptr(workspace),
                                                    _stream(stream)))


def ferret_accumulate_step(plan: "Plan", ring, grads, master, accum, scale: float, mode: Sequence[int],
                           staleness: Optional[Sequence[int]], lam: float, lr: float, norms_out=None,
                           grad_out=None, workspace=None, stream=None) -> None:
    P = plan.n_stages
    mode_arr = (c_int32 * P)(*[int(m) for m in mode])
    st_arr = (c_int32 * P)(*[int(x) for x in staleness]) if staleness is not None else None
    acc = ferret_accumulate(_ptr(accum), scale, mode_arr, st_arr)
    _check(load().ferret_accumulate_step(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), byref(acc), lam, lr,
                                         _ptr(norms_out), _ptr(grad_out), _ptr(workspace), _stream(stream)))


def ferret_accumulate_step_adaptive(plan: "Plan", ring, grads, master, accum, scale: float, mode: Sequence[int],
                                    staleness: Optional[Sequence[int]], lambda_dev, v_r, v_a, alpha: float,
                                    eta_lambda: float, lr: float, norms_out=None, grad_out=None, workspace=None,
                                    stream=None, fused: bool = False) -> None:
    P = plan.n_stages
    mode_arr = (c_int32 * P)(*[int(m) for m in mode])
    st_arr = (c_int32 * P)(*[int(x) for x in staleness]) if staleness is not None else None
    acc = ferret_accumulate(_ptr(accum), scale, mode_arr, st_arr)
    ad = ferret_adaptive(_ptr(lambda_dev), _ptr(v_r), _ptr(v_a), alpha, eta_lambda, int(fused), 0)
    _check(load().ferret_accumulate_step_adaptive(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), byref(acc),
                                                  byref(ad), lr, _ptr(norms_out), _ptr(grad_out), _ptr(workspace),
                                                  _stream(stream)))


def ferret_penalized_step(plan: "Plan", ring, grads, master, scale: Optional[Sequence[float]],
                          inv_c: Optional[Sequence[float]], lr: float, norms_out=None, grad_out=None, workspace=None,
                          stream=None) -> None:
    P = plan.n_stages
    sc = (c_float * P)(*scale) if scale is not None else None
    ic = (c_float * P)(*inv_c) if inv_c is not None else None
    _check(load().ferret_penalized_step(plan.handle, _ptr(ring), _ptr(grads), _ptr(master), sc, ic, lr,
                                        _ptr(norms_out), _ptr(grad_out), _ptr(workspace), _stream(stream)))


def ferret_stream_mix(dst, src, src_stride_bytes: int, n_reads: int, n_bytes: int, resident_cap: int = 0,
                      stream=None) -> None:
    _check(load().ferret_stream_mix(_ptr(dst), _ptr(src), src_stride_bytes, n_reads, n_bytes, resident_cap,
                                    _stream(stream)))


def ferret_copy_bytes(dst, src, n_bytes: int, stream=None) -> None:
    _check(load().ferret_copy_bytes(_ptr(dst), _ptr(src), n_bytes, _stream(stream)))


def ferret_read_bytes(src, n_bytes: int, sink, stream=None) -> None:
    _check(load().ferret_read_bytes(_ptr(src), n_bytes, _ptr(sink), _stream(stream)))


def ferret_profile_begin(capacity: int) -> None:
    _check(load().ferret_profile_begin(capacity))


def ferret_profile_end(capacity: int) -> List[float]:
    """Durations (ms) of the step-kernel launches recorded since ferret_profile_begin."""
    buf = (c_float * max(capacity, 1))()
    n = c_int32(0)
    _check(load().ferret_profile_end(buf, capacity, byref(n)))
    return [float(buf[i]) for i in range(min(n.value, capacity))]


class Plan:
    """Owner of a ferret_plan*; attribute-style access to the header's plan queries."""

    def __init__(self, handle):
        self.handle = handle
        self._lib = load()

    def destroy(self) -> None:
        if self.handle:
            self._lib.ferret_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def _q(self, name, *args):
        return getattr(self._lib, "ferret_plan_" + name)(self.handle, *args)

    n_stages = property(lambda s: s._q("n_stages"))
    n_tensors = property(lambda s: s._q("n_tensors"))
    precision = property(lambda s: s._q("precision"))
    n_iters = property(lambda s: s._q("n_iters"))
    chunk_elems = property(lambda s: s._q("chunk_elems"))
    n_chunks = property(lambda s: s._q("n_chunks"))
    flat_elems = property(lambda s: s._q("flat_elems"))
    ring_elems = property(lambda s: s._q("ring_elems"))
    ring_bytes = property(lambda s: s._q("ring_bytes"))
    grad_bytes = property(lambda s: s._q("grad_bytes"))
    master_bytes = property(lambda s: s._q("master_bytes"))
    workspace_bytes = property(lambda s: s._q("workspace_bytes"))
    total_params = property(lambda s: s._q("total_params"))
    step_bytes = property(lambda s: s._q("step_bytes"))

    def stage_params(self, j): return self._q("stage_params", j)
    def stage_numel(self, j): return self._q("stage_numel", j)
    def stage_flat_offset(self, j): return self._q("stage_flat_offset", j)
    def stage_ring_offset(self, j): return self._q("stage_ring_offset", j)
    def stage_slot_stride(self, j): return self._q("stage_slot_stride", j)
    def stage_ring_depth(self, j): return self._q("stage_ring_depth", j)
    def stage_staleness(self, j): return self._q("stage_staleness", j)
    def stage_chunk_elems(self, j): return self._q("stage_chunk_elems", j)
    def stage_n_chunks(self, j): return self._q("stage_n_chunks", j)
    def tensor_offset(self, i): return self._q("tensor_offset", i)
    def stage_effective_staleness(self, j): return self._q("stage_effective_staleness", j)
    def stage_effective_iters(self, j): return self._q("stage_effective_iters", j)
    def stage_write_slot(self, j): return self._q("stage_write_slot", j)

    def stage_read_slots(self, j) -> List[int]:
        n = self._q("stage_read_slots", j, None, 0)
        if n <= 0:
            return []
        buf = (c_int32 * n)()
        self._q("stage_read_slots", j, buf, n)
        return list(buf)

    def get_state(self):
        P = self.n_stages
        h, v = (c_int32 * P)(), (c_int32 * P)()
        _check(self._q("get_state", h, v))
        return list(h), list(v)

    def set_state(self, heads: Sequence[int], valid: Sequence[int]) -> None:
        P = self.n_stages
        if len(heads) != P or len(valid) != P:
            raise ValueError("heads/valid must have one entry per stage")
        _check(self._q("set_state", (c_int32 * P)(*heads), (c_int32 * P)(*valid)))

    def slot_offset(self, j: int, slot: int) -> int:
        """Element offset of (stage j, slot) in the ring."""
        return self.stage_ring_offset(j) + slot * self.stage_slot_stride(j)


def plan_for_workload(w, chunk_elems: int = 0, tuning: Optional[dict] = None,
                      ring_depth: Optional[int] = None, n_iters: Optional[int] = None) -> Plan:
    prec = FERRET_F32 if w.precision == "f32" else FERRET_BF16_MASTER_F32
    return ferret_plan_buckets([(n, s) for _, n, s in w.tensors], w.n_stages, w.staleness,
                               w.n_iters if n_iters is None else n_iters,
                               w.ring_depth if ring_depth is None else ring_depth, prec, chunk_elems,
                               tuning)


class DeviceState:
    """Device buffers for one plan, zero-filled, plus scatter/gather of logical stage data.

    Logical data of a stage = its tensors concatenated without padding (what the workload
    generator and the oracle use); the plan's layout puts each tensor at
    `plan.tensor_offset(i)` inside the stage.
    """

    def __init__(self, plan: Plan, tensors: Sequence, device="cuda", want_grad_out=True, want_norms=True):
        self.plan = plan
        self.tensors = list(tensors)        # (numel, stage) in plan order
        self.device = torch.device(device)
        self.storage = torch.float32 if plan.precision == FERRET_F32 else torch.bfloat16
        z = dict(device=self.device)
        self.ring = torch.zeros(plan.ring_elems, dtype=self.storage, **z)
        self.grads = torch.zeros(plan.flat_elems, dtype=self.storage, **z)
        self.master = (torch.zeros(plan.flat_elems, dtype=torch.float32, **z)
                       if plan.precision == FERRET_BF16_MASTER_F32 else None)
        self.grad_out = torch.zeros(plan.flat_elems, dtype=torch.float32, **z) if want_grad_out else None
        self.norms = torch.zeros(plan.n_stages, 3, dtype=torch.float32, **z) if want_norms else None
        self.workspace = (torch.zeros(max(plan.workspace_bytes // 4, 4), dtype=torch.float32, **z)
                          if want_norms else None)
        # per stage: list of (offset inside stage, numel)
        self._pieces = [[] for _ in range(plan.n_stages)]
        for i, (numel, stage) in enumerate(self.tensors):
            self._pieces[stage].append((plan.tensor_offset(i), int(numel)))

    # -- logical <-> padded ------------------------------------------------------------------
    def _scatter(self, dst: torch.Tensor, base: int, j: int, logical: torch.Tensor) -> None:
        pos = 0
        for off, n in self._pieces[j]:
            dst[base + off: base + off + n].copy_(logical[pos: pos + n])
            pos += n
        if pos != logical.numel():
            raise ValueError("logical stage data has the wrong size")

    def _gather(self, src: torch.Tensor, base: int, j: int) -> torch.Tensor:
        return torch.cat([src[base + off: base + off + n] for off, n in self._pieces[j]]).cpu()

    def set_version(self, j: int, slot: int, logical: torch.Tensor) -> None:
        self._scatter(self.ring, self.plan.slot_offset(j, slot), j, logical.to(self.storage))

    def get_version(self, j: int, slot: int) -> torch.Tensor:
        return self._gather(self.ring, self.plan.slot_offset(j, slot), j)

    def set_flat(self, buf: torch.Tensor, j: int, logical: torch.Tensor) -> None:
        self._scatter(buf, self.plan.stage_flat_offset(j), j, logical.to(buf.dtype))

    def get_flat(self, buf: torch.Tensor, j: int) -> torch.Tensor:
        return self._gather(buf, self.plan.stage_flat_offset(j), j)

    def load_versions(self, j: int, versions: Sequence[torch.Tensor], head: Optional[int] = None) -> int:
        """Write `versions` (oldest first) so that the newest sits in slot `head`
        (default: len-1 mod R); returns head.  Does not touch the plan's state."""
        R = self.plan.stage_ring_depth(j)
        n = len(versions)
        if n > R:
            raise ValueError("more versions than ring slots")
        if head is None:
            head = (n - 1) % R
        for age, v in enumerate(reversed(versions)):
            self.set_version(j, (head - age) % R, v)
        return head

    # -- calls -------------------------------------------------------------------------------
    def step(self, lam: float, lr: float, norms: bool = True, grad_out: bool = True, stream=None) -> None:
        ferret_compensate_step(self.plan, self.ring, self.grads, self.master, lam, lr,
                               self.norms if norms else None,
                               self.grad_out if grad_out else None,
                               self.workspace if norms else None, stream)

    def enable_adaptive(self, lambda0: float) -> None:
        """Allocate the self-tuning state: lambda_j = lambda0, v_r = v_a = 0 (Alg. 1, initialisation)."""
        z = dict(device=self.device, dtype=torch.float32)
        self.lambda_dev = torch.full((self.plan.n_stages,), float(lambda0), **z)
        self.v_r = torch.zeros(self.plan.flat_elems, **z)
        self.v_a = torch.zeros(self.plan.flat_elems, **z)
        if self.workspace is None:
            self.workspace = torch.zeros(max(self.plan.workspace_bytes // 4, 4), **z)

    def step_adaptive(self, alpha: float, eta_lambda: float, lr: float, norms: bool = True, grad_out: bool = True,
                      stream=None, fused: bool = False) -> None:
        ferret_compensate_step_adaptive(self.plan, self.ring, self.grads, self.master, self.lambda_dev, self.v_r,
                                        self.v_a, alpha, eta_lambda, lr, self.norms if norms else None,
                                        self.grad_out if grad_out else None, self.workspace, stream, fused)

    def commit(self, stage: int = -1) -> None:
        ferret_push_version(self.plan, self.ring, None, stage, None)

    def push(self, src: torch.Tensor, stage: int = -1, with_master: bool = True, stream=None) -> None:
        ferret_push_version(self.plan, self.ring, self.master if with_master else None, stage, src, stream)


# ---- pipeline planner (include/ferret_planner.h) -------------------------------------------------
def _layer_array(layers):
    arr = (ferret_layer * max(len(layers), 1))()
    for i, (t_f, t_b, n_params, n_acts) in enumerate(layers):
        arr[i].t_f, arr[i].t_b, arr[i].n_params, arr[i].n_acts = t_f, t_b, n_params, n_acts
    return arr


def ferret_pipeline_evaluate(layers, L, delay, recompute, accum, omit, c: float, v_d: float):
    """layers: (t_f, t_b, n_params, n_acts) tuples; accum/omit: list per worker of list per stage."""
    P, N = len(L) - 1, len(delay)
    flat = lambda rows: (c_int32 * max(N * P, 1))(*[int(x) for r in rows for x in r])
    R, M = ctypes.c_double(), ctypes.c_double()
    _check(load().ferret_pipeline_evaluate(_layer_array(layers), len(layers), (c_int32 * (P + 1))(*L), P, N,
                                           (c_int32 * max(N, 1))(*delay), (c_int32 * max(N, 1))(*recompute),
                                           flat(accum), flat(omit), c, v_d, byref(R), byref(M)))
    return R.value, M.value


class Pipeline:
    """Result of ferret_pipeline_search / ferret_pipeline_plan."""

    def __init__(self, handle):
        self.handle, self._lib = handle, load()

    def __del__(self):
        try:
            if self.handle:
                self._lib.ferret_pipeline_destroy(self.handle)
                self.handle = None
        except Exception:
            pass

    def _q(self, name, *a):
        return getattr(self._lib, "ferret_pipeline_" + name)(self.handle, *a)

    feasible = property(lambda s: bool(s._q("feasible")))
    n_stages = property(lambda s: s._q("n_stages"))
    n_workers = property(lambda s: s._q("n_workers"))
    rate = property(lambda s: s._q("rate"))
    memory = property(lambda s: s._q("memory"))
    stage_bound = property(lambda s: s._q("stage_bound"))

    @property
    def L(self):
        return [self._q("stage_begin", j) for j in range(self.n_stages + 1)]

    def worker(self, n):
        P = self.n_stages
        return dict(delay=self._q("worker_delay", n), recompute=self._q("worker_recompute", n),
                    accum=[self._q("worker_accum", n, j) for j in range(P)],
                    omit=[self._q("worker_omit", n, j) for j in range(P)],
                    versions=[self._q("stage_versions", n, j) for j in range(P)])

    @property
    def moves(self):
        out = []
        for k in range(self._q("n_moves")):
            w, kind, st = c_int32(), c_int32(), c_int32()
            _check(self._q("move", k, byref(w), byref(kind), byref(st)))
            out.append((w.value, "S%d" % kind.value, st.value))
        return out


def ferret_pipeline_search(layers, L, t_d: float, memory_budget: float, c: float, v_d: float) -> Pipeline:
    out = _P()
    P = len(L) - 1
    _check(load().ferret_pipeline_search(_layer_array(layers), len(layers), (c_int32 * (P + 1))(*L), P, t_d,
                                         memory_budget, c, v_d, byref(out)))
    return Pipeline(out)


def ferret_pipeline_plan(layers, t_d: float, memory_budget: float, c: float, v_d: float) -> Pipeline:
    out = _P()
    _check(load().ferret_pipeline_plan(_layer_array(layers), len(layers), t_d, memory_budget, c, v_d, byref(out)))
    return Pipeline(out)
