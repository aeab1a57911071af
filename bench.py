#!/usr/bin/env python3
"""Benchmark of the fused compensate + update step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-norms] [--no-cpu-baseline] [--no-others]

A "step" is one pass of the whole path over every stage of the workload:
ferret_compensate_step (gradient load, K'+1 version loads, K' iterations, update, store of the
new version into the next ring slot, per-stage norms) followed by ferret_push_version(src=NULL)
(head advance).  Heads advance every step, so successive steps touch different ring slots.

Inputs are seeded and synthetic (paper_2503_12053_amd.workloads) and resident in HBM before the timed
region.  One JSON line goes to stdout; context goes to stderr.  The top-level fields of that line are the
headline workload (the ViT-B-sized one unless --config says otherwise) in the mode the flags select; a default
run adds `others`: the same measurement of the other headline modes and of the 350 M-parameter workload.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def library_source_hash(B) -> str:
    """The source hash the loaded library was built from (last word of ferret_version())."""
    return B.load().ferret_version().decode().split()[-1]


def read_traffic(key, lib_hash):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE) from the summary committed
    under profiles/ for this workload and mode -- used only if that summary was taken from a library built from
    the same sources as the one being timed (the summary records the source hash).
    Returns (bytes or None, description of where it came from or why it is missing)."""
    if key is None:
        return None, "no counter summary is kept for this mode"
    name = f"hbm_traffic_{key}.txt"
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, f"profiles/{name} does not exist"
    text = open(path).read()
    m_hash = re.search(r"^library_source_hash:\s*(\S+)", text, re.M)
    m_bytes = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", text, re.M)
    if not m_hash or not m_bytes:
        return None, f"profiles/{name} has no source hash or traffic line"
    if m_hash.group(1) != lib_hash:
        return None, f"profiles/{name} was taken at source hash {m_hash.group(1)}, this library is {lib_hash}"
    return float(m_bytes.group(1)), f"profiles/{name} (source hash {lib_hash})"


def cpu_baseline(w, host, plan, budget_s=20.0):
    """Time the oracle (as it stands) on the host cores over one step of the same workload.
    host: {stage index: StageData on the CPU} for the stages that may be sampled."""
    import numpy as np
    from oracle import ferret_oracle as O
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))

    def one_step(n_threads, stages):
        t0 = time.perf_counter()
        n = 0
        for j in stages:
            tau = plan.stage_effective_staleness(j)
            window = host[j].versions[len(host[j].versions) - 1 - tau:]
            if w.precision == "f32":
                O.compensate_stage_f32(window, host[j].grads, w.n_iters, np.float32(w.lam), np.float32(w.lr),
                                       n_threads=n_threads, want_g=False)
            else:
                O.compensate_stage_bf16(window, host[j].grads, host[j].master, w.n_iters, np.float32(w.lam),
                                        np.float32(w.lr), n_threads=n_threads, want_g=False)
            n += w.stage_numel()[j]
        return time.perf_counter() - t0, n

    # bounded sample: whole stages in order, as many as fit the time budget (probe with the smallest one held)
    have = sorted(host)
    t_probe, n_probe = one_step(1, [min(have, key=lambda j: w.stage_numel()[j])])
    rate1 = n_probe / t_probe
    stages, acc = [], 0
    for j in have:
        if (acc + w.stage_numel()[j]) / rate1 > budget_s * 0.5 and stages:
            break
        stages.append(j)
        acc += w.stage_numel()[j]
    reps = max(1, min(5, int(budget_s * 0.4 / max(acc / rate1, 1e-3))))
    t1, n1 = min(one_step(1, stages) for _ in range(reps))
    reps_n = max(reps, min(30, int(budget_s * 0.1 / max(t1 / cores, 1e-3))))     # the threaded runs are short: more of them
    tn, nn = min(one_step(cores, stages) for _ in range(reps_n))
    sample = (f"one step of stages {stages[0]}..{stages[-1]} of {w.name} ({n1} of {w.numel} parameters), "
              f"fp64 oracle: 1 thread best of {reps} {t1:.2f} s, {cores} threads best of {reps_n} {tn:.3f} s")
    return {"value": nn / tn, "unit": "params/s", "cores": cores, "kind": "oracle", "sample": sample,
            "single_thread_value": n1 / t1}


def per_tensor_contrast(w, args, torch, B, W):
    """The same step issued as one launch per parameter tensor (what a per-tensor optimizer loop does)."""
    states = []
    for j in range(w.n_stages):
        d = W.generate_stage(w, j)
        pos = 0
        for _, n in w.stage_tensors(j):
            plan = B.ferret_plan_buckets([(n, 0)], 1, [w.staleness[j]], w.n_iters, w.ring_depth,
                                         B.FERRET_F32 if w.precision == "f32" else B.FERRET_BF16_MASTER_F32)
            st = B.DeviceState(plan, [(n, 0)], want_grad_out=False, want_norms=not args.no_norms)
            head = st.load_versions(0, [v[pos:pos + n] for v in d.versions])
            st.set_flat(st.grads, 0, d.grads[pos:pos + n])
            if d.master is not None:
                st.set_flat(st.master, 0, d.master[pos:pos + n])
            plan.set_state([head], [w.ring_depth])
            states.append(st)
            pos += n
    norms = not args.no_norms

    def one_step():
        for st in states:
            st.step(w.lam, w.lr, norms=norms, grad_out=False)
            st.commit()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    elapsed = (time.perf_counter() - t0) / args.steps
    step_bytes = sum(st.plan.step_bytes for st in states)
    log(f"per-tensor launches: {len(states)} launches per step, {elapsed * 1e6:.1f} us wall per step, "
        f"{w.numel / elapsed:.3e} params/s, {step_bytes / elapsed / 1e9:.0f} GB/s algorithmic")
    print(json.dumps({"metric": "compensated_params_per_sec", "value": w.numel / elapsed, "unit": "params/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed * 1e3,
                      "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.precision,
                      "data": "synthetic",
                      "config": {"workload": w.name, "mode": "one launch per tensor", "launches_per_step": len(states)}}),
          flush=True)


class Mode:
    """Which variant of the step is timed."""

    def __init__(self, adaptive=False, fused=False, accumulate=0, compensator="iter-fisher", graph=False,
                 norms=True, kernel_events=True):
        self.adaptive, self.fused, self.accumulate = adaptive or fused, fused, accumulate
        self.compensator, self.graph, self.norms, self.kernel_events = compensator, graph, norms, kernel_events

    @property
    def label(self):
        if self.accumulate:
            return f"accumulation of {self.accumulate} gradients"
        if self.fused:
            return "self-tuned lambda, one pass"
        if self.adaptive:
            return "self-tuned lambda, Alg. 1's order"
        return {"iter-fisher": "fixed lambda"}.get(self.compensator, self.compensator)


def load_inputs(torch, B, W, w, plan, st, device_draw, keep_host):
    """Fill the ring, the gradient and the master.  device_draw: draw on the GPU (fast; same recipe, other random
    streams) instead of with the CPU generators of the parity tests.  keep_host: stage indices whose data is kept
    (on the CPU) for the oracle.  Returns {stage: StageData}."""
    host, heads = {}, []
    for j in range(w.n_stages):
        d = W.generate_stage(w, j, device=st.device if device_draw else "cpu")
        heads.append(st.load_versions(j, d.versions))
        st.set_flat(st.grads, j, d.grads)
        if d.master is not None:
            st.set_flat(st.master, j, d.master)
        if j in keep_host:
            host[j] = W.StageData([v.cpu() for v in d.versions], d.grads.cpu(),
                                  None if d.master is None else d.master.cpu())
    plan.set_state(heads, [w.ring_depth] * w.n_stages)
    torch.cuda.synchronize()
    return host


def measure(torch, B, w, plan, st, mode, steps, warmup):
    """Warm up, then time `steps` steps of the workload in the given mode.  Returns the figures of the record."""
    dev, norms = st.device, mode.norms
    elt = 4 if w.precision == "f32" else 2
    kp = [plan.stage_effective_iters(j) for j in range(w.n_stages)]
    step_bytes = plan.step_bytes                     # the plain step; modes add to it below
    per_launch_bytes = step_bytes
    if mode.adaptive:
        # Alg. 1 with eta_lambda > 0: lambda_j starts at lambda0, averages at zero; the paper's run uses a small
        # lambda learning rate (its "mu" = 2e-6)
        st.enable_adaptive(w.lam)
        if mode.fused:   # g_0 and V[0] are read once; V[1] is extra only where it is not a segment boundary
            extra = sum((16 + (0 if t // k == 1 else elt)) * n for n, t, k in zip(w.stage_numel(), w.staleness, kp) if t >= 1)
            per_launch_bytes += extra
        else:            # a second pass over g_0, V[0], V[1], v_r, v_a (read) and v_r, v_a (written)
            extra = sum((3 * elt + 16) * n for n, t in zip(w.stage_numel(), w.staleness) if t >= 1)
        step_bytes += extra
    accum = None
    if mode.accumulate:
        ca = mode.accumulate
        accum = torch.zeros(plan.flat_elems, dtype=torch.float32, device=dev)
        per_arrival = sum((elt * (k + 2) + 8) * n for k, n in zip(kp, w.stage_numel()))
        last_extra = sum((elt + (8 if w.precision == "bf16" else 0)) * n for n in w.stage_numel())
        step_bytes = ca * per_arrival + last_extra
        per_launch_bytes = step_bytes / ca
    if mode.compensator in ("step-aware", "gap-aware") or (mode.compensator == "none" and norms):
        # V[0] is read besides V[tau] (for the gap, or for the weight-gap norm) in stages with staleness
        extra = sum(elt * n for n, t in zip(w.stage_numel(), w.staleness) if t >= 1)
        step_bytes += extra
        per_launch_bytes += extra

    def one_step():
        if mode.accumulate:
            for k in range(mode.accumulate):
                last = k == mode.accumulate - 1
                B.ferret_accumulate_step(plan, st.ring, st.grads, st.master, accum, 1.0 / mode.accumulate,
                                         [2 if last else 1] * w.n_stages, None, w.lam, w.lr,
                                         st.norms if norms else None, None, st.workspace if norms else None)
            st.commit()
            return
        if mode.compensator in ("step-aware", "gap-aware"):
            gap = mode.compensator == "gap-aware"
            B.ferret_penalized_step(plan, st.ring, st.grads, st.master, [1.0] * w.n_stages if gap else None,
                                    [1.0 / (w.lr * w.grad_std)] * w.n_stages if gap else None, w.lr,
                                    st.norms if norms else None, None, st.workspace if norms else None)
        elif mode.adaptive:
            st.step_adaptive(0.9, 2e-6, w.lr, norms=norms, grad_out=False, fused=mode.fused)
        else:
            st.step(w.lam, w.lr, norms=norms, grad_out=False)
        st.commit()

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()

    launches = max(mode.accumulate, 1)
    kernel_ms = None
    if mode.graph:
        # after ring_depth steps every head is back where it started, so a graph of one rotation
        # can be replayed for ever; the host-side commits inside the capture only move integers
        R = w.ring_depth
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                for _ in range(R):
                    one_step()
        torch.cuda.current_stream().wait_stream(side)
        replays = max(steps // R, 1)
        steps = replays * R
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        log(f"graph of {R} steps replayed {replays} times")
    else:
        if mode.kernel_events:
            B.ferret_profile_begin(steps * launches)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            one_step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        if mode.kernel_events:
            kernel_ms = B.ferret_profile_end(steps * launches)
    ms_per_step = elapsed * 1e3 / steps
    if not kernel_ms:
        kernel_ms = [ms_per_step / launches]         # no per-launch events: the roofline is taken from wall time

    # per-step spread: a second, untimed-for-`value` run of 50 steps with one event between steps
    # (step period = kernel(s) + launch gaps, as the device sees it)
    step_med_us = step_min_us = None
    if not mode.graph:
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(51)]
        marks[0].record()
        for i in range(50):
            one_step()
            marks[i + 1].record()
        torch.cuda.synchronize()
        periods = [marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(50)]
        step_med_us, step_min_us = statistics.median(periods), min(periods)
    if mode.adaptive:
        del st.lambda_dev, st.v_r, st.v_a
    k_avg, k_med = statistics.fmean(kernel_ms), statistics.median(kernel_ms)
    achieved = per_launch_bytes / (k_avg * 1e-3) / 1e9     # the fused step kernel alone
    log(f"{w.name}, {mode.label}: {ms_per_step * 1e3:.1f} us wall per step"
        + (f" (device step period median {step_med_us:.1f}, min {step_min_us:.1f} us)" if step_med_us else "")
        + f"; fused kernel avg {k_avg * 1e3:.1f} us, median {k_med * 1e3:.1f} us, min {min(kernel_ms) * 1e3:.1f} us"
        f" -> {achieved:.0f} GB/s algorithmic ({achieved / HBM_PEAK_GBS:.1%} of {HBM_PEAK_GBS:.0f} GB/s)")
    return dict(steps=steps, ms_per_step=ms_per_step, params_per_s=w.numel / (elapsed / steps), step_bytes=step_bytes,
                per_launch_bytes=per_launch_bytes, kernel_avg_us=k_avg * 1e3, kernel_median_us=k_med * 1e3,
                achieved=achieved, step_median_us=step_med_us, step_min_us=step_min_us,
                hbm_gbs_wall=step_bytes / (elapsed / steps) / 1e9)


def ceilings(torch, B, w, plan, st, with_mix):
    """Context: what plain streaming kernels of the library reach on the same buffers in the same run."""
    dev = st.device
    n_copy = min(plan.ring_bytes // 2, 1 << 30) // 16 * 16
    src_t = st.ring.view(torch.uint8)[:n_copy]
    dst_t = (st.ring.view(torch.uint8)[plan.ring_bytes - n_copy:] if plan.ring_bytes >= 2 * n_copy
             else torch.empty(n_copy, dtype=torch.uint8, device=dev))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for _ in range(3):
        B.ferret_copy_bytes(dst_t, src_t, n_copy)
    ev[0].record()
    for _ in range(10):
        B.ferret_copy_bytes(dst_t, src_t, n_copy)
    ev[1].record()
    torch.cuda.synchronize()
    copy_gbs = 2 * n_copy * 10 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    n_read = plan.ring_bytes // 16 * 16
    for _ in range(3):
        B.ferret_read_bytes(st.ring, n_read, sink)
    ev[0].record()
    for _ in range(10):
        B.ferret_read_bytes(st.ring, n_read, sink)
    ev[1].record()
    torch.cuda.synchronize()
    read_gbs = n_read * 10 / (ev[0].elapsed_time(ev[1]) * 1e-3) / 1e9
    log(f"context: copy kernel {copy_gbs:.0f} GB/s (read+write, {n_copy / 1e6:.0f} MB), "
        f"read-only kernel {read_gbs:.0f} GB/s ({n_read / 1e6:.0f} MB)")
    # the step's traffic shape without its arithmetic or tables -- per stage, a kernel that adds NR read streams
    # into one write stream, NR = that stage's read bytes / write bytes, sized so that the bytes written match the
    # stage's; the time of all stages together against the step's algorithmic bytes
    mix_gbs = None
    if with_mix:
        elt = 4 if w.precision == "f32" else 2
        shapes = []
        for j in range(w.n_stages):
            kp = plan.stage_effective_iters(j)
            rd = elt * (kp + 2) + (0 if w.precision == "f32" else 4)
            wr = elt + (0 if w.precision == "f32" else 4)
            nr = max(1, min(8, round(rd / wr)))
            shapes.append((nr, w.stage_numel()[j] * wr // 16 * 16))
        need = max((nr + 1) * nb for nr, nb in shapes)
        if need <= plan.ring_bytes:
            ring_u8 = st.ring.view(torch.uint8)
            best = None
            for cap in (-1, 2, 3, 4, 5):
                def emulate():
                    for nr, nb in shapes:
                        B.ferret_stream_mix(ring_u8[nr * nb:], ring_u8, nb, nr, nb, cap)
                for _ in range(2):
                    emulate()
                ev[0].record()
                for _ in range(5):
                    emulate()
                ev[1].record()
                torch.cuda.synchronize()
                t = ev[0].elapsed_time(ev[1]) * 1e-3 / 5
                best = t if best is None else min(best, t)
            mix_gbs = plan.step_bytes / best / 1e9
            log(f"context: same traffic shape without the arithmetic (per stage, {[nr for nr, _ in shapes]} read "
                f"streams + 1 write stream, best resident cap): {best * 1e6:.1f} us per step-equivalent "
                f"-> {mix_gbs:.0f} GB/s")
    return copy_gbs, read_gbs, mix_gbs


def roofline_of(m, traffic, traffic_source, extra=None):
    r = {"bound": "hbm", "achieved": m["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
         "frac": m["achieved"] / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
         "algorithmic_bytes_per_launch": m["per_launch_bytes"],
         "kernel": "ferret::step_kernel", "kernel_avg_us": m["kernel_avg_us"], "kernel_median_us": m["kernel_median_us"]}
    if extra:
        r.update(extra)
    return r


def traffic_key(w_name, mode, iters, tuned):
    """Name of the committed counter summary that covers this workload and mode, if one is kept.
    iters: None = the workload's own iteration count, -1 = one per version step."""
    if tuned or not mode.norms or mode.graph or mode.compensator != "iter-fisher" or iters not in (None, -1):
        return None
    if mode.accumulate:
        return w_name + "_accumulate2" if iters is None and mode.accumulate == 2 else None
    base = w_name + ("_full_iterations" if iters == -1 else "")
    if mode.fused:
        return base + "_one_pass_lambda"
    if mode.adaptive:
        return base + "_adaptive"
    return base


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (4 = the one the metric is quoted on)")
    ap.add_argument("--no-norms", action="store_true", help="skip the per-stage norms (not the default path)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="time only the workload and mode the flags select (a default run also times the other "
                         "headline modes and the 350 M-parameter workload and reports them under `others`)")
    ap.add_argument("--chunk-elems", type=int, default=0)
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--resident-cap", type=int, default=0)
    ap.add_argument("--chunk-bytes", type=int, default=0,
                    help="size every stage's chunks so that one chunk moves about this many bytes (sweeps)")
    ap.add_argument("--cache-policy", type=int, default=0, choices=[0, 1, 2],
                    help="0 by working-set size, 1 cached accesses where available, 2 non-temporal (sweeps)")
    ap.add_argument("--xcd-group", type=int, default=0,
                    help="consecutive chunks per XCD (ferret_tuning.xcd_group: 0 library default, 1 plain order)")
    ap.add_argument("--slot-align", type=int, default=0)
    ap.add_argument("--slot-skew", type=int, default=0)
    ap.add_argument("--iters", type=int, default=None, help="override K (-1 = one iteration per version step)")
    ap.add_argument("--precision", choices=["f32", "bf16"], default=None,
                    help="override the workload's storage type (for sweeps; not a benchmark configuration)")
    ap.add_argument("--adaptive", action="store_true",
                    help="time the self-tuned-lambda step (all of Alg. 1) instead of the fixed-lambda step")
    ap.add_argument("--adaptive-fused", action="store_true",
                    help="as --adaptive, but in one pass: each lambda step takes effect one call later than in Alg. 1")
    ap.add_argument("--accumulate", type=int, default=0, metavar="CA",
                    help="time gradient accumulation (T2): one step = CA arrivals per stage, the last one updates")
    ap.add_argument("--compensator", default="iter-fisher",
                    choices=["iter-fisher", "none", "fisher", "step-aware", "gap-aware"],
                    help="which compensation method the step applies (cost structure of the paper's comparison "
                         "of compensation methods): iter-fisher = the configured K, none = K 0, fisher = K 1")
    ap.add_argument("--newest-from-master", action="store_true",
                    help="bf16 workloads: recompute the newest version from the master instead of reading it")
    ap.add_argument("--graph", action="store_true",
                    help="capture one full ring rotation (ring_depth steps) in a HIP graph and time replays; "
                         "removes the launch overhead that dominates the small workloads")
    ap.add_argument("--per-tensor", action="store_true",
                    help="contrast: one plan and one launch per tensor instead of one bucketed launch per step")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not record per-launch HIP events (roofline is then taken from wall time)")
    ap.add_argument("--device-draw", action="store_true",
                    help="draw the inputs on the GPU (same recipe, other random streams): seconds instead of a "
                         "minute for the 350 M-parameter workload")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build measures one GPU only (the path has no cross-GPU step); run with --gpus 1")
        sys.exit(2)

    import torch
    from paper_2503_12053_amd import binding as B
    from paper_2503_12053_amd import workloads as W

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    B.load()
    lib_hash = library_source_hash(B)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    w = W.make_workload(args.config)
    if args.precision:                       # sweeps only: the same shapes in the other storage type
        w.precision = args.precision
        w.name += "_as_" + args.precision
    if args.iters is not None:
        w.n_iters = args.iters
    if args.compensator in ("none", "step-aware", "gap-aware"):
        w.n_iters = 0
    elif args.compensator == "fisher":
        w.n_iters = 1
    if args.per_tensor:
        return per_tensor_contrast(w, args, torch, B, W)
    tuning = None
    tuned = bool(args.blocks_per_cu or args.slot_align or args.slot_skew or args.newest_from_master or args.resident_cap
                 or args.chunk_bytes or args.cache_policy or args.xcd_group)
    if tuned:
        tuning = dict(blocks_per_cu=args.blocks_per_cu, slot_align_elems=args.slot_align, resident_cap=args.resident_cap,
                      slot_skew_elems=args.slot_skew, newest_from_master=int(args.newest_from_master),
                      chunk_bytes=args.chunk_bytes, cache_policy=args.cache_policy, xcd_group=args.xcd_group)
    tuned = tuned or bool(args.chunk_elems) or args.precision is not None
    mode = Mode(adaptive=args.adaptive, fused=args.adaptive_fused, accumulate=args.accumulate,
                compensator=args.compensator, graph=args.graph, norms=not args.no_norms,
                kernel_events=not (args.no_kernel_events or args.graph))
    plain_default = (not tuned and mode.label == "fixed lambda" and not mode.graph and mode.norms and args.iters is None)
    want_others = plain_default and args.config == 4 and not args.no_others

    plan = B.plan_for_workload(w, chunk_elems=args.chunk_elems, tuning=tuning)
    st = B.DeviceState(plan, [(n, s) for _, n, s in w.tensors], device=dev, want_grad_out=False,
                       want_norms=mode.norms or mode.adaptive)
    t0 = time.perf_counter()
    if args.no_cpu_baseline:
        keep = set()
    elif args.device_draw:
        keep = {0, 1} & set(range(w.n_stages))       # the oracle's sample: the first stages, copied back
    else:
        keep = set(range(w.n_stages))
    host = load_inputs(torch, B, W, w, plan, st, args.device_draw, keep)
    log(f"library {B.load().ferret_version().decode()}")
    log(f"workload {w.name}: {w.numel} parameters, {w.n_stages} stages, ring {plan.ring_bytes / 1e9:.2f} GB, "
        f"{plan.n_chunks} chunks of {sorted(set(plan.stage_chunk_elems(j) for j in range(w.n_stages)))} elements, "
        f"algorithmic bytes/step {plan.step_bytes} (inputs ready in {time.perf_counter() - t0:.1f} s)")

    m = measure(torch, B, w, plan, st, mode, args.steps, args.warmup)
    with_mix = mode.label == "fixed lambda" and not args.newest_from_master
    copy_gbs, read_gbs, mix_gbs = ceilings(torch, B, w, plan, st, with_mix)
    traffic, traffic_source = read_traffic(traffic_key(w.name, mode, args.iters, tuned), lib_hash)
    result = {
        "metric": "compensated_params_per_sec",
        "value": m["params_per_s"],
        "unit": "params/s",
        "n_gpus": 1,
        "steps": m["steps"],
        "warmup": args.warmup,
        "ms_per_step": m["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.precision == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": w.name, "params": w.numel, "stages": w.n_stages, "staleness": w.staleness,
                   "ring_depth": w.ring_depth, "n_iters": w.n_iters, "lambda": w.lam, "lr": w.lr,
                   "norms": mode.norms, "adaptive_lambda": ("one-pass" if mode.fused else bool(mode.adaptive)),
                   "accumulation_steps": mode.accumulate, "hip_graph": bool(mode.graph),
                   "newest_from_master": bool(args.newest_from_master), "compensator": mode.compensator,
                   "chunk_elems": [plan.stage_chunk_elems(j) for j in range(w.n_stages)],
                   "algorithmic_bytes_per_step": m["step_bytes"], "library_source_hash": lib_hash},
        "hbm_gbs_wall": m["hbm_gbs_wall"],
        "step_median_us": m["step_median_us"], "step_min_us": m["step_min_us"],
        "roofline": roofline_of(m, traffic, traffic_source,
                                {"copy_kernel_gbs": copy_gbs, "read_kernel_gbs": read_gbs, "mix_kernel_gbs": mix_gbs}),
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, host, plan)
        log("cpu baseline:", result["cpu_baseline"]["sample"])

    if want_others:
        others = []

        def record(wo, mo, mm, key, extra=None):
            tr, src = read_traffic(key, lib_hash)
            rec = {"workload": wo.name, "mode": mo.label, "n_iters": wo.n_iters, "value": mm["params_per_s"],
                   "unit": "params/s", "ms_per_step": mm["ms_per_step"], "steps": mm["steps"],
                   "dtype": "f32" if wo.precision == "f32" else "bf16 storage, f32 arithmetic",
                   "algorithmic_bytes_per_step": mm["step_bytes"], "hbm_gbs_wall": mm["hbm_gbs_wall"],
                   "roofline": roofline_of(mm, tr, src)}
            if extra:
                rec.update(extra)
            others.append(rec)

        # the same buffers in the other headline modes of the ViT-B-sized workload
        for mo, key in ((Mode(adaptive=True), w.name + "_adaptive"), (Mode(fused=True), w.name + "_one_pass_lambda"),
                        (Mode(accumulate=2), w.name + "_accumulate2")):
            record(w, mo, measure(torch, B, w, plan, st, mo, args.steps, args.warmup), key)
        # Alg. 1 literally: one iteration per version step (another plan over the same buffers: the layout is the same)
        w_full = W.make_workload(args.config)
        w_full.n_iters = -1
        plan_full = B.plan_for_workload(w_full)
        plan_full.set_state(*plan.get_state())
        st_full = B.DeviceState.__new__(B.DeviceState)
        st_full.__dict__.update(st.__dict__)
        st_full.plan = plan_full
        st_full.workspace = torch.zeros(max(plan_full.workspace_bytes // 4, 4), dtype=torch.float32, device=dev)
        for mo, key in ((Mode(), w.name + "_full_iterations"), (Mode(adaptive=True), w.name + "_full_iterations_adaptive"),
                        (Mode(fused=True), w.name + "_full_iterations_one_pass_lambda")):
            record(w_full, mo, measure(torch, B, w_full, plan_full, st_full, mo, args.steps, args.warmup), key)
        del st_full, st, plan_full
        torch.cuda.empty_cache()
        # the 350 M-parameter bf16 workload, inputs drawn on the device; the oracle beside it on its first stages
        w5 = W.make_workload(5)
        plan5 = B.plan_for_workload(w5)
        st5 = B.DeviceState(plan5, [(n, s) for _, n, s in w5.tensors], device=dev, want_grad_out=False)
        t0 = time.perf_counter()
        host5 = load_inputs(torch, B, W, w5, plan5, st5, True, set() if args.no_cpu_baseline else {0, 1})
        log(f"workload {w5.name}: {w5.numel} parameters, {plan5.n_chunks} chunks, ring {plan5.ring_bytes / 1e9:.2f} GB, "
            f"algorithmic bytes/step {plan5.step_bytes} (inputs drawn on the device in {time.perf_counter() - t0:.1f} s)")
        steps5 = max(args.steps // 4, 10)
        m5 = measure(torch, B, w5, plan5, st5, Mode(), steps5, max(args.warmup // 2, 3))
        extra = None
        if not args.no_cpu_baseline:
            extra = {"cpu_baseline": cpu_baseline(w5, host5, plan5, budget_s=10.0)}
            log("cpu baseline:", extra["cpu_baseline"]["sample"])
        record(w5, Mode(), m5, w5.name, extra)
        record(w5, Mode(fused=True), measure(torch, B, w5, plan5, st5, Mode(fused=True), steps5, 3),
               w5.name + "_one_pass_lambda")
        result["others"] = others
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
