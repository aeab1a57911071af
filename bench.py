#!/usr/bin/env python3
"""Benchmark of the fused compensate + update step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-norms] [--no-cpu-baseline]

A "step" is one pass of the whole path over every stage of the workload:
ferret_compensate_step (gradient load, K'+1 version loads, K' iterations, update, store of the
new version into the next ring slot, per-stage norms) followed by ferret_push_version(src=NULL)
(head advance).  Heads advance every step, so successive steps touch different ring slots.

Inputs are seeded and synthetic (paper_2503_12053_amd.workloads), generated on the host and
resident in HBM before the timed region.  One JSON line goes to stdout; context goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic(workload_name: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE), if a summary
    for this workload has been committed under profiles/."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload_name}.txt")
    if workload_name is None or not os.path.exists(path):
        return None
    for line in open(path):
        if line.startswith("traffic_bytes_per_launch:"):
            return float(line.split(":")[1])
    return None


def cpu_baseline(w, host, plan, budget_s=20.0):
    """Time the oracle (as it stands) on the host cores over one step of the same workload."""
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

    # bounded sample: whole stages, as many as fit the time budget (probe with the smallest stage)
    order = sorted(range(w.n_stages), key=lambda j: w.stage_numel()[j])
    t_probe, n_probe = one_step(1, order[:1])
    rate1 = n_probe / t_probe
    stages, acc = [], 0
    for j in range(w.n_stages):
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (4 = the one the metric is quoted on)")
    ap.add_argument("--no-norms", action="store_true", help="skip the per-stage norms (not the default path)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-elems", type=int, default=0)
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--resident-cap", type=int, default=0)
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
    if args.blocks_per_cu or args.slot_align or args.slot_skew or args.newest_from_master or args.resident_cap:
        tuning = dict(blocks_per_cu=args.blocks_per_cu, slot_align_elems=args.slot_align, resident_cap=args.resident_cap,
                      slot_skew_elems=args.slot_skew, newest_from_master=int(args.newest_from_master))
    plan = B.plan_for_workload(w, chunk_elems=args.chunk_elems, tuning=tuning)
    st = B.DeviceState(plan, [(n, s) for _, n, s in w.tensors], device=dev, want_grad_out=False,
                       want_norms=not args.no_norms)
    t0 = time.perf_counter()
    host, heads = [], []
    for j in range(w.n_stages):
        d = W.generate_stage(w, j)
        heads.append(st.load_versions(j, d.versions))
        st.set_flat(st.grads, j, d.grads)
        if d.master is not None:
            st.set_flat(st.master, j, d.master)
        host.append(d)
    plan.set_state(heads, [w.ring_depth] * w.n_stages)
    torch.cuda.synchronize()
    step_bytes = plan.step_bytes
    log(f"workload {w.name}: {w.numel} parameters, {w.n_stages} stages, ring {plan.ring_bytes / 1e9:.2f} GB, "
        f"{plan.n_chunks} chunks of {plan.chunk_elems}, algorithmic bytes/step {step_bytes} "
        f"(inputs ready in {time.perf_counter() - t0:.1f} s)")

    norms = not args.no_norms
    fused_extra = 0
    if args.adaptive_fused:
        args.adaptive = True
    if args.adaptive:
        # Alg. 1 with eta_lambda > 0: lambda_j starts at lambda0, averages at zero; the paper's run
        # uses a small lambda learning rate (its "mu" = 2e-6)
        st.enable_adaptive(w.lam)
        elt = 4 if w.precision == "f32" else 2
        state_bytes = sum((3 * elt + 16) * n for n, t in zip(w.stage_numel(), w.staleness) if t >= 1)
        if args.adaptive_fused:
            # in one pass g_0 and V[0] are read once; V[1] is extra only where it is not a segment boundary
            kp = [plan.stage_effective_iters(j) for j in range(w.n_stages)]
            state_bytes = sum((16 + (0 if t // k == 1 else elt)) * n
                              for n, t, k in zip(w.stage_numel(), w.staleness, kp) if t >= 1)
            fused_extra = state_bytes
        step_bytes += state_bytes
        log(f"adaptive lambda: the lambda block adds {state_bytes} algorithmic bytes per step")

    accum = None
    if args.accumulate:
        ca = args.accumulate
        accum = torch.zeros(plan.flat_elems, dtype=torch.float32, device=dev)
        elt = 4 if w.precision == "f32" else 2
        per_arrival = sum((elt * (plan.stage_effective_iters(j) + 2) + 8) * n for j, n in enumerate(w.stage_numel()))
        last_extra = sum((elt + (8 if w.precision == "bf16" else 0)) * n for n in w.stage_numel())
        step_bytes = ca * per_arrival + last_extra
        log(f"accumulation: {ca} arrivals per step, algorithmic bytes per step {step_bytes}")

    def one_step():
        if args.accumulate:
            for k in range(args.accumulate):
                last = k == args.accumulate - 1
                B.ferret_accumulate_step(plan, st.ring, st.grads, st.master, accum, 1.0 / args.accumulate,
                                         [2 if last else 1] * w.n_stages, None, w.lam, w.lr,
                                         st.norms if norms else None, None, st.workspace if norms else None)
            st.commit()
            return
        if args.compensator in ("step-aware", "gap-aware"):
            gap = args.compensator == "gap-aware"
            B.ferret_penalized_step(plan, st.ring, st.grads, st.master, [1.0] * w.n_stages if gap else None,
                                    [1.0 / (w.lr * w.grad_std)] * w.n_stages if gap else None, w.lr,
                                    st.norms if norms else None, None, st.workspace if norms else None)
        elif args.adaptive:
            st.step_adaptive(0.9, 2e-6, w.lr, norms=norms, grad_out=False, fused=args.adaptive_fused)
        else:
            st.step(w.lam, w.lr, norms=norms, grad_out=False)
        st.commit()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    if args.graph:
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
        replays = max(args.steps // R, 1)
        args.steps = replays * R
        args.no_kernel_events = True
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(replays):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        log(f"graph of {R} steps replayed {replays} times")
    elif not args.no_kernel_events:
        B.ferret_profile_begin(args.steps * max(args.accumulate, 1))
    if not args.graph:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one_step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    n_launch = args.steps * max(args.accumulate, 1)
    kernel_ms = B.ferret_profile_end(n_launch) if not args.no_kernel_events else [elapsed * 1e3 / args.steps]

    ms_per_step = elapsed * 1e3 / args.steps

    # per-step spread: a second, untimed-for-`value` run of 50 steps with one event between steps
    # (step period = kernel(s) + launch gaps, as the device sees it)
    step_med_us = step_min_us = None
    if not args.graph:
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(51)]
        marks[0].record()
        for i in range(50):
            one_step()
            marks[i + 1].record()
        torch.cuda.synchronize()
        periods = [marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(50)]
        step_med_us, step_min_us = statistics.median(periods), min(periods)
    params_per_s = w.numel / (elapsed / args.steps)
    k_avg = statistics.fmean(kernel_ms)
    k_med = statistics.median(kernel_ms)
    per_launch_bytes = step_bytes / args.accumulate if args.accumulate else plan.step_bytes + fused_extra
    if args.compensator in ("step-aware", "gap-aware") or (args.compensator == "none" and norms):
        # V[0] is read besides V[tau] (for the gap, or for the weight-gap norm) in stages with staleness
        elt = 4 if w.precision == "f32" else 2
        per_launch_bytes += sum(elt * n for n, t in zip(w.stage_numel(), w.staleness) if t >= 1)
    achieved = per_launch_bytes / (k_avg * 1e-3) / 1e9     # the fused step kernel alone
    if step_med_us is not None:
        log(f"step period on the device over 50 further steps: median {step_med_us:.1f} us, min {step_min_us:.1f} us")
    log(f"step: {ms_per_step * 1e3:.1f} us wall per step; fused kernel avg {k_avg * 1e3:.1f} us, median "
        f"{k_med * 1e3:.1f} us, min {min(kernel_ms) * 1e3:.1f} us -> {achieved:.0f} GB/s algorithmic "
        f"({achieved / HBM_PEAK_GBS:.1%} of {HBM_PEAK_GBS:.0f} GB/s)")

    # context: plain copy through the library's copy kernel (read + write of the same byte count)
    n_copy = min(plan.ring_bytes // 2, 1 << 30) // 16 * 16
    src_t = st.ring.view(torch.uint8)[:n_copy]
    dst_t = st.ring.view(torch.uint8)[plan.ring_bytes - n_copy:] if plan.ring_bytes >= 2 * n_copy else torch.empty(n_copy, dtype=torch.uint8, device=dev)
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

    # context: the step's traffic shape without its arithmetic or tables -- per stage, a kernel that adds
    # NR read streams into one write stream, NR = that stage's read bytes / write bytes, sized so that the
    # bytes written match the stage's; the time of all stages together against the step's algorithmic bytes
    mix_gbs = None
    plain_shape = not args.accumulate and args.compensator == "iter-fisher" and not args.newest_from_master
    if plain_shape and not args.adaptive:
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

    # the committed counter summaries cover the default step of a workload and its one-pass adaptive variant
    plain = plain_shape and args.iters is None and norms
    traffic_key = None
    if plain and not args.adaptive:
        traffic_key = w.name
    elif plain and args.adaptive_fused:
        traffic_key = w.name + "_one_pass_lambda"
    result = {
        "metric": "compensated_params_per_sec",
        "value": params_per_s,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if w.precision == "f32" else "bf16 storage, f32 arithmetic",
        "data": "synthetic",
        "config": {"workload": w.name, "params": w.numel, "stages": w.n_stages, "staleness": w.staleness,
                   "ring_depth": w.ring_depth, "n_iters": w.n_iters, "lambda": w.lam, "lr": w.lr,
                   "norms": norms, "adaptive_lambda": ("one-pass" if args.adaptive_fused else bool(args.adaptive)), "accumulation_steps": args.accumulate, "hip_graph": bool(args.graph), "newest_from_master": bool(args.newest_from_master), "compensator": args.compensator,
                   "chunk_elems": plan.chunk_elems,
                   "algorithmic_bytes_per_step": step_bytes},
        "hbm_gbs_wall": step_bytes / (elapsed / args.steps) / 1e9,
        "step_median_us": step_med_us, "step_min_us": step_min_us,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(traffic_key),
                     "kernel": "ferret::step_kernel", "kernel_avg_us": k_avg * 1e3, "kernel_median_us": k_med * 1e3,
                     "copy_kernel_gbs": copy_gbs, "read_kernel_gbs": read_gbs, "mix_kernel_gbs": mix_gbs},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, host, plan)
        log("cpu baseline:", result["cpu_baseline"]["sample"])
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
