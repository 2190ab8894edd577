#!/usr/bin/env python3
"""Benchmark of the SIDCo sparsifier on one MI355X.

A step is one pass of the whole hot path (error-compensation add, stage-1 fit, threshold refinement,
final compaction and residual update = one sidco_compress call) over one synthetic gradient that is
already resident in HBM.  The default workload is the configuration the headline metric is quoted on:
d = 25,557,032 fp32, Student-t(3) values, delta = 0.001, three generalized-Pareto stages, error feedback.

Several (gradient, residual) buffer pairs - more data than the 256 MB memory-side cache holds - are used in
rotation, as if that many workers took turns on the GPU: every step reads its gradient AND its carried
residual from HBM, as a training step does whose forward and backward passes have flushed the caches since
the previous compression.  Each pair carries its own residual from one of its steps to the next.
(`--residual-buffers 1` keeps one residual for all steps: it then stays in the memory-side cache between
steps and the first pass runs about a quarter faster - a figure that no training loop would see.)

Config 5 (`--workload cfg5`, or `--fresh-gradients` with any workload) follows its own definition instead:
ONE worker's consecutive iterations, a fresh i.i.d. gradient every step (a pool of distinct gradients drawn on
the device, used in turn) added to ONE carried residual; `--delta` selects the ratio (0.1, 0.01, 0.001).

Timing: the headline figure is the wall clock over exactly `--steps` calls between two device
synchronisations.  Beside it, `--timed-calls` further calls are timed one by one with HIP events on the call's
stream (median and minimum), and, with `--reset-residual`, once more with every pair's residual restored
(untimed) before each call, so that every call sees the configuration's own first-iteration distribution.

Prints ONE JSON line on stdout; everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0       # MI355X published HBM3E peak
ROTATE_BYTES = 768 << 20     # distinct gradient data kept in rotation (> memory-side cache)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def make_workload(name: str, d: int = 0):
    from paper_2101_10761_amd import workloads
    table = {
        "cfg1": workloads.config1, "cfg2": workloads.config2, "cfg3": workloads.config3,
        "cfg4": workloads.config4, "cfg5": workloads.config5,
    }
    return table[name](d) if d > 0 else table[name]()


def scope_formula_bytes(d, ec, n_stage, khat, fit_bpe=None):
    """The scope table's byte count of a call: gradient (+ residual read and acc write), the second pass over
    acc, every stage's exceedances written once and read once as 8-byte pairs, output pairs and residual
    zero-stores.  fit_bpe: bytes per element of the first pass when the gradient is not fp32."""
    b = d * (fit_bpe if fit_bpe is not None else 4 * (3 if ec else 1)) + 4 * d
    b += sum(16 * int(n) for n in n_stage[1:])
    b += 12 * khat
    return b


def moved_bytes_min(d, ec, n_stage, khat, fit_bpe=None):
    """The least this design can move in a call: the first pass, ONE further pass over the accumulated vector
    (whatever the number of stages: the dense stage only sums over the exceedances of eta_1 and writes
    candidates for the stage after it), the lists behind the dense stage - candidates that must at least hold
    the next stage's exceedances, then each later stage's exceedances, all written once and read once - and the
    output.  The exceedances of eta_1 are never written, so they are not counted."""
    b = d * (fit_bpe if fit_bpe is not None else 4 * (3 if ec else 1)) + 4 * d
    M = len(n_stage)
    if M >= 2:
        after = [int(n) for n in n_stage[2:]] + [khat]      # what stages 2..M leave: n_3 .. n_M, khat
        b += 16 * after[0]                                    # the dense stage's candidate lists
        b += sum(16 * a for a in after[:-1])                  # exceedance lists written by the list stages
    b += 12 * khat
    return b


def timing_summary(ms_list):
    a = np.asarray(ms_list, dtype=np.float64) * 1e3
    return {"calls": int(a.size), "median_us": round(float(np.median(a)), 2), "min_us": round(float(a.min()), 2),
            "mean_us": round(float(a.mean()), 2), "max_us": round(float(a.max()), 2)}


# ---- CPU baseline: the oracle as it stands, on one core and on all of them (one process per core, each on
# its own slice of the vector: the data-parallel use the paper describes, every worker compressing its own
# gradient).  Runs before anything touches the GPU: the worker processes are forked.
_CPU_ARGS = None


def _cpu_slice(bounds):
    import oracle
    w, oratios = _CPU_ARGS
    a, b = bounds
    rs = None if w.residual is None else np.ascontiguousarray(w.residual[a:b])
    tc = time.perf_counter()
    oracle.compress(np.ascontiguousarray(w.grad[a:b]), rs, ratios=oratios, dist=w.dist)
    return time.perf_counter() - tc


def cpu_baseline_legs(w, budget_s):
    global _CPU_ARGS
    import multiprocessing as mp
    import oracle
    oracle.build()
    oratios = oracle.schedule(w.delta, w.stages, w.delta1)
    d = w.d
    cores_host = os.cpu_count() or 1
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = cores_host
    workers = max(1, min(usable, 16))      # the share of a one-GPU machine, whatever the host shows
    _CPU_ARGS = (w, oratios)
    # one core: the whole vector, median of at least 5 runs
    t1 = []
    t_used = 0.0
    while len(t1) < 5 or (t_used < 0.4 * budget_s and len(t1) < 15):
        t = _cpu_slice((0, d))
        t1.append(t)
        t_used += t
    single = d / float(np.median(t1)) / 1e9
    # all cores: `workers` processes, each on its own d / workers slice, timed until the last one is done
    bounds = [(d * i // workers, d * (i + 1) // workers) for i in range(workers)]
    tall = []
    with mp.get_context("fork").Pool(workers) as pool:
        pool.map(_cpu_slice, bounds)       # warm-up: page the slices in, load the library
        t_used = 0.0
        while len(tall) < 5 or (t_used < 0.4 * budget_s and len(tall) < 15):
            tc = time.perf_counter()
            pool.map(_cpu_slice, bounds)
            tall.append(time.perf_counter() - tc)
            t_used += tall[-1]
    multi = d / float(np.median(tall)) / 1e9
    _CPU_ARGS = None
    return {
        "value": round(single, 5), "unit": "G elem/s", "cores": 1, "kind": "oracle",
        "sample": f"the workload's whole vector ({d} elements), first iteration's input, median of {len(t1)} runs "
                  f"({float(np.median(t1)):.3f} s each), single thread, fp64 plain C",
        "all_cores": {"value": round(multi, 5), "unit": "G elem/s", "cores": workers,
                      "sample": f"{workers} processes, each compressing its own {d // workers}-element slice of the same "
                                f"vector (one worker per core), median of {len(tall)} runs "
                                f"({float(np.median(tall)):.3f} s until the last one finishes)"},
        "cores_host": cores_host, "cores_usable": usable,
    }


def laplace_(out, scale, gen):
    """Fills `out` (a CUDA tensor) with Laplace(0, scale) draws: inverse CDF of a uniform."""
    import torch
    out.uniform_(-0.5, 0.5, generator=gen)
    sign = torch.sign(out)
    out.abs_().mul_(-2.0).add_(1.0).clamp_(min=1e-30).log_().mul_(sign).mul_(-scale)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg3", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--d", type=int, default=0, help="length of the vector, if not the workload's own (size sweeps)")
    ap.add_argument("--delta", type=float, default=0.0, help="target ratio, if not the workload's own (cfg5: 0.1, 0.01, 0.001)")
    ap.add_argument("--fresh-gradients", action="store_true",
                    help="a fresh i.i.d. gradient every step on ONE carried residual (always on for cfg5)")
    ap.add_argument("--timed-calls", type=int, default=60, help="calls timed one by one with HIP events (median, min)")
    ap.add_argument("--reset-residual", action="store_true",
                    help="also time calls whose residual is restored, untimed, before each of them")
    ap.add_argument("--profile-steps", type=int, default=50, help="steps timed kernel by kernel with HIP events")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the CPU-oracle baseline (both legs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-topk", action="store_true", help="skip the exact Top-k comparator leg")
    ap.add_argument("--no-dgc", action="store_true", help="skip the DGC comparator leg")
    ap.add_argument("--no-ceiling", action="store_true", help="skip the plain-kernel streaming ceiling leg")
    ap.add_argument("--graph", action="store_true",
                    help="also time the steps replayed from HIP graphs (one per buffer pair)")
    ap.add_argument("--residual-buffers", type=int, default=0,
                    help="carried residuals in rotation (0 = as many as gradient buffers; 1 = a single residual "
                         "that stays cache-resident between steps)")
    ap.add_argument("--grad-dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="element type of the gradient buffer (the residual and all arithmetic stay fp32/fp64); "
                         "16-bit gradients use the default stage schedule (delta_1 = 0.25) and skip the comparators")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (the sparsifier is local to a worker: no collectives, "
            "no sharding); --gpus must be 1")
        sys.exit(2)

    t0 = time.time()
    w = make_workload(args.workload, args.d)
    if args.delta > 0.0:
        w.delta = args.delta
    d = w.d
    fresh = args.fresh_gradients or args.workload == "cfg5"
    log(f"workload {w.name}: d={d} delta={w.delta} dist={w.dist} stages={w.stages} delta1={w.delta1} "
        f"(generated in {time.time() - t0:.1f}s){' fresh gradient every step, one carried residual' if fresh else ''}")

    # the CPU legs fork worker processes: before anything touches the GPU
    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = cpu_baseline_legs(w, args.cpu_seconds)
        log(f"cpu oracle: {cpu_baseline['value']} G elem/s on 1 core; {cpu_baseline['all_cores']['value']} G elem/s on "
            f"{cpu_baseline['all_cores']['cores']} cores (host has {cpu_baseline['cores_host']})")

    import torch
    import paper_2101_10761_amd as sidco

    sidco.load()  # fails loudly when the HIP library has not been built
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    ratios = sidco.sidco_stage_ratios(w.delta, w.stages, w.delta1)
    g0 = torch.from_numpy(w.grad).to(dev)
    typed = args.grad_dtype != "f32"
    gbytes = 2 if typed else 4
    if typed:
        if w.delta1 != 0.25:
            log("bench.py: --grad-dtype f16/bf16 needs a workload with delta_1 = 0.25")
            sys.exit(2)
        g0 = g0.to(torch.float16 if args.grad_dtype == "f16" else torch.bfloat16)
        args.no_topk = args.no_dgc = True
    ec = w.residual is not None
    if fresh:
        # ONE worker's consecutive iterations: a pool of distinct i.i.d. gradients of the workload's law (config 5:
        # Laplace(1e-3)), drawn on the device and used in turn, all added to ONE carried residual.  The pool is
        # larger than the memory-side cache many times over, so every gradient comes from HBM; the residual is
        # the one a training loop would carry.
        pool_bytes = 48 << 30
        nbuf = int(max(4, min(args.steps + args.warmup + args.timed_calls, pool_bytes // (gbytes * d), 128)))
        gen = torch.Generator(device=dev)
        grads = [g0]
        scale = 1e-3
        for i in range(1, nbuf):
            gen.manual_seed(210110761 + 5 + 1000 * (i + 1))
            gi = laplace_(torch.empty(d, dtype=torch.float32, device=dev), scale, gen)
            grads.append(gi if not typed else gi.to(g0.dtype))
        nres = 1
    else:
        nbuf = max(2, min(16, ROTATE_BYTES // (4 * d) + 1))
        # The same gradient in several buffers: every step reads its gradient from another address range, and the
        # carried residual reaches a steady state the way it does under a persistent gradient direction (an entry
        # grows until it is selected and starts over), instead of turning Gaussian as it would under a stream of
        # independent draws that are hardly ever selected.
        grads = [g0] + [g0.clone() for _ in range(nbuf - 1)]
        nres = nbuf if args.residual_buffers <= 0 else min(args.residual_buffers, nbuf)

    def fresh_residuals():
        if not ec:
            return [None] * nres
        r0 = torch.from_numpy(w.residual).to(dev)
        return [r0] + [r0.clone() for _ in range(nres - 1)]

    residuals = fresh_residuals()
    cap = max(sidco.sidco_out_capacity(d, w.delta), 1)
    out_idx = torch.empty(cap, dtype=torch.int32, device=dev)
    out_val = torch.empty(cap, dtype=torch.float32, device=dev)
    # every step reports its count and threshold into a slot of its own: the trajectory costs nothing
    n_slots = args.warmup + args.steps + args.timed_calls * (2 if args.reset_residual else 1) + args.profile_steps + 8
    counts = torch.zeros(n_slots, dtype=torch.int32, device=dev)
    etas = torch.zeros(n_slots, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()
    sidco.sidco_reserve(sidco.sidco_workspace_bytes_typed(d, {"f32": 0, "f16": 1, "bf16": 2}[args.grad_dtype], ec),
                        stream=stream)

    def step(i, slot=None):
        slot = i if slot is None else slot
        oc, oe = counts[slot:slot + 1], etas[slot:slot + 1]
        if typed:
            sidco.sidco_compress_typed(grads[i % nbuf], residuals[i % nres], w.delta, w.dist, w.stages, out_idx, out_val,
                                       oc, oe, stream=stream)
        else:
            sidco.sidco_compress_ex(grads[i % nbuf], residuals[i % nres], w.dist, ratios, out_idx, out_val, oc, oe,
                                    stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    ms_per_step = (t_end - t_start) * 1e3 / args.steps
    value = d / (ms_per_step * 1e-3) / 1e9
    n_done = args.warmup + args.steps
    traj = (counts[:n_done].cpu().numpy().astype(np.float64) / (w.delta * d))
    log(f"timed {args.steps} steps: {ms_per_step * 1e3:.1f} us/step -> {value:.1f} G elem/s; khat/k over the timed "
        f"steps: mean {traj[args.warmup:].mean():.4f}, first step {traj[0]:.4f}, last {traj[-1]:.4f}")

    # the same calls one by one between two HIP events on the call's stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.timed_calls, 1))]
    timing = {"wall_clock_loop": {"calls": args.steps, "mean_us": round(ms_per_step * 1e3, 2)}}
    if args.timed_calls > 0:
        for j in range(args.timed_calls):
            ev[j][0].record(stream)
            step(n_done + j)
            ev[j][1].record(stream)
        torch.cuda.synchronize()
        timing["per_call_events"] = timing_summary([a.elapsed_time(b) for a, b in ev[:args.timed_calls]])
        n_done += args.timed_calls
        log(f"per-call HIP events: {timing['per_call_events']}")
        if args.reset_residual and ec:
            pristine = torch.from_numpy(w.residual).to(dev)
            for j in range(args.timed_calls):
                residuals[(n_done + j) % nres].copy_(pristine)      # untimed
                ev[j][0].record(stream)
                step(n_done + j)
                ev[j][1].record(stream)
            torch.cuda.synchronize()
            timing["per_call_events_residual_reset"] = timing_summary([a.elapsed_time(b) for a, b in ev[:args.timed_calls]])
            rr = counts[n_done:n_done + args.timed_calls].cpu().numpy().astype(np.float64) / (w.delta * d)
            timing["per_call_events_residual_reset"]["khat_over_k_mean"] = round(float(rr.mean()), 4)
            n_done += args.timed_calls
            log(f"per-call HIP events, residual restored before each call: {timing['per_call_events_residual_reset']}")
            del pristine

    # kernel-by-kernel timing with HIP events on the same stream
    sidco.sidco_set_profiling(True)
    per_kernel: dict[str, list[float]] = {}
    order: list[str] = []
    n_stage = None
    khat = []
    for i in range(args.profile_steps):
        step(n_done + i, slot=n_slots - 1)
        prof = sidco.sidco_get_profile()
        seen: dict[str, int] = {}
        for name, ms in prof:
            seen[name] = seen.get(name, 0) + 1
            key = name if seen[name] == 1 else f"{name}#{seen[name]}"
            if key not in per_kernel:
                per_kernel[key] = []
                order.append(key)
            per_kernel[key].append(ms)
        diag = sidco.sidco_read_diag(stream)
        n_stage = [diag.n[m] for m in range(diag.stages)]
        khat.append(diag.count)
    sidco.sidco_set_profiling(False)
    n_done += args.profile_steps
    kern_us = {k: float(np.median(v)) * 1e3 for k, v in per_kernel.items()}
    log("per-kernel median (HIP events, each figure includes the events' own dispatch): " +
        ", ".join(f"{k} {kern_us[k]:.1f} us" for k in order))
    if not khat:   # no profiled steps asked for: take the diagnostics of the last timed step
        diag = sidco.sidco_read_diag(stream)
        n_stage = [diag.n[m] for m in range(diag.stages)]
        khat.append(diag.count)
    log(f"last step: n per stage {n_stage}, khat {khat[-1]} (target {w.delta * d:.0f})")

    # Dominant kernel on its own: batches of back-to-back k_fit launches (sidco_fit) between two HIP
    # events on the same stream, so that the events' own dispatch latency (several microseconds, which
    # the in-sequence figures above include) is spread over the batch.  Every launch of a batch gets its own
    # copy of the carried residual (restored, untimed, before each batch), so that each one sees the
    # values of a real step rather than a residual that has already absorbed the gradient several times.
    batch, fit_ms = (20 if d < 100_000_000 else 8), []
    ev_a, ev_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    residual = residuals[n_done % nres]          # the residual the next step would use
    scratch_res = [residual.clone() for _ in range(batch)] if ec else [None] * batch
    for rep in range(12):
        if ec:
            for sr in scratch_res:
                sr.copy_(residual)
        torch.cuda.synchronize()
        ev_a.record(stream)
        for i in range(batch):
            sidco.sidco_fit(grads[(rep * batch + i) % nbuf], scratch_res[i], w.dist, stream=stream)
        ev_b.record(stream)
        ev_b.synchronize()
        if rep >= 2:
            fit_ms.append(ev_a.elapsed_time(ev_b) / batch)
    del scratch_res
    fit_bpe = gbytes + (8 if ec else (4 if typed else 0))   # read g [, read r], write acc unless acc is g itself
    fit_bytes = fit_bpe * d
    fit_us = float(np.mean(fit_ms)) * 1e3
    log(f"k_fit alone: {fit_us:.1f} us per launch "
        f"(HIP events around batches of {batch})")
    achieved = fit_bytes / (fit_us * 1e-6) / 1e9
    traffic, counters = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath) and not typed and args.d == 0:
        try:
            counters = json.load(open(tpath)).get(args.workload)
            traffic = (counters or {}).get("k_fit")
        except Exception:
            traffic, counters = None, None
    roofline = {
        "kernel": "k_fit (first pass; from 12 M elements k_fit_flat + k_fit_reduce)", "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic,
        "traffic_source": None if traffic is None else "from profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE of an "
                          "earlier run of this workload, scaled by a device copy of known size); not measured in this run",
        "bytes_per_elem": fit_bpe, "elems_per_launch": d, "avg_launch_us": round(fit_us, 2),
    }
    khat_mean = int(np.mean(khat))
    moved = moved_bytes_min(d, ec, n_stage, khat_mean, fit_bpe)
    formula = scope_formula_bytes(d, ec, n_stage, khat_mean, fit_bpe)
    secs = ms_per_step * 1e-3
    path = {
        "bytes_moved_min": moved, "bytes_per_elem": round(moved / d, 2),
        "achieved": round(moved / secs / 1e9, 1), "unit": "GB/s",
        "frac": round(moved / secs / 1e9 / HBM_PEAK_GBPS, 4),
        "note": "frac prices the step against the bytes this design must move (the exceedances of eta_1 are never "
                "written as pairs); frac_scope_formula prices it against the scope table's formula, which charges them",
        "scope_formula_bytes": formula, "frac_scope_formula": round(formula / secs / 1e9 / HBM_PEAK_GBPS, 4),
        "counter_bytes": None if not counters else {k: v for k, v in counters.items()},
        "counter_source": None if not counters else "profiles/hbm_traffic.json, not measured in this run",
        "kernels_us": {k: round(kern_us[k], 2) for k in order},
    }

    # The same steps replayed from HIP graphs (one graph per buffer pair, captured through torch): what a
    # launch-bound loop gains when the host only issues one graph launch per step.
    graph_leg = None
    if args.graph:
        side = torch.cuda.Stream()
        sidco.sidco_reserve(sidco.sidco_workspace_bytes_typed(d, {"f32": 0, "f16": 1, "bf16": 2}[args.grad_dtype], ec),
                            stream=side)   # the capturing stream's workspace: allocated outside the capture
        side.wait_stream(stream)
        graphs = []
        with torch.cuda.stream(side):
            for i in range(min(nbuf, 16)):
                gph = torch.cuda.CUDAGraph()
                gph.capture_begin()
                oc, oe = counts[n_slots - 2:n_slots - 1], etas[n_slots - 2:n_slots - 1]
                if typed:
                    sidco.sidco_compress_typed(grads[i % nbuf], residuals[i % nres], w.delta, w.dist, w.stages, out_idx,
                                               out_val, oc, oe, stream=side)
                else:
                    sidco.sidco_compress_ex(grads[i % nbuf], residuals[i % nres], w.dist, ratios, out_idx, out_val,
                                            oc, oe, stream=side)
                gph.capture_end()
                graphs.append(gph)
        stream.wait_stream(side)
        torch.cuda.synchronize()
        for i in range(args.warmup):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for i in range(args.steps):
            graphs[(args.warmup + i) % len(graphs)].replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - tg) * 1e3 / args.steps
        graph_leg = {"ms_per_step": round(g_ms, 5), "value": round(d / (g_ms * 1e-3) / 1e9, 2), "unit": "G elem/s",
                     "graphs": len(graphs), "eager_ms_per_step": round(ms_per_step, 5)}
        log(f"graph replay: {g_ms * 1e3:.1f} us/step ({graph_leg['value']} G elem/s) against {ms_per_step * 1e3:.1f} us eager")

    # What this machine streams with nothing of ours in the way: torch's own in-place add (two reads and one
    # write per element, the traffic of k_fit) and device copy (one read, one write) over the same rotating
    # buffers.  The first pass cannot be faster than the first of these.
    ceiling = None
    if ec and not typed and not args.no_ceiling:
        scratch = fresh_residuals()
        ceiling = {}
        for name, bpe, fn in (("add_inplace_2r1w", 12, lambda i: scratch[i % nres].add_(grads[i % nbuf])),
                              ("copy_1r1w", 8, lambda i: scratch[i % nres].copy_(grads[i % nbuf]))):
            for i in range(8):
                fn(i)
            torch.cuda.synchronize()
            ev_a.record(stream)
            for i in range(48):
                fn(8 + i)
            ev_b.record(stream)
            ev_b.synchronize()
            us = ev_a.elapsed_time(ev_b) / 48 * 1e3
            ceiling[name] = {"us": round(us, 2), "GBps": round(bpe * d / (us * 1e-6) / 1e9, 1),
                             "frac_of_peak": round(bpe * d / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
        del scratch
        log(f"streaming ceiling (torch kernels, same buffers): {ceiling}")

    # Comparator: exact Top-k (radix select) with k = ceil(delta d) on the same gradients, same buffer rotation,
    # own carried residual (the paper's micro-benchmarks normalise every compressor by Top-k's time)
    topk = None
    if not args.no_topk:
        k = int(np.ceil(w.delta * d))
        t_idx = torch.empty(k, dtype=torch.int32, device=dev)
        t_val = torch.empty(k, dtype=torch.float32, device=dev)
        t_cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        t_kth = torch.zeros(1, dtype=torch.float32, device=dev)
        t_res = fresh_residuals()
        n_topk = max(1, min(args.steps, 100))
        for i in range(10):
            sidco.sidco_topk(grads[i % nbuf], t_res[i % nres], k, t_idx, t_val, t_cnt, t_kth, stream=stream)
        torch.cuda.synchronize()
        tt = time.perf_counter()
        for i in range(n_topk):
            sidco.sidco_topk(grads[(10 + i) % nbuf], t_res[(10 + i) % nres], k, t_idx, t_val, t_cnt, t_kth, stream=stream)
        torch.cuda.synchronize()
        topk_ms = (time.perf_counter() - tt) * 1e3 / n_topk
        topk = {
            "kind": "exact Top-k, radix select on magnitude bits (own HIP kernels)", "k": k, "steps": n_topk,
            "ms_per_step": round(topk_ms, 5), "value": round(d / (topk_ms * 1e-3) / 1e9, 2), "unit": "G elem/s",
            "sidco_speedup_over_topk": round(topk_ms / ms_per_step, 3),
            "kth_magnitude": float(t_kth.item()), "sidco_eta": float(etas[n_slots - 1].item()),
        }
        log(f"top-k comparator (k={k}): {topk_ms * 1e3:.1f} us/step -> {topk['value']} G elem/s; "
            f"SIDCo is {topk['sidco_speedup_over_topk']}x faster")

    # Comparator: DGC's sampling threshold (1 % subset, fresh seed every step) on the same gradients, own carried
    # residual; reports its time and how close the threshold's own selection comes to k (before the trim)
    dgc = None
    if not args.no_dgc:
        rho = 0.01
        n_s, k_s, k = sidco.sidco_dgc_sizes(d, w.delta, rho)
        g_idx = torch.empty(k, dtype=torch.int32, device=dev)
        g_val = torch.empty(k, dtype=torch.float32, device=dev)
        g_cnt = torch.zeros(1, dtype=torch.int32, device=dev)
        g_eta = torch.zeros(1, dtype=torch.float32, device=dev)
        g_res = fresh_residuals()
        n_dgc = max(1, min(args.steps, 100))
        for i in range(10):
            sidco.sidco_dgc(grads[i % nbuf], g_res[i % nres], w.delta, rho, i, g_idx, g_val, g_cnt, g_eta, stream=stream)
        torch.cuda.synchronize()
        tt = time.perf_counter()
        for i in range(n_dgc):
            sidco.sidco_dgc(grads[(10 + i) % nbuf], g_res[(10 + i) % nres], w.delta, rho, 10 + i, g_idx, g_val, g_cnt, g_eta,
                            stream=stream)
        torch.cuda.synchronize()
        dgc_ms = (time.perf_counter() - tt) * 1e3 / n_dgc
        firsts = []
        sidco.sidco_set_profiling(True)
        dgc_kern: dict[str, list[float]] = {}
        for i in range(min(args.profile_steps, 20)):
            sidco.sidco_dgc(grads[i % nbuf], g_res[i % nres], w.delta, rho, 1000 + i, g_idx, g_val, g_cnt, g_eta, stream=stream)
            for name, ms in sidco.sidco_get_profile():
                dgc_kern.setdefault(name, []).append(ms)
            firsts.append(sidco.sidco_dgc_result(stream)[2] / k)
        sidco.sidco_set_profiling(False)
        dgc = {
            "kind": "DGC sampling threshold: radix select on a 1 % subset, one pass, trim to k by a second select "
                    "(own HIP kernels)",
            "sample_ratio": rho, "n_sample": n_s, "k_sample": k_s, "k": k, "steps": n_dgc,
            "ms_per_step": round(dgc_ms, 5), "value": round(d / (dgc_ms * 1e-3) / 1e9, 2), "unit": "G elem/s",
            "sidco_speedup_over_dgc": round(dgc_ms / ms_per_step, 3),
            "first_pass_over_k": {"mean": round(float(np.mean(firsts)), 4), "min": round(float(np.min(firsts)), 4),
                                  "max": round(float(np.max(firsts)), 4)} if firsts else None,
            "kernels_us": {n: round(float(np.mean(v)) * 1e3, 2) for n, v in dgc_kern.items()},
        }
        log(f"DGC comparator (n_s={n_s}, k={k}): {dgc_ms * 1e3:.1f} us/step -> {dgc['value']} G elem/s; "
            f"first-pass count / k = {dgc['first_pass_over_k']}")

    # Layer-wise mode of a multi-tensor vector: every tensor sparsified on its own, (i) all tensors in one
    # batched launch sequence, (ii) one call per tensor
    per_tensor = None
    if w.tensor_offsets is not None:
        offs = [int(x) for x in w.tensor_offsets]
        nt = len(offs) - 1
        o_offs = sidco.sidco_batched_out_offsets(offs, w.delta)
        b_idx = torch.empty(o_offs[-1], dtype=torch.int32, device=dev)
        b_val = torch.empty(o_offs[-1], dtype=torch.float32, device=dev)
        b_cnt = torch.zeros(nt, dtype=torch.int32, device=dev)
        b_eta = torch.zeros(nt, dtype=torch.float32, device=dev)
        b_res = fresh_residuals()
        n_b = max(1, min(args.steps, 100))

        def batched(i):
            sidco.sidco_compress_batched(grads[i % nbuf], b_res[i % nres], offs, w.delta, w.dist, w.stages, b_idx, b_val, o_offs,
                                         b_cnt, b_eta, stream=stream)

        def looped(i):
            g = grads[i % nbuf]
            br = b_res[i % nres]
            for t in range(nt):
                a, b = offs[t], offs[t + 1]
                sidco.sidco_compress(g[a:b], None if br is None else br[a:b], w.delta, w.dist, w.stages,
                                     b_idx[o_offs[t]:o_offs[t + 1]], b_val[o_offs[t]:o_offs[t + 1]], b_cnt[t:t + 1],
                                     b_eta[t:t + 1], stream=stream)

        times = {}
        for name, fn, reps in (("batched", batched, n_b), ("one_call_per_tensor", looped, max(1, n_b // 5))):
            for i in range(5):
                fn(i)
            torch.cuda.synchronize()
            tt = time.perf_counter()
            for i in range(reps):
                fn(5 + i)
            torch.cuda.synchronize()
            times[name] = (time.perf_counter() - tt) * 1e3 / reps
        per_tensor = {
            "tensors": nt, "batched_ms_per_step": round(times["batched"], 5),
            "batched_value": round(d / (times["batched"] * 1e-3) / 1e9, 2),
            "one_call_per_tensor_ms_per_step": round(times["one_call_per_tensor"], 5),
            "whole_vector_ms_per_step": round(ms_per_step, 5), "unit": "G elem/s",
            "selected_total_batched": int(b_cnt.sum().item()),
        }
        log(f"per-tensor mode ({nt} tensors): batched {times['batched'] * 1e3:.1f} us/step "
            f"({per_tensor['batched_value']} G elem/s), one call per tensor {times['one_call_per_tensor'] * 1e3:.1f} us/step, "
            f"whole vector {ms_per_step * 1e3:.1f} us/step")

    result = {
        "metric": "G gradient elems/s compressed (d=25.6M fp32, delta=0.001)" if args.workload == "cfg3" and not typed and args.delta == 0.0 and args.d == 0
                  else f"G gradient elems/s compressed ({args.workload}, d={d}, delta={w.delta}" + (f", {args.grad_dtype} gradient)" if typed else ")"),
        "value": round(value, 2), "unit": "G elem/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": f"{w.name}: d={d} {'fp32' if not typed else args.grad_dtype + ' gradient, fp32 residual'}, delta={w.delta}, dist={['exp', 'gamma-gpd', 'gpd'][w.dist]}, "
                        f"stages={w.stages}, delta1={w.delta1}, error_feedback={'on' if ec else 'off'}",
            "gradients": ("pool of distinct i.i.d. gradients drawn on the device, used in turn" if fresh else
                          "the workload's seeded gradient in several buffers, used in rotation"),
            "gradient_buffers_in_rotation": nbuf, "residual_buffers_in_rotation": nres,
            "khat_over_k": round(float(traj[args.warmup:].mean()), 4),
        },
        "khat_over_k_trajectory": {"first_steps": [round(float(x), 4) for x in traj[:12]],
                                   "timed_mean": round(float(traj[args.warmup:].mean()), 4),
                                   "timed_min": round(float(traj[args.warmup:].min()), 4),
                                   "timed_max": round(float(traj[args.warmup:].max()), 4),
                                   "last": round(float(traj[-1]), 4)},
        "timing": timing,
        "roofline": roofline, "path": path, "streaming_ceiling": ceiling, "graph_replay": graph_leg,
        "cpu_baseline": cpu_baseline,
        "topk_comparator": topk,
        "dgc_comparator": dgc, "per_tensor": per_tensor,
        "paper_context": "the paper prints no absolute compression rate in text (its figures are the only source); it "
                         "states that on a V100 (PyTorch 1.1, CUDA 10.2) every threshold estimator is far faster than "
                         "Top-k and that SIDCo compresses at least 2x faster than DGC (Sec. 4.2, App. E)",
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
