"""Estimation quality of the threshold estimators on synthetic gradient streams: how close the number of
selected elements khat comes to the target k = delta * d (the quantity of the paper's Fig. 1c and of its
quality criterion, eq. (12): within 20 % of k on average).

Every estimator runs on the same seeded stream with its own carried residual (error compensation, App. B.2):

  SIDCo-E / -GP / -P   the three chains of Sec. 2.4 under the stage controller of Algorithm 1
                       (delta_1 = 0.25, Q = 5, eps_H = eps_L = 0.2, starting from one stage)
  DGC                  threshold from Top-k of a 1 % random subset (Sec. 1, related work); reported is
                       what that threshold selects, before the trim to k
  Top-k                exact, khat = k by construction (listed for completeness)

Streams (generated on the device, torch generator seeded per iteration):
  iid         a fresh Laplace(1e-3) gradient every iteration (the iterated configuration of the benchmark)
  persistent  a fixed Laplace(1e-3) mean gradient plus fresh Laplace(1e-3) noise every iteration (a
              gradient direction that persists, as in training between learning-rate changes)

Run:  python -m paper_2101_10761_amd.quality [--d 25557032] [--iters 100] [--deltas 0.1,0.01,0.001]
Prints one table per stream and a JSON line with every number.
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np

SEED = 210110761 + 50


def laplace_(out, scale, gen):
    """Fills `out` with Laplace(0, scale) draws (inverse-CDF of a uniform)."""
    import torch
    out.uniform_(-0.5, 0.5, generator=gen)
    sign = torch.sign(out)
    out.abs_().mul_(-2.0).add_(1.0).clamp_(min=1e-30).log_().mul_(sign).mul_(-scale)
    return out


def run_stream(sidco, torch, stream_kind, d, delta, iters, warm, dev):
    k = delta * d
    cap = sidco.sidco_out_capacity(d, delta)
    out_idx = torch.empty(cap, dtype=torch.int32, device=dev)
    out_val = torch.empty(cap, dtype=torch.float32, device=dev)
    out_count = torch.zeros(1, dtype=torch.int32, device=dev)
    out_eta = torch.zeros(1, dtype=torch.float32, device=dev)
    names = ["SIDCo-E", "SIDCo-GP", "SIDCo-P", "DGC", "Top-k"]
    dists = {"SIDCo-E": sidco.DIST_EXP, "SIDCo-GP": sidco.DIST_GAMMA_GPD, "SIDCo-P": sidco.DIST_GPD}
    ratio = {n: [] for n in names}
    stages = {n: [] for n in dists}
    gen = torch.Generator(device=dev)
    g = torch.empty(d, dtype=torch.float32, device=dev)
    res = torch.empty(d, dtype=torch.float32, device=dev)
    mean = None
    if stream_kind == "persistent":
        gen.manual_seed(SEED - 1)
        mean = laplace_(torch.empty(d, dtype=torch.float32, device=dev), 1e-3, gen)
    kk = sidco.sidco_dgc_sizes(d, delta, 0.01)[2]
    t_idx = torch.empty(kk, dtype=torch.int32, device=dev)
    t_val = torch.empty(kk, dtype=torch.float32, device=dev)
    # one estimator at a time over the whole stream (a controller's count lives on the device and other calls
    # in between would disturb it); the stream is seeded per iteration, so every estimator sees the same one
    for n in names:
        res.zero_()
        ctrl = sidco.Controller(delta, dists[n], stages=1) if n in dists else None
        for it in range(iters):
            gen.manual_seed(SEED + it)
            laplace_(g, 1e-3, gen)
            if mean is not None:
                g.add_(mean)
            if ctrl is not None:
                stages[n].append(ctrl.stages)
                ctrl.compress(g, res, out_idx, out_val, out_count, out_eta)
                ratio[n].append(int(out_count.item()) / k)
            elif n == "DGC":
                sidco.sidco_dgc(g, res, delta, 0.01, SEED + it, t_idx, t_val, out_count, out_eta)
                ratio[n].append(sidco.sidco_dgc_result()[2] / k)
            else:
                sidco.sidco_topk(g, res, kk, t_idx, t_val, out_count, out_eta)
                ratio[n].append(int(out_count.item()) / k)
        if ctrl is not None:
            ctrl.close()
    rows = {}
    for n in names:
        r = np.array(ratio[n][warm:])
        rows[n] = {
            "mean_khat_over_k": round(float(r.mean()), 4),
            "within_20pct": round(float(np.mean(np.abs(r - 1.0) <= 0.2)), 3),
            "min": round(float(r.min()), 4), "max": round(float(r.max()), 4),
        }
        if n in stages:
            rows[n]["stages_last"] = stages[n][-1]
            rows[n]["stages_mean"] = round(float(np.mean(stages[n][warm:])), 2)
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--d", type=int, default=25_557_032)
    ap.add_argument("--iters", type=int, default=100)
    ap.add_argument("--warm", type=int, default=30, help="iterations left out of the averages")
    ap.add_argument("--deltas", default="0.1,0.01,0.001")
    ap.add_argument("--streams", default="iid,persistent")
    args = ap.parse_args()

    import torch
    import paper_2101_10761_amd as sidco

    sidco.load()
    if not torch.cuda.is_available():
        print("quality.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    out = {}
    for kind in args.streams.split(","):
        out[kind] = {}
        for delta in (float(x) for x in args.deltas.split(",")):
            rows = run_stream(sidco, torch, kind, args.d, delta, args.iters, args.warm, dev)
            out[kind][str(delta)] = rows
            print(f"\nstream {kind}, d = {args.d}, delta = {delta}, iterations {args.warm}..{args.iters - 1}",
                  file=sys.stderr)
            print(f"{'estimator':10s} {'mean khat/k':>12s} {'within 20 %':>12s} {'min':>8s} {'max':>8s} {'stages':>8s}",
                  file=sys.stderr)
            for n, r in rows.items():
                st = f"{r['stages_mean']:.1f}" if "stages_mean" in r else "-"
                print(f"{n:10s} {r['mean_khat_over_k']:12.4f} {r['within_20pct']:12.3f} {r['min']:8.3f} "
                      f"{r['max']:8.3f} {st:>8s}", file=sys.stderr, flush=True)
    print(json.dumps({"d": args.d, "iters": args.iters, "warm": args.warm, "results": out}), flush=True)


if __name__ == "__main__":
    main()
