"""GPU parity on seeded random cases: lengths, laws, stage schedules, offsets, element types, single and batched
calls and both comparators drawn at random, each checked against the oracle like the hand-picked cases.  Repeated
calls on a carried residual exercise the threshold hints between calls of one shape and their reset between shapes."""
import numpy as np
import pytest

from gpu_harness import check_parity, run_gpu
from test_gpu_batched import check_batched, run_batched
from test_gpu_dgc import check_dgc, run_dgc
from test_gpu_topk import check_topk, run_topk

pytestmark = pytest.mark.gpu


def _draw(rng, d, kind):
    if kind == 0:
        return rng.laplace(0, 1e-3, d).astype(np.float32)
    if kind == 1:
        return (rng.standard_t(3.0, d) * 1e-3).astype(np.float32)
    if kind == 2:
        return (rng.standard_normal(d) * 1e-2).astype(np.float32)
    g = rng.laplace(0, 1e-4, d).astype(np.float32)          # a mixture: one element in ten a hundred times larger
    g[rng.random(d) < 0.1] *= np.float32(100.0)
    return g


def _length(rng):
    c = int(rng.integers(0, 5))
    if c == 0:
        return int(rng.integers(1, 3000))
    if c == 1:
        return int(rng.integers(3000, 300_000))
    if c == 2:
        return int(rng.integers(300_000, 4_000_000))
    if c == 3:                                               # around the lengths at which the dense stages prefetch
        return int(rng.integers(4, 8)) * 4096 * 256 + int(rng.integers(0, 300))
    return int(rng.integers(12_000_000, 16_000_000))         # the first pass in address order


@pytest.mark.parametrize("seed", range(8))
def test_random_single_calls(oracle, seed):
    rng = np.random.default_rng(7000 + seed)
    for case in range(5):
        d, dist, M, kind = _length(rng), int(rng.integers(0, 3)), int(rng.integers(1, 5)), int(rng.integers(0, 4))
        delta, delta1 = float(10 ** rng.uniform(-4, -0.7)), float(rng.choice([0.25, 0.05, 0.5]))
        ratios = oracle.schedule(delta, M, delta1)
        g = _draw(rng, d, kind)
        r = _draw(rng, d, kind) * np.float32(0.3) if rng.random() < 0.6 else None
        go, ro = (int(rng.integers(0, 4)), int(rng.integers(0, 4))) if rng.random() < 0.3 else (0, 0)
        label = f"seed {seed} case {case}: d={d} dist={dist} ratios={ratios} input {kind} ec={r is not None} offsets {go},{ro}"
        for _ in range(int(rng.integers(1, 4))):
            out = run_gpu(g, r, dist, ratios, grad_offset=go, res_offset=ro)
            check_parity(oracle, g, r, dist, ratios, out, label=label)
            if r is not None:
                r = out.residual


@pytest.mark.parametrize("seed", range(4))
def test_random_batched_calls(oracle, seed):
    import torch
    rng = np.random.default_rng(7100 + seed)
    for case in range(3):
        n, total = int(rng.integers(1, 40)), _length(rng)
        cuts = rng.integers(1, max(2, total), size=n - 1)
        offs = sorted(set([0] + [int(c) for c in cuts] + [max(total, n)]))
        d, dist, M, kind = offs[-1], int(rng.integers(0, 3)), int(rng.integers(1, 4)), int(rng.integers(0, 4))
        delta = float(10 ** rng.uniform(-3.5, -1))
        g = _draw(rng, d, kind)
        r = _draw(rng, d, kind) * np.float32(0.3) if rng.random() < 0.6 else None
        base = int(rng.integers(0, 4)) if rng.random() < 0.3 else 0
        label = f"seed {seed} case {case}: {len(offs) - 1} tensors, d={d} dist={dist} M={M} delta={delta:.2e} ec={r is not None} base {base}"
        if rng.random() < 0.4:
            g16 = torch.from_numpy(g * np.float32(10)).to(torch.bfloat16 if rng.random() < 0.5 else torch.float16)
            g, src = g16.to(torch.float32).numpy(), g16
        else:
            src = g
        out = run_batched(src, r, offs, delta, dist, M, base_offset=base, repeat=int(rng.integers(1, 3)))
        check_batched(oracle, g, r, offs, delta, dist, M, out, label)


@pytest.mark.parametrize("seed", range(3))
def test_random_comparator_calls(oracle, seed):
    import paper_2101_10761_amd as sidco
    rng = np.random.default_rng(7200 + seed)
    for case in range(3):
        d, kind = _length(rng), int(rng.integers(0, 4))
        g = _draw(rng, d, kind)
        r = _draw(rng, d, kind) * np.float32(0.3) if rng.random() < 0.6 else None
        k = int(max(1, min(d, d * 10 ** rng.uniform(-4, -0.5))))
        check_topk(oracle, g, r, k, run_topk(g, r, k), label=f"seed {seed} case {case}: top-k d={d} k={k}")
        delta, rho = float(10 ** rng.uniform(-3.5, -1)), float(rng.choice([0.01, 0.05, 0.002]))
        try:
            sidco.sidco_dgc_sizes(d, delta, rho)
        except Exception:
            continue                                          # too short a vector for this ratio and subset
        check_dgc(oracle, g, r, delta, rho, case, run_dgc(g, r, delta, rho, case), f"seed {seed} case {case}: dgc d={d}")
