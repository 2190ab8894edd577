"""Shared helpers of the GPU parity tests: run the HIP path through the C ABI, compare with the oracle.

Parity bar (same for every case):
  * fitted statistics and every stage threshold within 1e-5 relative of the oracle's, where the oracle's
    stage m is evaluated on the exceedance set of the GPU's own eta_{m-1} (thresholds are injected stage
    by stage, so a last-bit difference in an early threshold cannot blur the later comparison);
  * the number of elements each stage's fit ran over: exact;
  * given the GPU's eta_M: selected index set, values and updated residual bit-exact.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

STATS_RTOL = 1e-5


@dataclass
class GpuResult:
    idx: np.ndarray       # int32, in the library's traversal order
    val: np.ndarray
    count: int
    eta: float
    residual: np.ndarray | None
    etas: np.ndarray      # float32[M]
    n: np.ndarray         # int64[M]
    stats: np.ndarray     # float64[M,3]
    status: int
    selected: int


class GpuCall:
    """One sparsifier call on cuda:0 in three steps - buffers, enqueue on a stream, results - so that a test
    can have several calls in flight.  grad_offset / res_offset (in elements) place the vectors at unaligned
    addresses.  use_default_schedule=(delta, stages) calls sidco_compress instead of sidco_compress_ex."""

    def __init__(self, g, r, dist, ratios, cap=None, *, grad_offset=0, res_offset=0, use_default_schedule=None):
        import torch
        import paper_2101_10761_amd as sidco

        dev = torch.device("cuda:0")
        self.g, self.dist, self.ratios = g, dist, ratios
        self.grad_offset, self.res_offset, self.default = grad_offset, res_offset, use_default_schedule
        d = g.size
        self.gbuf = torch.zeros(d + grad_offset + 8, dtype=torch.float32, device=dev)
        self.gt = self.gbuf[grad_offset:grad_offset + d]
        self.gt.copy_(torch.from_numpy(g))
        self.rt = self.rbuf = None
        if r is not None:
            self.rbuf = torch.zeros(d + res_offset + 8, dtype=torch.float32, device=dev)
            self.rt = self.rbuf[res_offset:res_offset + d]
            self.rt.copy_(torch.from_numpy(r))
        if use_default_schedule is not None:
            cap = sidco.sidco_out_capacity(d, use_default_schedule[0])
        elif cap is None:
            cap = d
        self.cap = cap
        guard = 64
        self.out_idx = torch.full((cap + guard,), -7, dtype=torch.int32, device=dev)
        self.out_val = torch.full((cap + guard,), 7.0, dtype=torch.float32, device=dev)
        self.out_count = torch.full((1,), -1, dtype=torch.int32, device=dev)
        self.out_eta = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()

    def launch(self, stream=None):
        import paper_2101_10761_amd as sidco
        cap = self.cap
        if self.default is not None:
            delta, stages = self.default
            sidco.sidco_compress(self.gt, self.rt, delta, self.dist, stages, self.out_idx[:cap], self.out_val[:cap],
                                 self.out_count, self.out_eta, stream=stream)
        else:
            sidco.sidco_compress_ex(self.gt, self.rt, self.dist, list(self.ratios), self.out_idx[:cap], self.out_val[:cap],
                                    self.out_count, self.out_eta, stream=stream)
        return self

    def collect(self, stream=None):
        import torch
        import paper_2101_10761_amd as sidco
        diag = sidco.sidco_read_diag(stream)
        torch.cuda.synchronize()
        cap, g, d = self.cap, self.g, self.g.size
        k = int(self.out_count.item())
        assert 0 <= k <= cap
        # nothing may be written past the count / the capacity, and the gradient is read-only
        assert torch.all(self.out_idx[cap:] == -7) and torch.all(self.out_val[cap:] == 7.0)
        assert torch.all(self.out_idx[k:cap] == -7)
        np.testing.assert_array_equal(self.gt.cpu().numpy().view(np.uint32), g.view(np.uint32))
        if self.grad_offset:
            assert torch.all(self.gbuf[:self.grad_offset] == 0)
        assert torch.all(self.gbuf[self.grad_offset + d:] == 0)
        if self.rt is not None:
            assert torch.all(self.rbuf[self.res_offset + d:] == 0)
            if self.res_offset:
                assert torch.all(self.rbuf[:self.res_offset] == 0)
        M = diag.stages
        return GpuResult(
            idx=self.out_idx[:k].cpu().numpy(), val=self.out_val[:k].cpu().numpy(), count=k,
            eta=float(self.out_eta.item()), residual=None if self.rt is None else self.rt.cpu().numpy(),
            etas=np.array(diag.eta[:M], dtype=np.float32), n=np.array(diag.n[:M], dtype=np.int64),
            stats=np.array([[diag.stats[m][q] for q in range(3)] for m in range(M)]), status=diag.status,
            selected=diag.selected)


def run_gpu(g, r, dist, ratios, cap=None, *, grad_offset=0, res_offset=0, use_default_schedule=None):
    """Runs one call on cuda:0 on the current stream and returns its results."""
    return GpuCall(g, r, dist, ratios, cap, grad_offset=grad_offset, res_offset=res_offset,
                   use_default_schedule=use_default_schedule).launch().collect()


def _close(a, b, rtol=STATS_RTOL, atol=0.0):
    if math.isnan(a) or math.isnan(b):
        return math.isnan(a) and math.isnan(b)
    if math.isinf(a) or math.isinf(b):
        return a == b
    return abs(a - b) <= rtol * max(abs(a), abs(b)) + atol


def check_parity(oracle, g, r, dist, ratios, res: GpuResult, *, capacity=None, label=""):
    """Compares one GPU result with the oracle to the parity bar.  Returns the oracle result."""
    M = len(ratios)
    assert res.etas.size == M, label
    ref = oracle.compress(g, r, ratios=list(ratios), dist=dist, eta_inject=res.etas)
    # thresholds, stage by stage (oracle's stage m is computed on top of the GPU's eta_{m-1})
    for m in range(M):
        assert _close(float(res.etas[m]), float(ref.etas_own[m])), (
            f"{label} eta_{m + 1}: gpu {res.etas[m]!r} oracle {ref.etas_own[m]!r}")
    assert (math.isnan(res.eta) and math.isnan(ref.eta)) or res.eta == float(res.etas[M - 1])
    # fitted statistics (only those the law uses are produced on the GPU)
    np.testing.assert_array_equal(res.n, ref.n_stage, err_msg=f"{label} n per stage")
    for m in range(M):
        used = [0]
        if m == 0:
            used += [1] if dist == 2 else ([2] if dist == 1 else [])
        else:
            used += [1] if dist != 0 else []
        if ref.n_stage[m] == 0:
            continue
        for q in used:
            # a variance is a difference of two fp64 sums of size mean^2 + variance: below 1e-9 of that
            # it is summation-order noise (constant-magnitude vectors), not signal
            atol = 1e-9 * (ref.stats[m, 0] ** 2 + abs(ref.stats[m, 1])) if q == 1 else 0.0
            assert _close(res.stats[m, q], ref.stats[m, q], atol=atol), (
                f"{label} stage {m + 1} stat {q}: gpu {res.stats[m, q]!r} oracle {ref.stats[m, q]!r}")
    # Flags of clear-cut conditions agree.  The "limit" flags (variance <= 0, gamma s <= 0 / clamp) sit on
    # a knife edge by construction (a sum's rounding decides them) and the readings make the threshold
    # continuous across that edge, so they are asserted only by the tests that force them clearly.
    robust = 1 | 16
    assert (res.status & robust) == (ref.status & robust), f"{label} status gpu {res.status} oracle {ref.status}"
    # selection: bit-exact given the same threshold
    assert res.selected == ref.count, f"{label} selected {res.selected} vs {ref.count}"
    order = np.argsort(res.idx, kind="stable")
    gi, gv = res.idx[order], res.val[order]
    if capacity is None or ref.count <= capacity:
        assert not (res.status & 32)
        assert res.count == ref.count, f"{label} count {res.count} vs {ref.count}"
        np.testing.assert_array_equal(gi, ref.idx, err_msg=f"{label} index set")
        np.testing.assert_array_equal(gv.view(np.uint32), ref.val.view(np.uint32), err_msg=f"{label} values")
        if r is not None:
            np.testing.assert_array_equal(res.residual.view(np.uint32), ref.residual.view(np.uint32),
                                          err_msg=f"{label} residual")
    else:
        # overflow: exactly `capacity` pairs, all of them true exceedances with their values; the rest
        # stays in the residual
        assert res.status & 32 and res.count == capacity
        assert np.all(np.diff(gi) > 0)
        pos = np.searchsorted(ref.idx, gi)
        assert np.all(ref.idx[pos] == gi)
        np.testing.assert_array_equal(gv.view(np.uint32), ref.val[pos].view(np.uint32))
        if r is not None:
            acc = oracle.ec_add(g, r)
            want = acc.copy()
            want[gi] = 0
            np.testing.assert_array_equal(res.residual.view(np.uint32), want.view(np.uint32))
    return ref
