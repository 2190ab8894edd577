"""GPU: sidco_compress_static, the entry point that allocates nothing (its workspace is a fixed array in the
library's device code), against sidco_compress on the same inputs - two calls in a row, the second shorter."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _call(fn, g, r, delta, dist, stages):
    """One call of `fn` (sidco_compress or sidco_compress_static) on fresh device copies of (g, r)."""
    import torch
    import paper_2101_10761_amd as sidco
    dev = torch.device("cuda:0")
    d = g.size
    cap = sidco.sidco_out_capacity(d, delta)
    gt = torch.from_numpy(g).to(dev)
    rt = None if r is None else torch.from_numpy(r).to(dev)
    out_idx = torch.full((cap + 16,), -7, dtype=torch.int32, device=dev)
    out_val = torch.full((cap + 16,), 7.0, dtype=torch.float32, device=dev)
    out_count = torch.full((1,), -1, dtype=torch.int32, device=dev)
    out_eta = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    fn(gt, rt, delta, dist, stages, out_idx[:cap], out_val[:cap], out_count, out_eta)
    torch.cuda.synchronize()
    free_after = torch.cuda.mem_get_info()[0]
    k = int(out_count.item())
    assert 0 <= k <= cap
    assert torch.all(out_idx[k:] == -7) and torch.all(out_val[cap:] == 7.0)
    np.testing.assert_array_equal(gt.cpu().numpy().view(np.uint32), g.view(np.uint32))
    order = np.argsort(out_idx[:k].cpu().numpy(), kind="stable")
    return dict(idx=out_idx[:k].cpu().numpy()[order], val=out_val[:k].cpu().numpy()[order], count=k,
                eta=np.float32(out_eta.item()), residual=None if rt is None else rt.cpu().numpy(),
                allocated=free_before - free_after)


def test_static_entry_point_matches_sidco_compress(oracle):
    import paper_2101_10761_amd as sidco
    assert sidco.sidco_static_max_elements() == 2_097_152
    sidco.sidco_static_init()    # set-up: the array's address on this device (the runtime maps the array here)
    rng = np.random.default_rng(7)
    cases = [(1_500_003, 2, 0.001, 3, True), (70_001, 0, 0.01, 2, True), (2_097_152, 1, 0.002, 2, False), (999, 0, 0.05, 1, True)]
    for d, dist, delta, stages, ec in cases:       # each call after the first finds the previous call's lists in the scratch
        g = (rng.standard_t(3.0, size=d) * 1e-3).astype(np.float32)
        r = rng.laplace(0, 3e-4, size=d).astype(np.float32) if ec else None
        want = _call(sidco.sidco_compress, g, r, delta, dist, stages)
        got = _call(sidco.sidco_compress_static, g, r, delta, dist, stages)
        assert got["allocated"] <= 0, "the static entry point must not take device memory"
        # thresholds within the parity bar of the fitted values (1e-5 relative); given the threshold, the set is exact
        assert abs(float(got["eta"]) - float(want["eta"])) <= 1e-5 * abs(float(want["eta"]))
        if got["eta"].tobytes() == want["eta"].tobytes():
            assert got["count"] == want["count"]
            np.testing.assert_array_equal(got["idx"], want["idx"])
            np.testing.assert_array_equal(got["val"].view(np.uint32), want["val"].view(np.uint32))
            if ec:
                np.testing.assert_array_equal(got["residual"].view(np.uint32), want["residual"].view(np.uint32))
        # and against the oracle's selection at the call's own threshold
        M = len(oracle.schedule(delta, stages, 0.25))
        ref = oracle.compress(g, r, ratios=oracle.schedule(delta, stages, 0.25), dist=dist,
                              eta_inject=np.full(M, got["eta"], np.float32))
        assert got["count"] == ref.count
        np.testing.assert_array_equal(got["idx"], ref.idx)
        np.testing.assert_array_equal(got["val"].view(np.uint32), ref.val.view(np.uint32))
        if ec:
            np.testing.assert_array_equal(got["residual"].view(np.uint32), ref.residual.view(np.uint32))


def test_static_entry_point_rejects_longer_vectors():
    import torch
    import paper_2101_10761_amd as sidco
    d = sidco.sidco_static_max_elements() + 1
    dev = torch.device("cuda:0")
    g = torch.zeros(d, dtype=torch.float32, device=dev)
    cap = sidco.sidco_out_capacity(d, 0.001)
    oi = torch.zeros(cap, dtype=torch.int32, device=dev)
    ov = torch.zeros(cap, dtype=torch.float32, device=dev)
    oc = torch.full((1,), -1, dtype=torch.int32, device=dev)
    oe = torch.zeros(1, dtype=torch.float32, device=dev)
    with pytest.raises(sidco.SidcoError) as e:
        sidco.sidco_compress_static(g, None, 0.001, 0, 2, oi, ov, oc, oe)
    assert e.value.code == -2 and "2097152" in str(e.value)
    torch.cuda.synchronize()
    assert int(oc.item()) == -1   # nothing was enqueued
