"""GPU parity of the exact Top-k comparator (radix select), through the C ABI, against the oracle's sort."""
import numpy as np
import pytest

from paper_2101_10761_amd import workloads

pytestmark = pytest.mark.gpu


def run_topk(g, r, k, *, grad_offset=0, res_offset=0):
    """`g` is a float32 numpy vector (sidco_topk) or a 16-bit torch CPU tensor (sidco_topk_typed)."""
    import torch
    import paper_2101_10761_amd as sidco

    dev = torch.device("cuda:0")
    typed = isinstance(g, torch.Tensor)
    g_cpu = g if typed else torch.from_numpy(g)
    d = g_cpu.numel()
    gbuf = torch.zeros(d + grad_offset + 8, dtype=g_cpu.dtype, device=dev)
    gt = gbuf[grad_offset:grad_offset + d]
    gt.copy_(g_cpu)
    rt = None
    if r is not None:
        rbuf = torch.zeros(d + res_offset + 8, dtype=torch.float32, device=dev)
        rt = rbuf[res_offset:res_offset + d]
        rt.copy_(torch.from_numpy(r))
    guard = 64
    out_idx = torch.full((k + guard,), -7, dtype=torch.int32, device=dev)
    out_val = torch.full((k + guard,), 7.0, dtype=torch.float32, device=dev)
    out_count = torch.full((1,), -1, dtype=torch.int32, device=dev)
    out_kth = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
    (sidco.sidco_topk_typed if typed else sidco.sidco_topk)(gt, rt, k, out_idx[:k], out_val[:k], out_count, out_kth)
    torch.cuda.synchronize()
    assert torch.all(out_idx[k:] == -7) and torch.all(out_val[k:] == 7.0)
    assert torch.equal(gt.cpu().view(torch.uint8), g_cpu.view(torch.uint8))      # the gradient is read-only
    assert torch.all(gbuf[grad_offset + d:].view(torch.uint8) == 0) and torch.all(gbuf[:grad_offset].view(torch.uint8) == 0)
    if rt is not None:
        assert torch.all(rbuf[res_offset + d:] == 0)
    return (out_idx[:k].cpu().numpy(), out_val[:k].cpu().numpy(), int(out_count.item()), np.float32(out_kth.item()),
            None if rt is None else rt.cpu().numpy())


def check_topk(oracle, g, r, k, out, label=""):
    """The k-th largest magnitude and the entries above it are unique and must match exactly; the entries equal
    to it that complete the set may be any of the tied ones."""
    idx, val, count, kth, res = out
    acc = oracle.ec_add(g, r)
    mag = np.abs(acc)
    ref = oracle.topk(acc, k)                 # ascending indices; ties broken towards lower indices
    kth_ref = mag[ref].min()
    assert count == k, label
    assert kth == kth_ref, f"{label}: k-th magnitude gpu {kth!r} oracle {kth_ref!r}"
    assert np.unique(idx).size == k and idx.min() >= 0 and idx.max() < g.size, label
    np.testing.assert_array_equal(val.view(np.uint32), acc[idx].view(np.uint32), err_msg=f"{label} values")
    above = np.sort(idx[mag[idx] > kth_ref])
    np.testing.assert_array_equal(above, ref[mag[ref] > kth_ref], err_msg=f"{label} entries above the k-th magnitude")
    assert np.all(mag[idx] >= kth_ref), label
    if r is not None:
        want = acc.copy()
        want[idx] = 0
        np.testing.assert_array_equal(res.view(np.uint32), want.view(np.uint32), err_msg=f"{label} residual")
    return ref


def _inputs(d, seed, scale=1e-3):
    rng = np.random.default_rng(seed)
    return rng.laplace(0, scale, size=d).astype(np.float32), rng.laplace(0, 0.3 * scale, size=d).astype(np.float32)


@pytest.mark.parametrize("d", [1, 2, 63, 256, 257, 1000, 70_001, 1_048_576, 2_100_003])
def test_sizes_and_ks(oracle, d):
    g, r = _inputs(d, 900 + d % 89)
    for k in sorted({1, max(1, d // 1000), max(1, d // 10), max(1, d // 2), d}):
        for res in (r, None):
            check_topk(oracle, g, res, k, run_topk(g, res, k), label=f"d={d} k={k} ec={res is not None}")


@pytest.mark.parametrize("goff,roff", [(1, 0), (0, 3), (2, 1)])
def test_unaligned(oracle, goff, roff):
    g, r = _inputs(300_007, 17)
    check_topk(oracle, g, r, 3000, run_topk(g, r, 3000, grad_offset=goff, res_offset=roff), label="unaligned")


def test_ties_on_the_kth_magnitude(oracle):
    """Quantised magnitudes: many entries equal the k-th largest one, and k cuts through them."""
    rng = np.random.default_rng(3)
    g = (np.round(rng.laplace(0, 3.0, size=200_000)) * 0.125).astype(np.float32)
    for k in (1, 10, 1234, 50_000, 150_000, 200_000):
        check_topk(oracle, g, None, k, run_topk(g, None, k), label=f"ties k={k}")
    z = np.zeros(5000, np.float32)
    check_topk(oracle, z, z.copy(), 77, run_topk(z, z.copy(), 77), label="zeros")
    c = np.full(4097, -0.25, np.float32)
    check_topk(oracle, c, None, 4000, run_topk(c, None, 4000), label="constant")


def test_extreme_magnitudes(oracle):
    g, r = _inputs(100_000, 5)
    g[17] = np.inf
    g[18] = -3.0e38
    g[19] = np.float32(1e-45)      # denormal
    g[20] = -0.0
    for k in (1, 2, 3, 100, 99_999, 100_000):
        check_topk(oracle, g, None, k, run_topk(g, None, k), label=f"extremes k={k}")


def test_threshold_operator_equals_topk_at_khat(oracle):
    """Footnote of Sec. 2.3: C_eta keeps exactly the Top-khat entries (no tie straddles eta on continuous data)."""
    from gpu_harness import run_gpu
    w = workloads.config2()
    ratios = oracle.schedule(w.delta, w.stages, w.delta1)
    out = run_gpu(w.grad, w.residual, w.dist, ratios, cap=w.d // 50)
    t = run_topk(w.grad, w.residual, out.count)
    check_topk(oracle, w.grad, w.residual, out.count, t, label="config2 k=khat")
    np.testing.assert_array_equal(np.sort(t[0]), np.sort(out.idx))
    assert t[3] > out.eta
    np.testing.assert_array_equal(t[4].view(np.uint32), out.residual.view(np.uint32))


@pytest.mark.parametrize("cfg,delta", [("cfg3", 0.001), ("cfg5", 0.1)])
def test_full_size(oracle, cfg, delta):
    """The comparator at the benchmark configurations' own lengths; config 5 with a carried residual (the
    second iteration's input: fresh gradient plus what the first iteration left)."""
    if cfg == "cfg3":
        w = workloads.config3()
        g, r = w.grad, w.residual
    else:
        d = 138_357_544
        g0 = workloads.config5_grad(0, d)
        k0 = int(np.ceil(delta * d))
        first = run_topk(g0, np.zeros(d, np.float32), k0)
        r = first[4]                       # the residual after the first iteration's Top-k
        del g0, first
        g = workloads.config5_grad(1, d)
    k = int(np.ceil(delta * g.size))
    check_topk(oracle, g, r, k, run_topk(g, r, k), label=f"{cfg} delta={delta} k={k}")


def test_profile_hooks_topk():
    import paper_2101_10761_amd as sidco
    g, r = _inputs(1_000_000, 41)
    sidco.sidco_set_profiling(True)
    try:
        run_topk(g, r, 1000)
        prof = sidco.sidco_get_profile()
    finally:
        sidco.sidco_set_profiling(False)
    assert [n for n, _ in prof] == ["k_topk_zero", "k_topk_hist", "k_topk_compact", "k_topk_refine", "k_topk_final"]
