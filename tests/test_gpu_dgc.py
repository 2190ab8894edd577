"""GPU parity of the DGC comparator (threshold from a radix select on a random subset, first pass, trim), through
the C ABI, against the oracle."""
import numpy as np
import pytest

from paper_2101_10761_amd import workloads

pytestmark = pytest.mark.gpu


def run_dgc(g, r, delta, rho, seed, *, grad_offset=0, res_offset=0):
    """`g` is a float32 numpy vector (sidco_dgc) or a 16-bit torch CPU tensor (sidco_dgc_typed)."""
    import torch
    import paper_2101_10761_amd as sidco

    dev = torch.device("cuda:0")
    typed = isinstance(g, torch.Tensor)
    g_cpu = g if typed else torch.from_numpy(g)
    d = g_cpu.numel()
    k = sidco.sidco_dgc_sizes(d, delta, rho)[2]
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
    out_eta = torch.full((1,), -1.0, dtype=torch.float32, device=dev)
    (sidco.sidco_dgc_typed if typed else sidco.sidco_dgc)(gt, rt, delta, rho, seed, out_idx[:k], out_val[:k], out_count,
                                                          out_eta)
    torch.cuda.synchronize()
    n_s, k_s, first, written = sidco.sidco_dgc_result()
    count = int(out_count.item())
    assert written == count and 0 <= count <= k
    assert torch.all(out_idx[count:] == -7) and torch.all(out_val[count:] == 7.0)
    assert torch.equal(gt.cpu().view(torch.uint8), g_cpu.view(torch.uint8))      # the gradient is read-only
    assert torch.all(gbuf[grad_offset + d:].view(torch.uint8) == 0) and torch.all(gbuf[:grad_offset].view(torch.uint8) == 0)
    if rt is not None:
        assert torch.all(rbuf[res_offset + d:] == 0)
    return dict(idx=out_idx[:count].cpu().numpy(), val=out_val[:count].cpu().numpy(), count=count,
                eta=np.float32(out_eta.item()), first=first, n_s=n_s, k_s=k_s, k=k,
                res=None if rt is None else rt.cpu().numpy())


def check_dgc(oracle, g, r, delta, rho, seed, out, label=""):
    ref = oracle.dgc(g, r, delta=delta, sample_ratio=rho, seed=seed)
    acc = oracle.ec_add(g, r)
    mag = np.abs(acc)
    assert (out["n_s"], out["k_s"], out["k"]) == oracle.dgc_sizes(g.size, delta, rho), label
    assert out["eta"].view(np.uint32) == ref.eta.view(np.uint32), f"{label}: eta gpu {out['eta']!r} oracle {ref.eta!r}"
    assert out["first"] == ref.first_pass, label
    assert out["count"] == ref.count, label
    idx, val = out["idx"], out["val"]
    assert np.unique(idx).size == idx.size, label
    np.testing.assert_array_equal(val.view(np.uint32), acc[idx].view(np.uint32), err_msg=f"{label} values")
    if ref.first_pass <= out["k"]:
        np.testing.assert_array_equal(np.sort(idx), ref.idx, err_msg=f"{label} untrimmed selection")
    else:
        # trimmed: the smallest magnitude that stayed and the entries above it are unique; ties may differ
        kth = mag[ref.idx].min()
        assert mag[idx].min() == kth, label
        np.testing.assert_array_equal(np.sort(idx[mag[idx] > kth]), ref.idx[mag[ref.idx] > kth],
                                      err_msg=f"{label} entries above the k-th magnitude")
    if r is not None:
        want = acc.copy()
        want[idx] = 0
        np.testing.assert_array_equal(out["res"].view(np.uint32), want.view(np.uint32), err_msg=f"{label} residual")
    return ref


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("with_residual", [False, True])
def test_random_vectors_both_branches(oracle, seed, with_residual):
    rng = np.random.Generator(np.random.PCG64(500 + seed))
    d = int(rng.integers(200_000, 3_000_000))
    g = rng.laplace(0.0, 1e-3, d).astype(np.float32)
    r = rng.laplace(0.0, 3e-4, d).astype(np.float32) if with_residual else None
    delta, rho = (0.001, 0.05) if seed % 2 else (0.01, 0.01)
    out = run_dgc(g, r, delta, rho, seed)
    check_dgc(oracle, g, r, delta, rho, seed, out, f"seed {seed} d {d}")


def test_trimmed_and_untrimmed_branches_are_both_exercised(oracle):
    rng = np.random.Generator(np.random.PCG64(77))
    d = 1_000_003
    g = rng.standard_t(3, d).astype(np.float32) * np.float32(1e-3)
    seen = set()
    for seed in range(12):
        out = run_dgc(g, None, 0.002, 0.02, seed)
        ref = check_dgc(oracle, g, None, 0.002, 0.02, seed, out, f"seed {seed}")
        seen.add(ref.first_pass > out["k"])
        if len(seen) == 2 and seed >= 3:
            break
    assert seen == {False, True}


@pytest.mark.parametrize("d", [1, 2, 63, 255, 256, 257, 1023, 4097, 100_001])
def test_small_and_ragged_sizes(oracle, d):
    rng = np.random.Generator(np.random.PCG64(d))
    g = rng.laplace(0.0, 1e-3, d).astype(np.float32)
    r = rng.laplace(0.0, 1e-3, d).astype(np.float32)
    for delta, rho in ((0.1, 0.5), (0.01, 1.0), (0.5, 0.05)):
        out = run_dgc(g, r, delta, rho, 5)
        check_dgc(oracle, g, r, delta, rho, 5, out, f"d {d} delta {delta} rho {rho}")


@pytest.mark.parametrize("go,ro", [(1, 0), (0, 3), (2, 2)])
def test_unaligned_buffers(oracle, go, ro):
    rng = np.random.Generator(np.random.PCG64(11))
    d = 300_007
    g = rng.laplace(0.0, 1e-3, d).astype(np.float32)
    r = rng.laplace(0.0, 1e-3, d).astype(np.float32)
    out = run_dgc(g, r, 0.01, 0.02, 9, grad_offset=go, res_offset=ro)
    check_dgc(oracle, g, r, 0.01, 0.02, 9, out, f"offsets {go},{ro}")


def test_ties_zeros_and_constant_vectors(oracle):
    d = 50_000
    z = np.zeros(d, dtype=np.float32)
    out = run_dgc(z, z.copy(), 0.01, 0.1, 1)
    assert out["count"] == 0 and out["first"] == 0 and out["eta"] == 0
    # every magnitude equal: nothing is strictly above the threshold
    c = np.full(d, -2.5e-3, dtype=np.float32)
    out = run_dgc(c, None, 0.01, 0.1, 1)
    assert out["count"] == 0 and out["eta"] == np.float32(2.5e-3)
    # two levels: the trim must keep exactly k of the tied large entries
    g = np.full(d, 1e-3, dtype=np.float32)
    g[::5] = 4e-3
    for seed in range(50):
        out = run_dgc(g, None, 0.01, 0.0004, seed)     # 20 draws, k_s = 1
        if out["eta"] == np.float32(1e-3):
            break
    else:
        pytest.fail("no seed drew only small entries")
    assert out["first"] == d // 5 and out["count"] == out["k"] == 500
    assert np.all(out["val"] == np.float32(4e-3)) and np.unique(out["idx"]).size == 500
    assert np.all(out["idx"] % 5 == 0)


def test_non_finite_entries(oracle):
    rng = np.random.Generator(np.random.PCG64(21))
    d = 400_000
    g = rng.laplace(0.0, 1e-3, d).astype(np.float32)
    g[[5, 70_000, 399_999]] = [np.inf, -np.inf, np.nan]
    out = run_dgc(g, None, 0.005, 0.02, 3)
    ref = oracle.dgc(g, None, delta=0.005, sample_ratio=0.02, seed=3)
    assert out["eta"].view(np.uint32) == ref.eta.view(np.uint32)
    assert out["first"] == ref.first_pass and out["count"] == ref.count
    if ref.first_pass <= out["k"]:
        np.testing.assert_array_equal(np.sort(out["idx"]), ref.idx)
    assert 399_999 not in out["idx"]          # a NaN is not above any threshold
    assert 5 in out["idx"] and 70_000 in out["idx"]


def test_headline_size(oracle):
    w = workloads.config3()
    out = run_dgc(w.grad, None, w.delta, 0.01, 2101)
    check_dgc(oracle, w.grad, None, w.delta, 0.01, 2101, out, "cfg3")
    out = run_dgc(w.grad, w.residual, w.delta, 0.01, 2102)
    check_dgc(oracle, w.grad, w.residual, w.delta, 0.01, 2102, out, "cfg3 with residual")
