"""GPU parity of the batched call: every tensor of a flat buffer against the oracle run on that tensor alone."""
import numpy as np
import pytest

from gpu_harness import GpuResult, check_parity
from paper_2101_10761_amd import workloads

pytestmark = pytest.mark.gpu


def run_batched(g, r, offsets, delta, dist, stages, *, base_offset=0, repeat=1):
    """One batched call (or `repeat` identical ones, each on a fresh copy of the residual); returns one GpuResult
    per tensor of the last call.  `g` is a float32 numpy vector (sidco_compress_batched) or a 16-bit torch CPU
    tensor (sidco_compress_batched_typed)."""
    import torch
    import paper_2101_10761_amd as sidco
    dev = torch.device("cuda:0")
    n = len(offsets) - 1
    typed = isinstance(g, torch.Tensor)
    g_cpu = g if typed else torch.from_numpy(g)
    d = g_cpu.numel()
    call = sidco.sidco_compress_batched_typed if typed else sidco.sidco_compress_batched
    gbuf = torch.zeros(d + base_offset + 8, dtype=g_cpu.dtype, device=dev)
    gt = gbuf[base_offset:base_offset + d]
    gt.copy_(g_cpu)
    rbuf = rt = None
    if r is not None:
        rbuf = torch.zeros(d + base_offset + 8, dtype=torch.float32, device=dev)
        rt = rbuf[base_offset:base_offset + d]
    out_offsets = sidco.sidco_batched_out_offsets(offsets, delta)
    guard = 64
    total = out_offsets[-1]
    for _ in range(repeat):
        if rt is not None:
            rt.copy_(torch.from_numpy(r))
        out_idx = torch.full((total + guard,), -7, dtype=torch.int32, device=dev)
        out_val = torch.full((total + guard,), 7.0, dtype=torch.float32, device=dev)
        out_counts = torch.full((n,), -1, dtype=torch.int32, device=dev)
        out_etas = torch.full((n,), -1.0, dtype=torch.float32, device=dev)
        call(gt, rt, offsets, delta, dist, stages, out_idx[:total], out_val[:total], out_offsets, out_counts, out_etas)
    torch.cuda.synchronize()
    assert torch.all(out_idx[total:] == -7) and torch.all(out_val[total:] == 7.0)
    assert torch.equal(gt.cpu().view(torch.uint8), g_cpu.view(torch.uint8))      # the gradient is read-only
    assert torch.all(gbuf[base_offset + d:].view(torch.uint8) == 0) and torch.all(gbuf[:base_offset].view(torch.uint8) == 0)
    if rbuf is not None:
        assert torch.all(rbuf[base_offset + d:] == 0) and torch.all(rbuf[:base_offset] == 0)
    counts = out_counts.cpu().numpy()
    etas = out_etas.cpu().numpy()
    idx_all, val_all = out_idx.cpu().numpy(), out_val.cpu().numpy()
    res_all = None if rt is None else rt.cpu().numpy()
    results = []
    for t in range(n):
        k, o0, o1 = int(counts[t]), out_offsets[t], out_offsets[t + 1]
        assert 0 <= k <= o1 - o0
        assert np.all(idx_all[o0 + k:o1] == -7), f"tensor {t}: written past its count"
        diag = sidco.sidco_read_diag_batched(t)
        M = diag.stages
        results.append(GpuResult(
            idx=idx_all[o0:o0 + k].copy(), val=val_all[o0:o0 + k].copy(), count=k, eta=float(etas[t]),
            residual=None if res_all is None else res_all[offsets[t]:offsets[t + 1]].copy(),
            etas=np.array(diag.eta[:M], dtype=np.float32), n=np.array(diag.n[:M], dtype=np.int64),
            stats=np.array([[diag.stats[m][q] for q in range(3)] for m in range(M)]), status=diag.status,
            selected=diag.selected))
    return results


def check_batched(oracle, g, r, offsets, delta, dist, stages, results, label):
    import paper_2101_10761_amd as sidco
    ratios = oracle.schedule(delta, stages, 0.25)
    for t, res in enumerate(results):
        a, b = offsets[t], offsets[t + 1]
        gt = np.ascontiguousarray(g[a:b])
        rt = None if r is None else np.ascontiguousarray(r[a:b])
        cap = sidco.sidco_out_capacity(b - a, delta)
        check_parity(oracle, gt, rt, dist, ratios, res, capacity=cap, label=f"{label} tensor {t} (d={b - a})")


@pytest.mark.parametrize("dist,stages,delta", [(1, 2, 1e-3), (0, 3, 1e-2), (2, 1, 0.02)])
def test_config4_ragged_tensors(oracle, dist, stages, delta):
    w = workloads.config4(d=6_600_000, ragged=True)   # 50 ragged, unaligned tensors with scales over three decades
    offs = [int(x) for x in w.tensor_offsets]
    r = np.random.default_rng(4).laplace(0, 1e-5, size=w.d).astype(np.float32)
    for res_in in (r, None):
        out = run_batched(w.grad, res_in, offs, delta, dist, stages)
        check_batched(oracle, w.grad, res_in, offs, delta, dist, stages, out, f"cfg4 dist={dist} M={stages}")


def test_config4_full_size_per_tensor(oracle):
    """Config 4 as the benchmark runs its per-tensor mode: 66,000,000 elements, 50 tensors, one batched call."""
    w = workloads.config4()
    offs = [int(x) for x in w.tensor_offsets]
    out = run_batched(w.grad, w.residual, offs, w.delta, w.dist, w.stages)
    check_batched(oracle, w.grad, w.residual, offs, w.delta, w.dist, w.stages, out, "cfg4 full per tensor")


@pytest.mark.parametrize("base_offset", [0, 3])
def test_long_batches_take_the_flat_first_pass(oracle, base_offset):
    """From 12 M elements in all the first pass runs as a grid in address order (chunks of four tiles per block of
    the dense grid): long and tiny tensors side by side, ragged ends, and - with an odd base offset - tensors that
    do not start on a 16-byte boundary and take the guarded element-wise accesses."""
    rng = np.random.default_rng(21 + base_offset)
    sizes = [1, 5_000_003, 17, 7_000_001, 256, 3_000_000, 63, 1025, 2_000_000]
    offs = [0] + [int(x) for x in np.cumsum(sizes)]
    g = rng.laplace(0, 1e-3, size=offs[-1]).astype(np.float32)
    r = rng.laplace(0, 3e-4, size=offs[-1]).astype(np.float32)
    for dist, stages, delta in ((0, 3, 0.01), (1, 2, 0.001), (2, 3, 0.001)):
        for res_in in (r, None):
            out = run_batched(g, res_in, offs, delta, dist, stages, base_offset=base_offset)
            check_batched(oracle, g, res_in, offs, delta, dist, stages, out,
                          f"flat batched dist={dist} M={stages} ec={res_in is not None} offset={base_offset}")


def test_one_long_tensor_among_many_short_ones_keeps_the_per_wave_first_pass(oracle):
    """400 short tensors leave the long one a fifth of the blocks: a flat grid would be mostly empty chunks, so the
    per-wave shape stays; the result does not depend on the choice."""
    rng = np.random.default_rng(23)
    sizes = [300] * 200 + [13_000_001] + [500] * 200
    offs = [0] + [int(x) for x in np.cumsum(sizes)]
    g = rng.laplace(0, 1e-3, size=offs[-1]).astype(np.float32)
    r = rng.laplace(0, 3e-4, size=offs[-1]).astype(np.float32)
    out = run_batched(g, r, offs, 0.01, 0, 2)
    check_batched(oracle, g, r, offs, 0.01, 0, 2, out, "one long among 400 short")


def test_sizes_from_one_element_to_millions(oracle):
    rng = np.random.default_rng(8)
    sizes = [1, 2, 63, 64, 255, 256, 257, 1000, 4099, 1, 70_001, 300_000, 5, 2_000_003, 17]
    offs = [0] + list(np.cumsum(sizes))
    g = rng.laplace(0, 1e-3, size=offs[-1]).astype(np.float32)
    r = rng.laplace(0, 3e-4, size=offs[-1]).astype(np.float32)
    for dist in (0, 1, 2):
        out = run_batched(g, r, offs, 0.01, dist, 3, base_offset=3)
        check_batched(oracle, g, r, offs, 0.01, dist, 3, out, f"sizes dist={dist}")


def test_512_tensors_and_one_tensor(oracle):
    rng = np.random.default_rng(9)
    sizes = rng.integers(1, 5000, size=512).tolist()
    offs = [0] + list(np.cumsum(sizes))
    g = (rng.standard_t(3.0, size=offs[-1]) * 1e-3).astype(np.float32)
    out = run_batched(g, np.zeros_like(g), offs, 0.02, 2, 2)
    check_batched(oracle, g, np.zeros_like(g), offs, 0.02, 2, 2, out, "512 tensors")
    g1 = rng.laplace(0, 1e-3, size=1_234_567).astype(np.float32)
    out = run_batched(g1, None, [0, g1.size], 0.001, 0, 3)
    check_batched(oracle, g1, None, [0, g1.size], 0.001, 0, 3, out, "one tensor")


def test_repeated_layout_and_layout_change(oracle):
    """The second identical call reuses the table on the device and the tensors' threshold hints; a different
    layout afterwards uploads a new table.  Results do not depend on either."""
    rng = np.random.default_rng(10)
    sizes = [400_001, 123_456, 999, 800_000]
    offs = [0] + list(np.cumsum(sizes))
    g = (rng.standard_t(3.0, size=offs[-1]) * 1e-3).astype(np.float32)
    r = rng.laplace(0, 1e-4, size=offs[-1]).astype(np.float32)
    first = run_batched(g, r, offs, 0.001, 2, 3)
    again = run_batched(g, r, offs, 0.001, 2, 3, repeat=3)
    check_batched(oracle, g, r, offs, 0.001, 2, 3, again, "repeated")
    for a, b in zip(first, again):
        np.testing.assert_array_equal(np.sort(a.idx), np.sort(b.idx))
        assert a.etas.tobytes() == b.etas.tobytes()
    offs2 = [0, 500_000, offs[-1]]
    out = run_batched(g, r, offs2, 0.001, 2, 3)
    check_batched(oracle, g, r, offs2, 0.001, 2, 3, out, "new layout")
