"""GPU parity of the decompression / aggregation step (Algorithm 2) against the oracle, bit for bit."""
import numpy as np
import pytest

from gpu_harness import run_gpu

pytestmark = pytest.mark.gpu


def test_aggregate_four_workers(oracle):
    import torch
    import paper_2101_10761_amd as sidco
    rng = np.random.default_rng(12)
    d, N = 1_000_003, 4
    dev = torch.device("cuda:0")
    dense = torch.zeros(d, dtype=torch.float32, device=dev)
    want = np.zeros(d, np.float32)
    ratios = oracle.schedule(0.001, 3, 0.25)
    for n in range(N):
        g = (rng.standard_t(3.0, size=d) * 1e-3).astype(np.float32)
        r = rng.laplace(0, 1e-4, size=d).astype(np.float32)
        out = run_gpu(g, r, 2, ratios)
        idx = torch.from_numpy(out.idx).to(dev)
        val = torch.from_numpy(out.val).to(dev)
        cnt = torch.tensor([out.count], dtype=torch.int32, device=dev)
        sidco.sidco_scatter_add(dense, idx, val, cnt, 1.0 / N)
        assert oracle.scatter_add(want, out.idx, out.val, 1.0 / N) == 0
        # one worker alone: pairs scattered onto zeros plus the updated residual give back acc exactly
        one = torch.zeros(d, dtype=torch.float32, device=dev)
        sidco.sidco_scatter_add(one, idx, val, cnt, 1.0)
        np.testing.assert_array_equal((one.cpu().numpy() + out.residual).view(np.uint32),
                                      oracle.ec_add(g, r).view(np.uint32))
    np.testing.assert_array_equal(dense.cpu().numpy().view(np.uint32), want.view(np.uint32))
    assert not sidco.sidco_scatter_check()


def test_count_is_read_on_the_device_and_bad_indices_are_skipped(oracle):
    import torch
    import paper_2101_10761_amd as sidco
    dev = torch.device("cuda:0")
    d = 1000
    dense = torch.arange(d, dtype=torch.float32, device=dev)
    idx = torch.tensor([5, -1, 999, 1000, 17, 3], dtype=torch.int32, device=dev)
    val = torch.tensor([1.0, 1.0, 2.0, 1.0, 4.0, 8.0], dtype=torch.float32, device=dev)
    for count in (0, 5, 6, 9):          # 9 > capacity: clipped to the six pairs there are
        got = dense.clone()
        sidco.sidco_scatter_add(got, idx, val, torch.tensor([count], dtype=torch.int32, device=dev), 0.5)
        want = np.arange(d, dtype=np.float32)
        n = min(count, 6)
        bad = oracle.scatter_add(want, idx.cpu().numpy()[:n], val.cpu().numpy()[:n], 0.5)
        np.testing.assert_array_equal(got.cpu().numpy(), want)
        assert sidco.sidco_scatter_check() == (bad > 0)
        assert not sidco.sidco_scatter_check()      # the flag is cleared by the check
