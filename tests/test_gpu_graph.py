"""A sparsifier call captured into a HIP graph (through torch's stream capture) and replayed: the library's
calls only enqueue kernels - no allocation, no synchronisation, no memset node once the workspace exists - so a
launch-bound training loop can replay them.  Every replay is checked against the oracle, with eager work and
synchronisations between the replays."""
import numpy as np
import pytest

from gpu_harness import GpuResult, check_parity

pytestmark = pytest.mark.gpu


def _vec(seed, d):
    rng = np.random.Generator(np.random.PCG64(seed))
    return (rng.standard_t(3.0, d) * 1e-3).astype(np.float32)


@pytest.mark.parametrize("d,dist,delta,stages", [(269_722, 0, 0.01, 1), (1_000_003, 2, 0.002, 3), (13_000_000, 1, 0.001, 2)])
def test_captured_call_replays_correctly(oracle, d, dist, delta, stages):
    import torch
    import paper_2101_10761_amd as sidco

    dev = torch.device("cuda:0")
    ratios = sidco.sidco_stage_ratios(delta, stages)
    cap = sidco.sidco_out_capacity(d, delta)
    g = torch.zeros(d, dtype=torch.float32, device=dev)
    r = torch.zeros(d, dtype=torch.float32, device=dev)
    out_idx = torch.full((cap,), -7, dtype=torch.int32, device=dev)
    out_val = torch.full((cap,), 7.0, dtype=torch.float32, device=dev)
    out_count = torch.zeros(1, dtype=torch.int32, device=dev)
    out_eta = torch.zeros(1, dtype=torch.float32, device=dev)

    host_g = _vec(1, d)
    host_r = np.zeros(d, np.float32)
    g.copy_(torch.from_numpy(host_g))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    # the capturing stream's workspace is allocated outside the capture
    sidco.sidco_reserve(sidco.sidco_workspace_bytes(d), stream=side)
    torch.cuda.synchronize()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin()
        sidco.sidco_compress(g, r, delta, dist, stages, out_idx, out_val, out_count, out_eta, stream=side)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for it in range(4):
        host_g = _vec(10 + it, d)                       # new data in the same buffers
        g.copy_(torch.from_numpy(host_g))
        out_idx.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        diag = sidco.sidco_read_diag(stream=side)
        k = int(out_count.item())
        M = diag.stages
        res = GpuResult(idx=out_idx[:k].cpu().numpy(), val=out_val[:k].cpu().numpy(), count=k,
                        eta=float(out_eta.item()), residual=r.cpu().numpy(),
                        etas=np.array(diag.eta[:M], dtype=np.float32), n=np.array(diag.n[:M], dtype=np.int64),
                        stats=np.array([[diag.stats[m][q] for q in range(3)] for m in range(M)]),
                        status=diag.status, selected=diag.selected)
        ref = check_parity(oracle, host_g, host_r, dist, ratios, res, capacity=cap, label=f"replay {it} d {d}")
        host_r = ref.residual
        assert torch.all(out_idx[k:] == -7)
        # eager work of the library on the same workspace between replays must not disturb the next replay
        sidco.sidco_fit(g, None, dist, stream=side)
        torch.cuda.synchronize()
    sidco.sidco_release(stream=side)
