"""GPU parity of the sparsifier with its stage controller (Algorithm 1 as a whole) against the oracle's loop."""
import numpy as np
import pytest

from gpu_harness import check_parity, GpuResult

pytestmark = pytest.mark.gpu


def _run_controller(grads, residual0, *, delta, dist, stages, max_stages, Q, eps=0.2, delta1=0.25):
    """Drives sidco_controller_compress over the gradients; returns per iteration (stages used, GpuResult)."""
    import torch
    import paper_2101_10761_amd as sidco
    dev = torch.device("cuda:0")
    d = grads[0].numel() if isinstance(grads[0], torch.Tensor) else grads[0].size
    ctrl = sidco.Controller(delta, dist, stages=stages, max_stages=max_stages, Q=Q, eps_high=eps, eps_low=eps,
                            delta1=delta1)
    cap = sidco.sidco_out_capacity(d, delta)
    rt = None if residual0 is None else torch.from_numpy(residual0.copy()).to(dev)
    out_idx = torch.empty(cap, dtype=torch.int32, device=dev)
    out_val = torch.empty(cap, dtype=torch.float32, device=dev)
    out_count = torch.zeros(1, dtype=torch.int32, device=dev)
    out_eta = torch.zeros(1, dtype=torch.float32, device=dev)
    out = []
    for i, g in enumerate(grads, start=1):
        M = ctrl.stages
        assert ctrl.iteration == i - 1
        ctrl.compress((g if isinstance(g, torch.Tensor) else torch.from_numpy(g)).to(dev), rt, out_idx, out_val,
                      out_count, out_eta)
        diag = sidco.sidco_read_diag()
        k = int(out_count.item())
        Md = diag.stages
        out.append((M, GpuResult(
            idx=out_idx[:k].cpu().numpy(), val=out_val[:k].cpu().numpy(), count=k, eta=float(out_eta.item()),
            residual=None if rt is None else rt.cpu().numpy(),
            etas=np.array(diag.eta[:Md], dtype=np.float32), n=np.array(diag.n[:Md], dtype=np.int64),
            stats=np.array([[diag.stats[m][q] for q in range(3)] for m in range(Md)]), status=diag.status,
            selected=diag.selected), ctrl.last_average))
    ctrl.close()
    return out


@pytest.mark.parametrize("dist,kind", [(0, "gauss"), (2, "gauss"), (0, "laplace")])
def test_controller_follows_the_oracle_loop(oracle, dist, kind):
    rng = np.random.default_rng(91)
    d, delta, Q, W = 400_003, 0.001, 5, 6
    draw = (lambda: rng.standard_normal(d) * 1e-3) if kind == "gauss" else (lambda: rng.laplace(0, 1e-3, size=d))
    grads = [draw().astype(np.float32) for _ in range(W * Q)]
    r0 = np.zeros(d, np.float32)
    got = _run_controller(grads, r0, delta=delta, dist=dist, stages=1, max_stages=6, Q=Q)
    ref = oracle.adaptive_run(grads, r0, delta=delta, dist=dist, stages=1, max_stages=6, Q=Q)
    assert [m for m, _, _ in got] == [m for m, _ in ref]
    r = r0
    window = []
    for i, ((M, out, last_avg), (_, o)) in enumerate(zip(got, ref), start=1):
        ratios = oracle.schedule(delta, M, 0.25)
        check_parity(oracle, grads[i - 1], r, dist, ratios, out, label=f"controller it={i} M={M}")
        assert out.count == o.count
        r = out.residual
        window.append(out.count)
        if i % Q == 0:
            assert last_avg == pytest.approx(np.mean(window), rel=1e-12)   # all Q counts of the window
            window = []
    if kind == "gauss" and dist == 0:
        assert [m for m, _, _ in got][::Q][:4] == [1, 2, 3, 4]
