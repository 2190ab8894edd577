"""GPU: workspaces per stream, the reserve call, the status word, delta_1 of the default schedule, and the
stage controller's window stamp - all through the C ABI, results against the CPU oracle."""
import numpy as np
import pytest

from gpu_harness import GpuCall, check_parity, run_gpu
from paper_2101_10761_amd import workloads

pytestmark = pytest.mark.gpu


def _inputs(d, seed, heavy=False):
    rng = np.random.default_rng(seed)
    g = (rng.standard_t(3.0, size=d) * 1e-3).astype(np.float32) if heavy else rng.laplace(0, 1e-3, size=d).astype(np.float32)
    r = rng.laplace(0, 3e-4, size=d).astype(np.float32)
    return g, r


def test_two_streams_compress_different_vectors_concurrently(oracle):
    """Each stream has its own workspace: calls that overlap on two streams do not disturb each other, and
    the diagnostics of a stream are those of its own last call."""
    import torch
    ga, ra = _inputs(3_000_001, 1, heavy=True)
    gb, rb = _inputs(1_700_003, 2)
    ratios_a, ratios_b = oracle.schedule(0.001, 3, 0.25), oracle.schedule(0.01, 2, 0.25)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):   # the second and third round run with threshold hints, each from its own stream's history
        a, b = GpuCall(ga, ra, 2, ratios_a), GpuCall(gb, rb, 0, ratios_b)
        a.launch(s1)
        b.launch(s2)
        a2 = GpuCall(gb, rb, 0, ratios_b).launch(s1)   # a different shape behind the first call of stream 1
        b2 = GpuCall(ga, ra, 2, ratios_a).launch(s2)
        torch.cuda.synchronize()
        out_a2, out_b2 = a2.collect(s1), b2.collect(s2)
        check_parity(oracle, gb, rb, 0, ratios_b, out_a2, label=f"stream 1 second call, round {rep}")
        check_parity(oracle, ga, ra, 2, ratios_a, out_b2, label=f"stream 2 second call, round {rep}")
        # the first calls' outputs (the diagnostics now belong to the second calls: compare the outputs alone)
        for call, g, r, dist, ratios in ((a, ga, ra, 2, ratios_a), (b, gb, rb, 0, ratios_b)):
            k = int(call.out_count.item())
            eta = np.float32(call.out_eta.item())
            ref = oracle.compress(g, r, ratios=list(ratios), dist=dist, eta_inject=np.full(len(ratios), eta, np.float32))
            assert k == ref.count
            np.testing.assert_array_equal(np.sort(call.out_idx[:k].cpu().numpy()), ref.idx)
            np.testing.assert_array_equal(call.rt.cpu().numpy().view(np.uint32), ref.residual.view(np.uint32))


def test_reserve_release_and_caller_workspace(oracle):
    import torch
    import paper_2101_10761_amd as sidco
    g, r = _inputs(2_000_000, 3)
    ratios = oracle.schedule(0.001, 2, 0.25)
    s = torch.cuda.Stream()
    need = sidco.sidco_workspace_bytes(g.size)
    call = GpuCall(g, r, 0, ratios)
    free0 = torch.cuda.mem_get_info()[0]
    sidco.sidco_reserve(need, stream=s)
    free1 = torch.cuda.mem_get_info()[0]
    assert free0 - free1 >= 0.9 * need
    out = call.launch(s).collect(s)
    assert torch.cuda.mem_get_info()[0] == free1         # the call itself allocated nothing
    check_parity(oracle, g, r, 0, ratios, out, label="reserved")
    sidco.sidco_release(stream=s)
    assert torch.cuda.mem_get_info()[0] >= free1 + 0.9 * need   # the stream's workspace is gone
    with pytest.raises(sidco.SidcoError) as e:
        sidco.sidco_read_diag(stream=s)                  # and with it the record of its last call
    assert e.value.code == -6
    out = GpuCall(g, r, 0, ratios).launch(s).collect(s)  # a later call allocates again
    check_parity(oracle, g, r, 0, ratios, out, label="after release")
    sidco.sidco_release(stream=s)


def test_status_word_reports_overflow_without_a_host_round_trip(oracle):
    import torch
    import paper_2101_10761_amd as sidco
    g, r = _inputs(600_000, 4)
    word = torch.full((1,), 0x7fffffff, dtype=torch.int32, device="cuda:0")
    sidco.sidco_set_status_word(word)
    try:
        for ratios, cap in (([0.25, 0.04], 100), ([0.01], 7), ([0.25, 0.2, 0.2], None)):
            out = run_gpu(g, r, 0, ratios, cap=cap)
            check_parity(oracle, g, r, 0, ratios, out, capacity=cap, label=f"status word {ratios}")
            assert int(word.item()) == out.status          # the OVERFLOW bit included
            assert bool(int(word.item()) & sidco.ST_OVERFLOW) == (cap is not None)
    finally:
        sidco.sidco_set_status_word(None)
    word.fill_(5)
    run_gpu(g, r, 0, [0.01])
    assert int(word.item()) == 5                           # switched off: not written any more


def test_config2_through_the_default_schedule_with_its_own_delta1(oracle):
    """Config 2 (delta_1 = 0.05) through sidco_compress: the default schedule's delta_1 is a setting."""
    import paper_2101_10761_amd as sidco
    w = workloads.config2()
    sidco.sidco_set_delta1(w.delta1)
    try:
        out = run_gpu(w.grad, w.residual, w.dist, None, use_default_schedule=(w.delta, w.stages))
    finally:
        sidco.sidco_set_delta1(0.25)
    ratios = oracle.schedule(w.delta, w.stages, w.delta1)
    assert ratios[0] == pytest.approx(0.05)
    check_parity(oracle, w.grad, w.residual, w.dist, ratios, out, label="config2 via sidco_compress")
    d1 = sidco.sidco_get_diag()
    d2 = sidco.sidco_read_diag()
    assert bytes(d1) == bytes(d2)


def test_controller_notices_foreign_calls_in_its_window(oracle):
    import torch
    import paper_2101_10761_amd as sidco
    d = 400_000
    rng = np.random.default_rng(9)
    dev = torch.device("cuda:0")
    cap = sidco.sidco_out_capacity(d, 0.01)
    oi = torch.empty(cap, dtype=torch.int32, device=dev)
    ov = torch.empty(cap, dtype=torch.float32, device=dev)
    oc = torch.zeros(1, dtype=torch.int32, device=dev)
    oe = torch.zeros(1, dtype=torch.float32, device=dev)
    res = torch.zeros(d, dtype=torch.float32, device=dev)
    c = sidco.Controller(0.01, 0, stages=1, max_stages=4, Q=3)
    other = sidco.Controller(0.01, 0, stages=1, max_stages=4, Q=3)
    grads = [torch.from_numpy(rng.normal(0, 1e-3, size=d).astype(np.float32)).to(dev) for _ in range(6)]
    for it in range(3):                       # an undisturbed window: the controller adapts
        c.compress(grads[it], res, oi, ov, oc, oe)
    assert c.disturbed == 0 and c.last_average >= 0
    m_after_first = c.stages
    for it in range(3):                       # a window with another controller's call on the same stream inside
        c.compress(grads[3 + it], res, oi, ov, oc, oe)
        if it == 1:
            other.compress(grads[0], torch.zeros_like(res), oi, ov, oc, oe)
    assert c.disturbed == 1 and c.stages == m_after_first
    s2 = torch.cuda.Stream()                  # the other controller on a stream of its own disturbs nothing
    res2, oi2, ov2, oc2, oe2 = torch.zeros_like(res), oi.clone(), ov.clone(), oc.clone(), oe.clone()
    torch.cuda.synchronize()
    for it in range(3):
        c.compress(grads[it], res, oi, ov, oc, oe)
        other.compress(grads[it], res2, oi2, ov2, oc2, oe2, stream=s2)
    torch.cuda.synchronize()
    assert c.disturbed == 1
    c.close()
    other.close()
