"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest

from gpu_harness import check_parity, run_gpu
from paper_2101_10761_amd import workloads

pytestmark = pytest.mark.gpu

DISTS = [0, 1, 2]


def _inputs(d, seed, scale=1e-3, heavy=False):
    rng = np.random.default_rng(seed)
    if heavy:
        g = (rng.standard_t(3.0, size=d) * scale).astype(np.float32)
    else:
        g = rng.laplace(0, scale, size=d).astype(np.float32)
    r = rng.laplace(0, 0.3 * scale, size=d).astype(np.float32)
    return g, r


# sizes: below one tile, exact tiles, ragged tails, several tiles per wave, more tiles than waves
SIZES = [1, 2, 63, 255, 256, 257, 1000, 4099, 70_001, 269_722, 1_048_576, 2_100_003]


@pytest.mark.parametrize("d", SIZES)
@pytest.mark.parametrize("dist", DISTS)
def test_small_sizes_all_laws(oracle, d, dist):
    g, r = _inputs(d, 100 + d % 97 + dist, heavy=(dist == 2))
    for stages, delta, delta1 in ((1, 0.05, 0.25), (3, 0.01, 0.25), (3, 0.002, 0.1)):
        ratios = oracle.schedule(delta, stages, delta1)
        for res_in in (r, None):
            out = run_gpu(g, res_in, dist, ratios)
            check_parity(oracle, g, res_in, dist, ratios, out, label=f"d={d} dist={dist} M={stages} ec={res_in is not None}")


@pytest.mark.parametrize("tiles_per_wave,tail", [(4, 100), (5, 0), (5, 100), (5, 255), (6, 1), (9, 17)])
def test_lengths_around_the_prefetching_dense_stage(oracle, tiles_per_wave, tail):
    """From 5 complete 256-element tiles per wave (4096 waves) the dense stages request their first tiles before
    the threshold is known and stay one batch ahead; the ragged last tile belongs to the last wave and is never
    part of such a request.  Ratios 0.25, 0.63, 0.63 make both directions run (stage 1 walks back, stage 2 forward)."""
    d = tiles_per_wave * 4096 * 256 + tail
    g, r = _inputs(d, 40 + tiles_per_wave + tail)
    for dist, ratios in ((0, oracle.schedule(0.1, 3, 0.25)), (2, oracle.schedule(0.001, 3, 0.25))):
        for res_in in (r, None):
            out = run_gpu(g, res_in, dist, ratios)
            check_parity(oracle, g, res_in, dist, ratios, out,
                         label=f"tiles/wave {tiles_per_wave} tail {tail} dist {dist} ec={res_in is not None}")


@pytest.mark.parametrize("goff,roff", [(1, 0), (0, 3), (1, 1), (2, 3)])
def test_unaligned_slices(oracle, goff, roff):
    """Per-tensor slices of a flat buffer start at any 4-byte boundary."""
    d = 300_007
    g, r = _inputs(d, 7)
    ratios = oracle.schedule(0.001, 2, 0.05)
    out = run_gpu(g, r, 0, ratios, grad_offset=goff, res_offset=roff)
    check_parity(oracle, g, r, 0, ratios, out, label=f"offsets {goff},{roff}")
    out = run_gpu(g, None, 2, ratios, grad_offset=goff)
    check_parity(oracle, g, None, 2, ratios, out, label=f"offset {goff} no-ec")


def test_config1_and_count_band(oracle):
    w = workloads.config1()
    out = run_gpu(w.grad, w.residual, w.dist, None, use_default_schedule=(w.delta, w.stages))
    ratios = oracle.schedule(w.delta, w.stages, 0.25)
    check_parity(oracle, w.grad, w.residual, w.dist, ratios, out, label="config1")
    k, sigma = w.delta * w.d, math.sqrt(w.d * w.delta * (1 - w.delta))
    assert abs(out.count - k) <= 4 * sigma
    assert out.eta == pytest.approx(1e-3 * math.log(100), rel=4 / math.sqrt(w.d))


@pytest.mark.parametrize("clustered", [False, True])
def test_config2_full_size(oracle, clustered):
    w = workloads.config2(clustered=clustered)
    ratios = oracle.schedule(w.delta, w.stages, w.delta1)
    out = run_gpu(w.grad, w.residual, w.dist, ratios, cap=w.d // 50)
    check_parity(oracle, w.grad, w.residual, w.dist, ratios, out, label=w.name)


def test_config3_full_size_default_schedule(oracle):
    """The benchmark's headline configuration, through sidco_compress exactly as bench.py calls it."""
    w = workloads.config3()
    out = run_gpu(w.grad, w.residual, w.dist, None, use_default_schedule=(w.delta, w.stages))
    ratios = oracle.schedule(w.delta, w.stages, 0.25)
    check_parity(oracle, w.grad, w.residual, w.dist, ratios, out, label="config3")
    assert 0.5 < out.count / (w.delta * w.d) < 1.5


def test_config4_whole_vector_and_per_tensor(oracle):
    w = workloads.config4(d=6_600_000, ragged=True)   # a tenth of the full length, 50 ragged unaligned tensors
    ratios = oracle.schedule(w.delta, w.stages, 0.25)
    out = run_gpu(w.grad, w.residual, w.dist, ratios)
    check_parity(oracle, w.grad, w.residual, w.dist, ratios, out, label="config4 whole")
    offs = w.tensor_offsets
    for t in (0, 7, 49):
        g = np.ascontiguousarray(w.grad[offs[t]:offs[t + 1]])
        out = run_gpu(g, np.zeros_like(g), w.dist, ratios, grad_offset=int(offs[t] % 4), res_offset=int(offs[t] % 4))
        check_parity(oracle, g, np.zeros_like(g), w.dist, ratios, out, label=f"config4 tensor {t}")


@pytest.mark.parametrize("delta", [0.1, 0.001])
def test_config5_iterated_with_carried_residual(oracle, delta):
    d = 13_835_754   # a tenth of the full length; the full length runs in test_config5_full_size
    r = np.zeros(d, np.float32)
    ratios = oracle.schedule(delta, 3, 0.25)
    for it in range(3):
        g = workloads.config5_grad(it, d)
        out = run_gpu(g, r, 0, ratios, cap=workloads_cap(d, delta))
        check_parity(oracle, g, r, 0, ratios, out, label=f"config5 it={it} delta={delta}")
        assert abs(out.count / (delta * d) - 1) < 0.2     # eq. (12) with the paper's 20 % tolerance
        r = out.residual


def workloads_cap(d, delta):
    import paper_2101_10761_amd as sidco
    return sidco.sidco_out_capacity(d, delta)


def test_config4_full_size(oracle):
    """Config 4 at full length, one call on the whole vector, compared element by element."""
    w = workloads.config4()
    out = run_gpu(w.grad, w.residual, w.dist, None, use_default_schedule=(w.delta, w.stages))
    check_parity(oracle, w.grad, w.residual, w.dist, oracle.schedule(w.delta, w.stages, 0.25), out, label="config4 full")


@pytest.mark.parametrize("delta", [0.1, 0.01, 0.001])
def test_config5_full_size_iterated(oracle, delta):
    """Config 5 as the benchmark configuration defines it: d = 138,357,544, a fresh Laplace gradient every
    iteration, the residual carried from one iteration to the next, three exponential stages, every iteration
    compared element by element (delta = 0.1 is the configuration whose output is heavy: 13.8 M pairs)."""
    import paper_2101_10761_amd as sidco
    d = 138_357_544
    r = np.zeros(d, np.float32)
    ratios = oracle.schedule(delta, 3, 0.25)
    cap = sidco.sidco_out_capacity(d, delta)
    for it in range(3):
        g = workloads.config5_grad(it, d)
        out = run_gpu(g, r, 0, ratios, cap=cap)
        check_parity(oracle, g, r, 0, ratios, out, capacity=cap, label=f"config5 full it={it} delta={delta}")
        assert abs(out.count / (delta * d) - 1) < 0.2     # eq. (12) with the paper's 20 % tolerance
        r = out.residual
        del g, out


# ----------------------------------------------------------------------------------------------
# edge and degenerate cases
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("stages", [1, 3])
def test_all_zero(oracle, dist, stages):
    g = np.zeros(5000, np.float32)
    ratios = oracle.schedule(0.01, stages, 0.25)
    out = run_gpu(g, g.copy(), dist, ratios)
    check_parity(oracle, g, g.copy(), dist, ratios, out, label="zeros")
    assert out.count == 0 and out.eta == 0.0


@pytest.mark.parametrize("dist", DISTS)
def test_constant_magnitude(oracle, dist):
    for c, n in ((0.25, 4096), (0.1, 77_777)):
        g = np.full(n, c, np.float32)
        g[::2] *= -1
        out = run_gpu(g, None, dist, [0.05])
        check_parity(oracle, g, None, dist, [0.05], out, label=f"const {c}")
        assert out.count == {0: 0, 1: n, 2: 0}[dist]


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("bad", [np.nan, np.inf, -np.inf])
def test_nonfinite_input(oracle, dist, bad):
    g, r = _inputs(10_000, 5)
    g[1234] = bad
    ratios = oracle.schedule(0.01, 2, 0.25)
    out = run_gpu(g, r, dist, ratios)
    check_parity(oracle, g, r, dist, ratios, out, label=f"nonfinite {bad}")
    assert out.count == 0 and math.isnan(out.eta) and out.status & 1


def test_planted_tie_on_the_threshold(oracle):
    """n entries of magnitude a and m entries b with b = L (n a + m b)/(n + m): the exponential threshold
    lands exactly on b, and the strict comparison must leave all of them out."""
    n, m, a, delta = 1000, 10, 1.0, 0.5
    L = math.log(1 / delta)
    b = np.float32(L * n * a / (n + m - L * m))
    g = np.concatenate([np.full(n, a, np.float32), np.full(m, b, np.float32)])
    g[::3] *= -1
    ref = oracle.compress(g, ratios=[delta], dist=0)
    assert np.float32(ref.eta) == b, "construction must put the threshold on b"
    out = run_gpu(g, g * 0, 0, [delta])
    check_parity(oracle, g, g * 0, 0, [delta], out, label="tie")
    assert np.float32(out.eta) == b
    assert out.count == n            # the a's (a > b) are kept, the b's (== eta) are not
    g2 = g.copy()
    g2[n] = np.nextafter(b, np.float32(2))   # one entry an ulp above the others: parity must still hold
    out2 = run_gpu(g2, None, 0, [delta])
    check_parity(oracle, g2, None, 0, [delta], out2, label="tie+1ulp")


def test_gamma_clamp_flag(oracle):
    """delta_1 * Gamma(alpha) >= 1 (shape ~ 0.2, delta_1 = 0.25): the closed form is clearly negative."""
    rng = np.random.default_rng(11)
    g = rng.gamma(0.2, 1e-3, size=200_000).astype(np.float32)
    out = run_gpu(g, None, 1, [0.25, 0.1])
    check_parity(oracle, g, None, 1, [0.25, 0.1], out, label="gamma clamp")
    assert out.status & 8 and out.etas[0] == 0.0


def test_refinement_stops(oracle):
    g = np.full(100_000, 1e-3, np.float32)
    g[5] = 10.0
    ratios = oracle.schedule(0.001, 3, 0.25)
    for dist in DISTS:
        out = run_gpu(g, None, dist, ratios)
        check_parity(oracle, g, None, dist, ratios, out, label=f"stop dist={dist}")


def test_output_overflow_is_safe(oracle):
    g, r = _inputs(500_000, 11)
    ratios = oracle.schedule(0.01, 2, 0.25)
    for cap in (1, 100, 4999):
        out = run_gpu(g, r, 0, ratios, cap=cap)
        check_parity(oracle, g, r, 0, ratios, out, capacity=cap, label=f"overflow cap={cap}")


def test_deterministic_and_workspace_reuse(oracle):
    """Same input twice -> same thresholds, same selected set, same values (the order of the pairs may differ
    for M >= 2 and is fixed for M = 1), also after a larger and a smaller call in between (the workspace
    keeps stale lists), and with a caller-provided workspace."""
    import torch
    import paper_2101_10761_amd as sidco
    g, r = _inputs(1_500_000, 21, heavy=True)
    ratios = oracle.schedule(0.001, 3, 0.25)
    a = run_gpu(g, r, 2, ratios)
    big, rb = _inputs(3_000_000, 22)
    run_gpu(big, rb, 0, oracle.schedule(0.1, 2, 0.25))
    small, rs = _inputs(999, 23)
    run_gpu(small, rs, 1, [0.05])
    b = run_gpu(g, r, 2, ratios)

    def same(x, y, ordered=False):
        ox, oy = (slice(None), slice(None)) if ordered else (np.argsort(x.idx), np.argsort(y.idx))
        np.testing.assert_array_equal(x.idx[ox], y.idx[oy])
        np.testing.assert_array_equal(x.val[ox].view(np.uint32), y.val[oy].view(np.uint32))
        assert x.etas.tobytes() == y.etas.tobytes()
        np.testing.assert_array_equal(x.residual.view(np.uint32), y.residual.view(np.uint32))

    same(a, b)
    s1 = run_gpu(g, r, 2, [0.001])
    s2 = run_gpu(g, r, 2, [0.001])
    same(s1, s2, ordered=True)
    check_parity(oracle, g, r, 2, ratios, b, label="reuse")
    ws = torch.empty(sidco.sidco_workspace_bytes(g.size), dtype=torch.uint8, device="cuda:0")
    assert ws.data_ptr() % 256 == 0
    sidco.sidco_set_workspace(ws)
    try:
        c = run_gpu(g, r, 2, ratios)
        same(a, c)
        with pytest.raises(sidco.SidcoError) as e:
            run_gpu(big, rb, 0, ratios)   # needs more than the provided workspace
        assert e.value.code == -6
    finally:
        sidco.sidco_set_workspace(None)
    d2 = run_gpu(g, r, 2, ratios)
    same(a, d2)


def test_eight_stages(oracle):
    g, r = _inputs(2_000_000, 31)
    ratios = oracle.schedule(1e-4, 8, 0.25)
    out = run_gpu(g, r, 0, ratios)
    check_parity(oracle, g, r, 0, ratios, out, label="M=8")


def test_profile_hooks():
    import paper_2101_10761_amd as sidco
    g, r = _inputs(1_000_000, 41)
    sidco.sidco_set_profiling(True)
    try:
        run_gpu(g, r, 0, [0.25, 0.04])
        prof = sidco.sidco_get_profile()
    finally:
        sidco.sidco_set_profiling(False)
    # delta_1 = 0.25 keeps too much to be worth writing out, but the candidates for the next stage
    # (quantile of the same fit at 0.25 * sqrt(0.04) = 0.05) are: stage 1 sums over the exceedances of
    # eta_1 and writes the candidate lists, the last stage reads those
    assert [n for n, _ in prof] == ["k_fit", "k_compact_dense", "k_final_lists"]
    assert all(0 < ms < 50 for _, ms in prof)
    seen = {}
    sidco.sidco_set_profiling(True)
    try:
        for ratios in ([0.25, 0.2, 0.2], [0.5, 0.5, 0.5, 0.02], [0.1, 0.3, 0.3], [0.01]):
            run_gpu(g, r, 0, ratios)
            seen[tuple(ratios)] = [n for n, _ in sidco.sidco_get_profile()]
    finally:
        sidco.sidco_set_profiling(False)
    assert seen[(0.25, 0.2, 0.2)] == ["k_fit", "k_compact_dense", "k_lists", "k_final_lists"]
    assert seen[(0.5, 0.5, 0.5, 0.02)] == ["k_fit", "k_scan_dense", "k_scan_dense", "k_compact_dense", "k_final_lists"]
    assert seen[(0.1, 0.3, 0.3)] == ["k_fit", "k_compact_dense", "k_lists", "k_final_lists"]
    assert seen[(0.01,)] == ["k_fit", "k_compact_dense", "k_gather"]


def _light_tailed(d, seed, lo=0.0, hi=2e-3):
    """Magnitudes uniform on [lo, hi]: far lighter-tailed than an exponential law.  On [0, 2e-3] the mean is
    1e-3, the exponential eta_1 at delta_1 = 0.25 is 1.386e-3, and the mean excess over it is 0.31e-3, under
    a third of the 1e-3 the fit predicts: the next threshold lands below the candidate threshold.  On a narrow
    band such as [0.9e-3, 1.1e-3] nothing exceeds eta_1 at all."""
    rng = np.random.default_rng(seed)
    g = (rng.uniform(lo, hi, size=d) * rng.choice([-1.0, 1.0], size=d)).astype(np.float32)
    return g


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("ratios", [[0.25, 0.2], [0.25, 0.2, 0.2], [0.05, 0.2]])
@pytest.mark.parametrize("band", [(0.0, 2e-3), (0.9e-3, 1.1e-3)])
def test_candidate_lists_fall_back_to_the_dense_vector(oracle, dist, ratios, band):
    """Speculative candidate lists (see sidco_set_speculation) never change the result: on light-tailed input
    the next threshold lands below the candidate threshold and the stage reads the dense vector again; on
    well-modelled input it does not; with theta = 0 it never does.  Parity holds in all three."""
    import paper_2101_10761_amd as sidco
    d = 700_001
    g = _light_tailed(d, 51, *band)
    r = np.zeros(d, np.float32)
    out = run_gpu(g, r, dist, ratios)
    check_parity(oracle, g, r, dist, ratios, out, label=f"light tail dist={dist} {ratios}")
    if dist == 0:   # exponential chain: the mean excess is under half of the model's, or nothing exceeds eta_1
        assert out.status & sidco.ST_FALLBACK
        if band[0] == 0.0 and ratios[0] == 0.25:
            assert out.count > 0.01 * d
    g2, r2 = _inputs(d, 52, heavy=(dist == 2))
    run_gpu(g2[:1000], None, dist, [0.1])     # another shape in between: the next call starts without a hint
    out2 = run_gpu(g2, r2, dist, ratios)
    check_parity(oracle, g2, r2, dist, ratios, out2, label=f"modelled dist={dist} {ratios}")
    if dist != 1:   # Laplace under the exponential chain, Student-t under the GPD chain: the law fits
        assert not out2.status & sidco.ST_FALLBACK
    sidco.sidco_set_speculation(0.0)
    try:
        out3 = run_gpu(g, r, dist, ratios)
        check_parity(oracle, g, r, dist, ratios, out3, label=f"theta=0 dist={dist} {ratios}")
        assert not out3.status & sidco.ST_FALLBACK
        np.testing.assert_array_equal(np.sort(out3.idx), np.sort(out.idx))
        assert out3.etas.tobytes() == out.etas.tobytes()
        sidco.sidco_set_speculation(1.0)
        out4 = run_gpu(g2, r2, dist, ratios)      # a changed theta is a changed shape: no hint either
        check_parity(oracle, g2, r2, dist, ratios, out4, label=f"theta=1 dist={dist} {ratios}")
        np.testing.assert_array_equal(np.sort(out4.idx), np.sort(out2.idx))
    finally:
        sidco.sidco_set_speculation(0.5)


@pytest.mark.parametrize("dist", [0, 2])
def test_repeated_calls_take_the_previous_thresholds_as_a_hint(oracle, dist):
    """A call that repeats the previous call's shape (same d, law, ratios) places its candidate threshold where
    the previous call's next threshold fell.  Results never depend on that: the same input gives the same
    output whatever ran before, and a change of distribution under the same shape falls back to the dense
    vector and still matches the oracle."""
    import paper_2101_10761_amd as sidco
    d = 900_001
    gh, rh = _inputs(d, 61, heavy=True)
    gl, rl = _light_tailed(d, 62), np.zeros(d, np.float32)
    ratios = [0.25, 0.2, 0.2]
    run_gpu(gh[:1000], None, dist, [0.1])                     # another shape: the next call starts without a hint
    outs = []
    for g, r, label in ((gh, rh, "unhinted"), (gh, rh, "hinted"), (gl, rl, "hint from another distribution"),
                        (gh, rh, "hint from the light-tailed call"), (gh, rh, "hinted again")):
        out = run_gpu(g, r, dist, ratios)
        check_parity(oracle, g, r, dist, ratios, out, label=f"{label} dist={dist}")
        outs.append(out)
    for o in (outs[1], outs[3], outs[4]):
        np.testing.assert_array_equal(np.sort(o.idx), np.sort(outs[0].idx))
        assert o.etas.tobytes() == outs[0].etas.tobytes()
        np.testing.assert_array_equal(o.residual.view(np.uint32), outs[0].residual.view(np.uint32))
    assert not outs[0].status & sidco.ST_FALLBACK and not outs[1].status & sidco.ST_FALLBACK
    assert not outs[4].status & sidco.ST_FALLBACK
    if dist == 0:
        assert outs[2].status & sidco.ST_FALLBACK             # exponential fit of uniform magnitudes


def test_fallback_in_the_last_stage_respects_capacity_and_ragged_ends(oracle):
    """The last stage's dense fallback on an unaligned, ragged vector, with and without output overflow."""
    d = 333_337
    g = _light_tailed(d, 53)
    for cap in (None, 50):
        run_gpu(g[:1000], None, 0, [0.1])     # another shape in between: the next call starts without a hint
        out = run_gpu(g, np.zeros(d, np.float32), 0, [0.25, 0.2], cap=cap, grad_offset=1, res_offset=3)
        check_parity(oracle, g, np.zeros(d, np.float32), 0, [0.25, 0.2], out, capacity=cap, label=f"fallback cap={cap}")
        assert out.status & 64 and out.selected > 0.02 * d
    # the same call again: the hint now says how low the next threshold falls, and the lists reach down to it
    again = run_gpu(g, np.zeros(d, np.float32), 0, [0.25, 0.2], cap=50, grad_offset=1, res_offset=3)
    check_parity(oracle, g, np.zeros(d, np.float32), 0, [0.25, 0.2], again, capacity=50, label="fallback learnt")
    assert not again.status & 64


@pytest.mark.parametrize("dist", DISTS)
@pytest.mark.parametrize("d,off", [(1, 0), (257, 0), (1_000_003, 0), (3_000_001, 1), (25_557_032, 0),
                                   (100_000_003, 0)])   # the last one takes the large-vector launch shape
def test_fit_alone(oracle, dist, d, off):
    """Steps 1-2 on their own: acc bit-exact (one fp32 add), sums within 1e-5 of the oracle's moments."""
    import torch
    import paper_2101_10761_amd as sidco
    g, r = _inputs(d, 300 + dist, heavy=(dist == 2))
    gbuf = torch.zeros(d + off, dtype=torch.float32, device="cuda:0")
    rbuf = torch.zeros(d + off, dtype=torch.float32, device="cuda:0")
    gt, rt = gbuf[off:], rbuf[off:]
    gt.copy_(torch.from_numpy(g))
    rt.copy_(torch.from_numpy(r))
    sidco.sidco_fit(gt, rt, dist)
    s1, s2, sl, n = sidco.sidco_fit_result()
    acc = oracle.ec_add(g, r)
    np.testing.assert_array_equal(rt.cpu().numpy().view(np.uint32), acc.view(np.uint32))
    np.testing.assert_array_equal(gt.cpu().numpy().view(np.uint32), g.view(np.uint32))
    mu, var, mulog = oracle.moments_all(acc)
    assert n == d
    assert s1 / d == pytest.approx(mu, rel=1e-5)
    if dist == 2:
        assert s2 / d - (s1 / d) ** 2 == pytest.approx(var, rel=1e-5)
    if dist == 1:
        assert sl / d == pytest.approx(mulog, rel=1e-5)
        assert sl / d == pytest.approx(mulog, abs=2e-7)     # hardware log2 only sees mantissas in [0.5, 1)
    # memoryless: nothing is written
    sidco.sidco_fit(gt, None, dist)
    s1b, _, _, _ = sidco.sidco_fit_result()
    assert s1b / d == pytest.approx(float(np.abs(g.astype(np.float64)).mean()), rel=1e-5)
