"""Pins of the oracle's DGC comparator (Sec. 1, related work: threshold from Top-k of a random subset, trimmed
by a second Top-k when it selects too many).  None of these re-calls the oracle's own routine: the generator is
checked against published outputs, the threshold and both selection branches against numpy's sort."""
import numpy as np
import pytest


# First outputs of the splitmix64 generator (Steele, Lea, Flood, "Fast splittable pseudorandom number
# generators", OOPSLA 2014; constants of Vigna's public-domain C version) for the seeds 0 and 1234567.
SPLITMIX_KNOWN = {
    0: [0xE220A8397B1DCDAF],
    1234567: [6457827717110365317, 3203168211198807973, 9817491932198370423, 4593380528125082431,
              16408922859458223821],
}


def test_generator_reproduces_published_outputs(oracle):
    for seed, outs in SPLITMIX_KNOWN.items():
        assert [oracle.splitmix64(seed, j) for j in range(len(outs))] == outs


def test_sample_indices_are_uniform_draws(oracle):
    d, n_s = 1_000_003, 20000
    idx = oracle.dgc_sample_indices(99, n_s, d)
    assert idx.min() >= 0 and idx.max() < d
    # the draw is floor(u * d / 2^32) of the generator's upper 32 bits
    want = [(oracle.splitmix64(99, j) >> 32) * d >> 32 for j in range(50)]
    assert idx[:50].tolist() == want
    counts = np.bincount(idx * 16 // d, minlength=16)
    chi2 = float(((counts - n_s / 16) ** 2 / (n_s / 16)).sum())
    assert chi2 < 45.0                       # 15 degrees of freedom: P(chi2 > 45) < 1e-4
    assert abs(idx.mean() / d - 0.5) < 0.01


def _laplace(seed, d, scale=1e-3):
    return np.random.Generator(np.random.PCG64(seed)).laplace(0.0, scale, d).astype(np.float32)


def test_sizes(oracle):
    assert oracle.dgc_sizes(1_000_000, 0.001, 0.01) == (10000, 10, 1000)
    assert oracle.dgc_sizes(269_722, 0.01, 0.01) == (2698, 27, 2698)
    assert oracle.dgc_sizes(10, 0.001, 0.01) == (1, 1, 1)


@pytest.mark.parametrize("seed", range(8))
def test_threshold_and_both_branches_against_numpy(oracle, seed):
    d, delta, rho = 200_003, 0.01, 0.02
    g = _laplace(seed, d)
    r = _laplace(100 + seed, d, 3e-4)
    acc = (g + r).astype(np.float32)
    n_s, k_s, k = oracle.dgc_sizes(d, delta, rho)
    out = oracle.dgc(g, r, delta=delta, sample_ratio=rho, seed=seed)
    sample = np.abs(acc[oracle.dgc_sample_indices(seed, n_s, d)])
    eta = np.sort(sample)[n_s - k_s]
    assert out.eta == eta
    above = np.flatnonzero(np.abs(acc) > eta)
    assert out.first_pass == above.size
    if above.size <= k:
        np.testing.assert_array_equal(out.idx, above)
    else:
        order = np.argsort(-np.abs(acc), kind="stable")[:k]   # continuous data: no ties at the cut
        np.testing.assert_array_equal(out.idx, np.sort(order))
    assert out.count == min(above.size, k) == out.idx.size
    np.testing.assert_array_equal(out.val, acc[out.idx])
    want_res = acc.copy()
    want_res[out.idx] = 0
    np.testing.assert_array_equal(out.residual, want_res)


def test_both_branches_occur_and_the_count_is_near_k(oracle):
    """The k_s-th largest of n_s draws sits near the (1 - delta) quantile: the first-pass count scatters around
    k with a relative spread of about 1/sqrt(k_s), above it about as often as below."""
    d, delta, rho = 400_000, 0.005, 0.05
    n_s, k_s, k = oracle.dgc_sizes(d, delta, rho)
    g = _laplace(7, d)
    first = np.array([oracle.dgc(g, None, delta=delta, sample_ratio=rho, seed=s).first_pass for s in range(24)])
    ratio = first / k
    assert (ratio > 1).sum() >= 4 and (ratio < 1).sum() >= 4
    assert np.all(np.abs(ratio - 1) < 5.0 / np.sqrt(k_s))
    assert abs(ratio.mean() - 1) < 2.5 / np.sqrt(k_s * 24) + 1.0 / k_s


def test_trim_with_ties_keeps_exactly_k(oracle):
    d = 1000
    g = np.full(d, 1e-3, dtype=np.float32)
    g[::7] = -5e-3                            # 143 large entries, all tied
    # a tiny subset: the threshold is the small magnitude unless a draw hits a large entry
    for seed in range(40):
        out = oracle.dgc(g, None, delta=0.05, sample_ratio=0.001, seed=seed)
        if out.eta == np.float32(1e-3):
            break
    else:
        pytest.fail("no seed drew a small entry")
    k = oracle.dgc_sizes(d, 0.05, 0.001)[2]
    assert k == 50 and out.first_pass == 143 and out.count == 50
    np.testing.assert_array_equal(out.idx, np.arange(0, d, 7)[:50])   # ties: lower index first
    assert np.all(out.val == np.float32(-5e-3))


def test_memoryless_leaves_no_residual_and_zero_gradient_selects_nothing(oracle):
    g = _laplace(3, 5000)
    out = oracle.dgc(g, None, delta=0.01, sample_ratio=0.1, seed=1)
    assert out.residual is None and out.count > 0
    z = oracle.dgc(np.zeros(5000, np.float32), np.zeros(5000, np.float32), delta=0.01, sample_ratio=0.1, seed=1)
    assert z.count == 0 and z.first_pass == 0 and z.eta == 0 and not z.residual.any()
