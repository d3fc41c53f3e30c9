"""Pins for the dense-Gaussian oracle: what the mathematics fixes about
S_ij ~ N(0, 1/k) i.i.d. (paper Sections 1 and 3)."""
import numpy as np
from scipy import stats

from oracle import gaussian as G


def test_moments_and_normality():
    k, d = 128, 2048
    S = G.gaussian_matrix(k, d, seed=0)
    z = S.ravel() * np.sqrt(k)
    n = z.size
    assert abs(z.mean()) < 4 / np.sqrt(n)
    assert abs(z.var() - 1.0) < 4 * np.sqrt(2.0 / n)
    assert abs(stats.skew(z)) < 4 * np.sqrt(6.0 / n)
    assert abs(stats.kurtosis(z)) < 4 * np.sqrt(24.0 / n)
    assert stats.kstest(z[:20000], "norm").pvalue > 1e-3
    # Box-Muller from 24-bit uniforms: tails are bounded by sqrt(2 ln 2^24)
    assert np.abs(z).max() <= np.sqrt(2 * np.log(2.0 ** 24)) + 1e-6


def test_entries_uncorrelated_and_seed_dependent():
    k, d = 64, 1024
    S = G.gaussian_matrix(k, d, seed=3) * np.sqrt(k)
    n = S.size
    for a, b in ((S[:, :-1], S[:, 1:]), (S[:-1], S[1:])):  # neighbours along rows / columns
        r = np.corrcoef(a.ravel(), b.ravel())[0, 1]
        assert abs(r) < 4 / np.sqrt(n)
    S2 = G.gaussian_matrix(k, d, seed=4) * np.sqrt(k)
    assert abs(np.corrcoef(S.ravel(), S2.ravel())[0, 1]) < 4 / np.sqrt(n)
    assert np.array_equal(G.gaussian_matrix(k, d, seed=3) * np.sqrt(k), S)  # deterministic


def test_norm_preserved_in_expectation():
    """E ||S x||^2 = ||x||^2 and the JL concentration 2/k of its variance."""
    k, d = 256, 512
    x = np.random.default_rng(0).standard_normal(d)
    r = np.array([(G.apply(G.gaussian_matrix(k, d, seed), x) ** 2).sum() / (x @ x) for seed in range(200)])
    assert abs(r.mean() - 1.0) < 4 * r.std(ddof=1) / np.sqrt(len(r))
    assert abs(r.var(ddof=1) / (2.0 / k) - 1.0) < 0.5


def test_apply_is_the_plain_product():
    S = G.gaussian_matrix(8, 16, seed=1)
    A = np.arange(16 * 3, dtype=np.float64).reshape(16, 3)
    want = np.array([[sum(S[i, t] * A[t, j] for t in range(16)) for j in range(3)] for i in range(8)])
    np.testing.assert_allclose(G.apply(S, A), want, rtol=1e-13)
