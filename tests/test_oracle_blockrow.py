"""Pins for the FlashBlockRow oracle (paper Appendix D, Alg. 2)."""
import math

import numpy as np
import pytest

from oracle import blockperm as O
from oracle import blockrow as R


@pytest.mark.parametrize("cfg", [(4096, 256, 512, 32, 2, 4), (1152, 72, 96, 6, 5, 3), (1000, 64, 128, 8, 8, 2)])
def test_row_structure(cfg):
    p = O.Params(*cfg)
    cols, signs = R.build_tables(p, 5)
    assert cols.shape == (p.k, p.kappa * p.s) and set(np.unique(signs)) <= {-1, 1}
    _, k1 = O.seed_keys(5)
    a, b = O.wiring(p.M, k1)
    for g in range(p.M):
        nb = O.neighbourhood(g, p.M, a, b, p.kappa)
        assert len(set(nb)) == p.kappa  # |N_row(g)| = kappa distinct blocks (Alg. 2)
        blk = cols[g * p.Br:(g + 1) * p.Br] // p.Bc
        for l, h in enumerate(nb):
            assert (blk[:, l * p.s:(l + 1) * p.s] == h).all()
    S = R.build_csr(p, 5)
    # every row: kappa*s updates of magnitude sqrt(d/k)/sqrt(kappa s), minus those in the padding;
    # entries are integer multiples of the scale (repeats add or cancel)
    q = S.toarray() / R.scale(p)
    np.testing.assert_allclose(q, np.round(q), atol=1e-12)
    in_range = (cols < p.d).sum(1)
    assert (np.abs(q).sum(1) <= in_range).all() and ((in_range - np.abs(q).sum(1)) % 2 == 0).all()


def test_brute_force_loops_equal_csr():
    p = O.Params(96, 24, 8, 2, 3, 2)
    seed = 9
    _, k1 = O.seed_keys(seed)
    a, b = O.wiring(p.M, k1)
    A = np.random.default_rng(1).standard_normal((p.d, 4))
    Y = np.zeros((p.k, 4))
    for g in range(p.M):
        for h in O.neighbourhood(g, p.M, a, b, p.kappa):
            bk = O.block_key(k1, g, h, p.M)
            for r in range(p.Br):
                for t in range(p.s):
                    w1 = O.mix32_int(bk ^ O.C1 ^ (r * 32 + t))
                    w2 = O.mix32_int(w1 ^ O.C2)
                    sign = 1.0 if w2 % 2 == 0 else -1.0
                    Y[g * p.Br + r] += sign * A[h * p.Bc + w1 % p.Bc]
    Y *= math.sqrt(p.d / p.k) / math.sqrt(p.kappa * p.s)
    np.testing.assert_allclose(R.apply(R.build_csr(p, seed), A), Y, rtol=1e-13, atol=1e-13)


def test_unbiased_norm_and_empty_columns():
    """E||Sx||^2 = ||x||^2, and -- the fragility the paper names -- a fraction of about
    exp(-k*kappa*s/d) of the input coordinates is never read."""
    p = O.Params(2048, 128, 256, 16, 4, 4)  # k*kappa*s = d
    rng = np.random.default_rng(2)
    x = rng.standard_normal((p.d, 1))
    ratios, empty = [], []
    for seed in range(400):
        S = R.build_csr(p, seed)
        ratios.append(float((R.apply(S, x) ** 2).sum() / (x ** 2).sum()))
        empty.append(float((np.diff(S.tocsc().indptr) == 0).mean()))
    ratios = np.array(ratios)
    assert abs(ratios.mean() - 1.0) < 4 * ratios.std(ddof=1) / math.sqrt(len(ratios))
    assert abs(np.mean(empty) - math.exp(-1.0)) < 0.02


def test_indices_uniform_over_the_block():
    p = O.Params(4096, 256, 512, 32, 2, 4)
    counts = np.zeros(p.Bc)
    for seed in range(20):
        cols, _ = R.build_tables(p, seed)
        counts += np.bincount((cols % p.Bc).ravel(), minlength=p.Bc)
    expected = counts.sum() / p.Bc
    chi2 = ((counts - expected) ** 2 / expected).sum()
    assert abs(chi2 - (p.Bc - 1)) < 5 * math.sqrt(2 * (p.Bc - 1))
