"""Pins for the CPU oracle: values the paper prints, closed forms, invariants,
special cases and brute force.  None of these tests touches the HIP path.

Citations are to the paper: Section 4 (sketch definition, Fig. 2), Appendix A
(energy identity, block output equation, coherence bounds), Appendix E
(wiring, full-period conditions, within-block hashing).
"""
import math
import os

import numpy as np
import pytest

from oracle import blockperm as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")

PARAM_GRID = [
    # d, k, Bc, Br, kappa, s
    (4096, 256, 512, 32, 2, 4),     # tiny benchmark config
    (2048, 1024, 128, 64, 4, 2),    # Fig. 2
    (1024, 64, 1024, 64, 1, 8),     # M = 1: plain SJLT
    (1152, 72, 96, 6, 5, 3),        # M = 12 (composite), Br not a power of two
    (1440, 180, 80, 10, 18, 10),    # M = 18, kappa = M, s = Br
    (512, 512, 1, 1, 3, 1),         # Br = Bc = 1
    (4096, 64, 512, 8, 8, 2),       # kappa = M = 8, gradient-config block shape
    (4000, 256, 512, 32, 2, 4),     # d not a multiple of Bc: last input block partly filled
    (1100, 72, 96, 6, 5, 3),        # the same with composite M and odd Br
]


def _read_kv(path):
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            out[k.strip()] = int(v)
    return out


# ---------------------------------------------------------------- P11 -----
def test_spec_words_fixture():
    p = O.Params(4096, 256, 512, 32, 2, 4)
    _, k1 = O.seed_keys(0)
    a, b = O.wiring(p.M, k1)
    S = None
    for line in open(os.path.join(GOLD, "spec_words.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        lhs, rhs = [t.strip() for t in line.split("=")]
        name, *args = lhs.split()
        if name == "mix32":
            x = int(args[0], 16)
            assert O.mix32_int(x) == int(rhs, 16)
            assert int(O.mix32(np.array([x], dtype=np.uint32))[0]) == int(rhs, 16)
        elif name == "keys":
            assert O.seed_keys(int(args[0])) == tuple(int(t, 16) for t in rhs.split())
        elif name == "k1":
            assert O.seed_keys(int(args[0]))[1] == int(rhs, 16)
        elif name == "wiring":
            kk = O.seed_keys(int(args[0]))[1]
            assert O.wiring(int(args[1]), kk) == tuple(int(t) for t in rhs.split())
        elif name == "nbr":
            assert O.neighbourhood(int(args[0]), p.M, a, b, p.kappa) == [int(t) for t in rhs.split()]
        elif name == "blockkey":
            assert O.block_key(k1, int(args[0]), int(args[1]), p.M) == int(rhs, 16)
        elif name == "rowhash":
            bk = O.block_key(k1, int(args[0]), int(args[1]), p.M)
            h1 = O.mix32_int(bk ^ int(args[2]))
            assert (h1, O.mix32_int(h1 ^ O.C2)) == tuple(int(t, 16) for t in rhs.split())
        elif name == "rows":
            bk = O.block_key(k1, int(args[0]), int(args[1]), p.M)
            r, sg = O.row_targets(np.uint32(bk), np.uint32(int(args[2])), p.Br, p.s)
            want_r, want_s = rhs.split(";")
            assert list(r) == [int(t) for t in want_r.split()]
            assert list(sg) == [1 if t == "+" else -1 for t in want_s.split()]
        elif name == "column":
            S = S if S is not None else O.build_csc(p, 0)
            col = S[:, int(args[0])].tocoo()
            assert sorted(col.row.tolist()) == [int(t) for t in rhs.split()]
            np.testing.assert_allclose(np.abs(col.data), 1 / math.sqrt(8))
        else:
            raise AssertionError(f"unknown fixture line {line}")


def test_mix32_scalar_and_vector_agree_and_avalanche():
    rng = np.random.default_rng(0)
    x = rng.integers(0, 2**32, size=4096, dtype=np.uint64).astype(np.uint32)
    v = O.mix32(x)
    assert [O.mix32_int(int(t)) for t in x[:256]] == [int(t) for t in v[:256]]
    assert len(np.unique(v)) == len(np.unique(x))  # bijective mixer: no collisions
    for bit in (0, 7, 16, 31):
        flipped = O.mix32(x ^ np.uint32(1 << bit)) ^ v
        frac = np.unpackbits(flipped.view(np.uint8)).mean()
        assert 0.48 < frac < 0.52


# ----------------------------------------------------------------- P1 -----
def test_fig2_worked_example():
    f = _read_kv(os.path.join(GOLD, "fig2_example.txt"))
    p = O.Params(f["M"] * f["Bc"], f["M"] * f["Br"], f["Bc"], f["Br"], f["kappa"], f["s"])
    assert (p.d, p.k, p.M) == (f["d"], f["k"], f["M"])
    S = O.build_csc(p, seed=7)
    assert (np.diff(S.indptr) == f["nnz_per_column"]).all()
    # block sparsity mask: exactly kappa nonzero blocks in every block row / column
    D = (S.toarray() != 0)
    mask = D.reshape(p.M, p.Br, p.M, p.Bc).any(axis=(1, 3))
    assert (mask.sum(0) == f["kappa"]).all() and (mask.sum(1) == f["kappa"]).all()
    # inside a nonzero block every column has exactly s nonzeros
    per_block_col = D.reshape(p.M, p.Br, p.M, p.Bc).sum(axis=1)  # [g, h, u]
    assert set(np.unique(per_block_col[mask])) == {f["s"]}
    assert set(np.unique(per_block_col[~mask])) == {0}


# ----------------------------------------------------------------- P2 -----
@pytest.mark.parametrize("cfg", PARAM_GRID)
@pytest.mark.parametrize("seed", [0, 1, 2**40 + 12345])
def test_structure_invariants(cfg, seed):
    p = O.Params(*cfg)
    rows, signs = O.build_tables(p, seed)
    S = O.build_csc(p, seed)
    ks = p.kappa * p.s
    assert S.shape == (p.k, p.d) and S.nnz == ks * p.d
    assert set(np.unique(signs)) <= {-1, 1}
    np.testing.assert_allclose(np.abs(S.data), 1 / math.sqrt(ks), rtol=1e-15)
    # all kappa*s rows of a column are distinct => unit column norms, ||S||_F^2 = d
    assert (np.diff(np.sort(rows, axis=1), axis=1) > 0).all()
    np.testing.assert_allclose(np.asarray(S.multiply(S).sum(0)).ravel(), 1.0, rtol=1e-13)
    # per block: the s updates of slot l land in one output block, distinct rows
    g_of = rows // p.Br
    for l in range(p.kappa):
        blk = g_of[:, l * p.s:(l + 1) * p.s]
        assert (blk == blk[:, :1]).all()
    # block graph kappa-regular on both sides, neighbours distinct (set union = kappa)
    _, k1 = O.seed_keys(seed)
    a, b = O.wiring(p.M, k1)
    indeg = np.zeros(p.M, dtype=int)
    for g in range(p.M):
        nb = O.neighbourhood(g, p.M, a, b, p.kappa)
        assert len(set(nb)) == p.kappa
        indeg[nb] += 1
        # the table agrees: slot l of the columns of block nb[l] points at g
        for l, h in enumerate(nb):
            assert (g_of[h * p.Bc:(h + 1) * p.Bc, l * p.s] == g).all()
    assert (indeg == p.kappa).all()


def _set_union_degrees(perms, M):
    return [len({pi[g] for pi in perms}) for g in range(M)]


def test_overlapping_permutations_counterexample():
    """Appendix E: identity + one swap on M=4 is NOT edge-disjoint (two block
    rows keep a single distinct neighbour); the affine wiring never does this."""
    ident, swap = [0, 1, 2, 3], [1, 0, 2, 3]
    assert _set_union_degrees([ident, swap], 4) == [2, 2, 1, 1]
    for seed in range(20):
        a, b = O.wiring(4, O.seed_keys(seed)[1])
        perms = [[O.neighbourhood(g, 4, a, b, 2)[l] for g in range(4)] for l in range(2)]
        assert _set_union_degrees(perms, 4) == [2, 2, 2, 2]


# ----------------------------------------------------------------- P3 -----
@pytest.mark.parametrize("M", [1, 2, 3, 4, 8, 12, 16, 18, 36, 45, 100, 128, 360, 1024, 1155])
def test_full_period(M):
    for seed in range(8):
        a, b = O.wiring(M, O.seed_keys(seed)[1])
        if M == 1:
            assert (a, b) == (0, 0)
            continue
        assert math.gcd(b, M) == 1
        n, p = M, 2
        while n > 1:
            if n % p == 0:
                assert (a - 1) % p == 0
                while n % p == 0:
                    n //= p
            p += 1
        if M % 4 == 0:
            assert (a - 1) % 4 == 0
        for x0 in (0, M // 2, M - 1):
            x, seen = x0, set()
            for _ in range(M):
                seen.add(x)
                x = (a * x + b) % M
            assert len(seen) == M and x == x0


# ----------------------------------------------------------------- P4 -----
def test_energy_identity_and_block_output_equation():
    p = O.Params(1152, 72, 96, 6, 5, 3)
    seed = 3
    rng = np.random.default_rng(5)
    x = rng.standard_normal(p.d)
    U = rng.standard_normal((p.d, 4))
    _, k1 = O.seed_keys(seed)
    a, b = O.wiring(p.M, k1)
    xb = x.reshape(p.M, p.Bc)
    Ub = U.reshape(p.M, p.Bc, 4)
    lhs, lhsU = 0.0, np.zeros((4, 4))
    S = O.build_csc(p, seed)
    y = O.apply(S, x[:, None])[:, 0]
    for g in range(p.M):
        nb = O.neighbourhood(g, p.M, a, b, p.kappa)
        lhs += sum(np.dot(xb[h], xb[h]) for h in nb)
        lhsU += sum(Ub[h].T @ Ub[h] for h in nb)
        # (Sx)^(g) = Phi_g x_N(g) / sqrt(kappa), Phi_g built here from the scalar hash
        acc = np.zeros(p.Br)
        for h in nb:
            bk = O.block_key(k1, g, h, p.M)
            r, sg = O.row_targets(np.uint32(bk), np.arange(p.Bc, dtype=np.uint32), p.Br, p.s)
            Phi = np.zeros((p.Br, p.Bc))
            for i in range(p.s):
                Phi[r[:, i], np.arange(p.Bc)] += sg[:, i] / math.sqrt(p.s)
            acc += Phi @ xb[h]
        np.testing.assert_allclose(y[g * p.Br:(g + 1) * p.Br], acc / math.sqrt(p.kappa), atol=1e-12)
    np.testing.assert_allclose(lhs, p.kappa * np.dot(x, x), rtol=1e-12)
    np.testing.assert_allclose(lhsU, p.kappa * U.T @ U, rtol=1e-12, atol=1e-9)


# ----------------------------------------------------------------- P5 -----
def test_norm_unbiased_over_seeds():
    p = O.Params(1024, 128, 128, 16, 2, 2)
    rng = np.random.default_rng(11)
    xs = np.stack([rng.standard_normal(p.d),
                   np.r_[10.0, 5.0, np.zeros(p.d - 2)],          # spiky
                   np.r_[np.ones(p.Bc), np.zeros(p.d - p.Bc)]],  # one block only
                  axis=1)
    n2 = (xs ** 2).sum(0)
    ratios = np.array([(O.apply(O.build_csc(p, seed), xs) ** 2).sum(0) / n2 for seed in range(1500)])
    mean, se = ratios.mean(0), ratios.std(0, ddof=1) / math.sqrt(len(ratios))
    assert (np.abs(mean - 1.0) < 4 * se + 1e-12).all(), (mean, se)
    assert (se > 0).all()


# ----------------------------------------------------------------- P6 -----
@pytest.mark.parametrize("cfg", [(64, 16, 64, 16, 1, 4), (96, 24, 8, 2, 3, 2), (60, 30, 10, 5, 6, 5)])
def test_bruteforce_dense_equals_csc(cfg):
    p = O.Params(*cfg)
    rng = np.random.default_rng(2)
    A = rng.standard_normal((p.d, 7))
    for seed in (0, 9):
        Sd = O.dense_by_loops(p, seed)
        Sc = O.build_csc(p, seed)
        np.testing.assert_array_equal(Sd, Sc.toarray())
        np.testing.assert_allclose(O.apply(Sc, A), Sd @ A, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("cfg,d_short", [((96, 24, 8, 2, 3, 2), 91), ((60, 30, 10, 5, 6, 5), 51),
                                         ((4096, 256, 512, 32, 2, 4), 3585)])
def test_padding_is_the_sketch_of_the_zero_padded_input(cfg, d_short):
    """Section 4 handles d not divisible by Bc "by padding": S for the short d must be the
    first d columns of the full-grid S, so S_short @ A == S_full @ [A; 0]."""
    full = O.Params(*cfg)
    short = O.Params(d_short, *cfg[1:])
    assert short.M == full.M and short.d_padded == full.d
    Sf, Ss = O.build_csc(full, 3), O.build_csc(short, 3)
    assert Ss.shape == (full.k, d_short)
    assert (Sf[:, :d_short] != Ss).nnz == 0
    A = np.random.default_rng(0).standard_normal((d_short, 5))
    Apad = np.vstack([A, np.zeros((full.d - d_short, 5))])
    np.testing.assert_allclose(O.apply(Ss, A), O.apply(Sf, Apad), rtol=1e-14, atol=1e-14)
    if full.d <= 128:
        np.testing.assert_array_equal(O.dense_by_loops(short, 3), Ss.toarray())
    with pytest.raises(ValueError):
        O.Params(full.d - full.Bc, *cfg[1:]).check()  # one whole block short: grid no longer square


def test_plain_sjlt_special_case():
    """M = 1, kappa = 1: S is an ordinary SJLT -- s entries +-1/sqrt(s) per column."""
    p = O.Params(512, 32, 512, 32, 1, 4)
    S = O.build_csc(p, 4).toarray()
    assert ((S != 0).sum(0) == 4).all()
    np.testing.assert_allclose(np.abs(S[S != 0]), 0.5)
    # rows roughly balanced: every output row is hit (512*4/32 = 64 expected)
    assert ((S != 0).sum(1) > 20).all()


def test_one_hot_and_linearity():
    p = O.Params(4096, 256, 512, 32, 2, 4)
    S = O.build_csc(p, 0)
    cols = [0, 511, 512, 3584, 4095]
    E = np.zeros((p.d, len(cols)))
    E[cols, np.arange(len(cols))] = 1.0
    np.testing.assert_array_equal(O.apply(S, E), S[:, cols].toarray())
    rng = np.random.default_rng(0)
    A, B = rng.standard_normal((2, p.d, 3))
    np.testing.assert_allclose(O.apply(S, 2 * A - 3 * B), 2 * O.apply(S, A) - 3 * O.apply(S, B),
                               rtol=1e-12, atol=1e-12)


def test_rows_layout_is_the_same_map_row_by_row():
    """apply_rows: vectors held as rows.  Pinned by brute force, one row at a time, against the
    scalar-loop dense S (not against apply), and by one-hot rows reproducing columns of S."""
    p = O.Params(96, 24, 32, 8, 2, 2)
    S = O.build_csc(p, 5)
    D = O.dense_by_loops(p, 5)
    rng = np.random.default_rng(3)
    G = rng.standard_normal((7, p.d))
    out = O.apply_rows(S, G)
    assert out.shape == (7, p.k)
    for i in range(7):
        want = np.array([sum(D[r, c] * G[i, c] for c in range(p.d)) for r in range(p.k)])
        np.testing.assert_allclose(out[i], want, rtol=1e-12, atol=1e-12)
    E = np.zeros((3, p.d))
    E[[0, 1, 2], [0, 40, 95]] = 1.0
    np.testing.assert_array_equal(O.apply_rows(S, E), D[:, [0, 40, 95]].T)


def test_kappa_buys_robustness_to_localized_inputs():
    """Section 4 / Section 6: an input whose energy sits in one input block reaches only kappa
    output blocks, i.e. kappa*Br rows of S A.  With more columns than that the sketch cannot be
    an embedding (rank argument: the OSE error is at least 1 exactly); a larger kappa spreads
    the block over enough rows.  A dense (non-localized) input does not care."""
    d, k, Bc, Br, s, n = 4096, 512, 256, 32, 4, 48     # M = 16
    rng = np.random.default_rng(0)
    A = np.zeros((d, n))
    A[:Bc] = rng.standard_normal((Bc, n))              # all energy in input block 0
    Q = np.linalg.qr(A)[0]
    errs = {}
    for kappa in (1, 2, 4, 8, 16):
        S = O.build_csc(O.Params(d, k, Bc, Br, kappa, s), 1)
        SQ = O.apply(S, Q)
        assert (np.abs(SQ).sum(1) > 0).sum() <= kappa * Br      # only kappa output blocks are reached
        errs[kappa] = O.ose_error(SQ)
    assert errs[1] >= 1 - 1e-9                          # 32 rows cannot embed 48 dimensions
    assert errs[1] > errs[2] > errs[4] > errs[8] > errs[16]   # more neighbours, less distortion
    assert errs[16] < 0.9                               # M = 16 neighbours: the whole sketch is used
    Qd = np.linalg.qr(rng.standard_normal((d, n)))[0]   # dense input: kappa = 1 is already fine
    assert O.ose_error(O.apply(O.build_csc(O.Params(d, k, Bc, Br, 1, s), 1), Qd)) < 0.9


# ---------------------------------------------------------------- P10 -----
@pytest.mark.parametrize("kappa", [1, 2, 4, 8])
def test_coherence_bounds(kappa):
    M, Bc = 16, 32
    rng = np.random.default_rng(kappa)
    X = rng.standard_normal((M * Bc, 6))
    X[:3] *= 50.0  # a few high-leverage rows
    U, _ = np.linalg.qr(X)
    a, b = O.wiring(M, O.seed_keys(0)[1])
    blk = O.block_coherence(U, M)
    nbr = O.nbr_coherence(U, M, a, b, kappa)
    assert blk / kappa - 1e-9 <= nbr <= blk + 1e-9
    assert 1.0 - 1e-9 <= blk <= M + 1e-9
    if kappa == 1:
        np.testing.assert_allclose(nbr, blk, rtol=1e-12)


def test_ose_error_closed_forms():
    Q, _ = np.linalg.qr(np.random.default_rng(0).standard_normal((50, 5)))
    assert O.ose_error(Q) < 1e-12
    assert abs(O.ose_error(2 * Q) - 3.0) < 1e-12
    assert O.rel_fro_err(np.ones((2, 2)), np.ones((2, 2))) == 0.0
    assert abs(O.rel_fro_err(np.zeros((2, 2)), np.ones((2, 2))) - 1.0) < 1e-15


# ------------------------------------------------ planted mistakes --------
def test_planted_mistakes_are_caught(monkeypatch):
    """Each plausible slip in the oracle must break at least one pin above."""
    p = O.Params(4096, 256, 512, 32, 2, 4)
    good = O.build_csc(p, 0)

    # (1) identity permutation included (l starting at 0)
    def nb0(g, M, a, b, kappa):
        out, h = [], g
        for _ in range(kappa):
            out.append(h)
            h = (a * h + b) % M
        return out
    assert nb0(0, 8, 5, 7, 2) != [7, 2]

    # (2) sign convention flipped -> golden signs differ
    r, sg = O.row_targets(np.uint32(0x15378950), np.uint32(0), 32, 4)
    assert list(-sg) != [1, 1, 1, -1]

    # (3) scale without the 1/sqrt(kappa) factor -> column norms are not 1
    bad = good * math.sqrt(p.kappa)
    assert abs(bad.multiply(bad).sum(0).max() - 1.0) > 0.5

    # (4) transposed block index in the key (h*M+g) -> different matrix
    monkeypatch.setattr(O, "block_key", lambda k1, g, h, M: O.mix32_int(k1 ^ O.mix32_int((h * M + g + O.C3) & 0xFFFFFFFF)))
    assert O.block_key(O.seed_keys(0)[1], 0, 7, 8) != 0x15378950
