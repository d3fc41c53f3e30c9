"""Float64 CPU oracle for FlashBlockRow, the gather-only block-row sampling sketch of the
paper's Appendix D ("A Fast but Fragile Alternative", Alg. 2).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

Definition (Alg. 2): output block row g samples kappa input blocks; every output row r of
that block row draws, from each sampled block, s row indices uniformly in [Bc] (with
replacement) and s signs, and

    (SA)[g*Br + r, :] = sqrt(d/k) / sqrt(kappa*s) * sum_{h, t} sigma_t * A[h*Bc + i_t, :].

Nothing constrains the columns of S: some input coordinates are never read (the paper's
"fragile").  Readings where the paper is silent: the kappa blocks of block row g are the
wiring neighbours f^l(g), l = 1..kappa, of the BlockPerm sketch (distinct, on-the-fly); index and
sign of update t of row r in block (g, h) come from two hash words
w1 = mix32(BK(g,h) ^ C1 ^ (r*32 + t)), i_t = w1 mod Bc, w2 = mix32(w1 ^ C2), sigma_t = + if
w2 is even.  Rows of a partly filled last input block (d not a multiple of Bc) read as zero.
"""
from __future__ import annotations

import math

import numpy as np
import scipy.sparse as sp

from .blockperm import C1, C2, Params, block_key, mix32, neighbourhood, seed_keys, wiring


def build_tables(p: Params, seed: int):
    """Per output row: global column indices [k, kappa*s] (may exceed d-1 only in the padding)
    and signs [k, kappa*s]; entry (row, (l-1)*s + t)."""
    p.check()
    M, Bc, Br, kappa, s = p.M, p.Bc, p.Br, p.kappa, p.s
    _, k1 = seed_keys(seed)
    a, b = wiring(M, k1)
    cols = np.empty((p.k, kappa * s), dtype=np.int64)
    signs = np.empty((p.k, kappa * s), dtype=np.int8)
    r = np.arange(Br, dtype=np.uint32)
    t = np.arange(s, dtype=np.uint32)
    ctr = (r[:, None] * np.uint32(32) + t[None, :]).astype(np.uint32)  # [Br, s]
    for g in range(M):
        for l, h in enumerate(neighbourhood(g, M, a, b, kappa)):
            bk = block_key(k1, g, h, M)
            w1 = mix32(np.uint32(bk ^ C1) ^ ctr)
            w2 = mix32(w1 ^ np.uint32(C2))
            cols[g * Br:(g + 1) * Br, l * s:(l + 1) * s] = h * Bc + (w1.astype(np.int64) % Bc)
            signs[g * Br:(g + 1) * Br, l * s:(l + 1) * s] = np.where((w2 & np.uint32(1)) == 0, 1, -1)
    return cols, signs


def scale(p: Params) -> float:
    return math.sqrt(p.d / p.k) / math.sqrt(p.kappa * p.s)


def build_csr(p: Params, seed: int) -> sp.csr_matrix:
    """S as an explicit k x d CSR matrix (repeated indices of a row add up)."""
    cols, signs = build_tables(p, seed)
    rows = np.repeat(np.arange(p.k, dtype=np.int64), p.kappa * p.s)
    c, v = cols.reshape(-1), signs.reshape(-1).astype(np.float64) * scale(p)
    keep = c < p.d  # indices that fall in the zero padding contribute nothing
    S = sp.coo_matrix((v[keep], (rows[keep], c[keep])), shape=(p.k, p.d))
    return S.tocsr()


def apply(S, A) -> np.ndarray:
    return np.asarray(S @ np.asarray(A, dtype=np.float64))
