"""Float64 CPU oracle for BlockPerm-SJLT (paper Section 4, Appendix E, Alg. 1).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

What it computes is the plain definition: the sketch ``S`` (k x d) is written
out as an explicit sparse matrix and ``SA = S @ A`` is evaluated in float64.

Structure of ``S`` (Section 4):
  * ``M x M`` grid of ``Br x Bc`` blocks, ``M = d/Bc = k/Br``;
  * block ``(g, h)`` is nonzero iff ``h`` is one of the ``kappa`` neighbours
    ``pi_l(g) = f^l(g)``, ``l = 1..kappa``, of output block ``g``, where
    ``f(x) = (a x + b) mod M`` is a full-period affine map (Appendix E,
    "Full-cycle affine construction");
  * every column of a nonzero block holds exactly ``s`` entries ``+-1/sqrt(s)``
    in distinct rows, and the block enters ``S`` scaled by ``1/sqrt(kappa)``,
    so a full column of ``S`` has ``kappa*s`` entries of magnitude
    ``1/sqrt(kappa*s)``.

The paper fixes neither the 32-bit mixing hash nor how ``(a, b)``, the row
positions and the signs are drawn from it (Appendix E, "Within-block
hashing").  The reading used by this repository is spelled out in the
functions below, one function per step, so that each can be checked by eye.

All hash arithmetic is on unsigned 32-bit words with wrap-around.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np
import scipy.sparse as sp

# First 32 fractional bits of sqrt(2), sqrt(3), sqrt(5) (the last forced odd).
C1 = 0x6A09E667
C2 = 0xBB67AE85
C3 = 0x3C6EF373
_MASK = 0xFFFFFFFF


# --------------------------------------------------------------------------
# 32-bit mixer
# --------------------------------------------------------------------------
def mix32_int(x: int) -> int:
    """Bijective 32-bit mixer on a Python int (xor-shift / odd-multiply x3)."""
    x &= _MASK
    x ^= x >> 16
    x = (x * C1) & _MASK
    x ^= x >> 15
    x = (x * C2) & _MASK
    x ^= x >> 16
    x = (x * C3) & _MASK
    x ^= x >> 15
    return x


def mix32(x) -> np.ndarray:
    """The same mixer, element-wise on a uint32 array."""
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= np.uint32(C1)
    x ^= x >> np.uint32(15)
    x *= np.uint32(C2)
    x ^= x >> np.uint32(16)
    x *= np.uint32(C3)
    x ^= x >> np.uint32(15)
    return x


def seed_keys(seed: int) -> tuple[int, int]:
    """Two key words from the 64-bit seed (low word first)."""
    lo = seed & _MASK
    hi = (seed >> 32) & _MASK
    k0 = mix32_int(lo ^ C1)
    k1 = mix32_int(hi ^ k0 ^ C2)
    return k0, k1


# --------------------------------------------------------------------------
# Block wiring (Appendix E, "Full-cycle affine construction")
# --------------------------------------------------------------------------
def radical(m: int) -> int:
    """Product of the distinct prime factors of m."""
    r, p, n = 1, 2, m
    while p * p <= n:
        if n % p == 0:
            r *= p
            while n % p == 0:
                n //= p
        p += 1
    if n > 1:
        r *= n
    return r


def wiring(M: int, k1: int) -> tuple[int, int]:
    """Seed-derived (a, b) with f(x) = (a x + b) mod M of period M.

    The three full-period conditions of Appendix E are met by construction:
    a - 1 is a multiple of L = lcm(rad(M), 4 if 4 | M), and b is moved up to
    the next unit modulo M.
    """
    if M == 1:
        return 0, 0
    L = math.lcm(radical(M), 4 if M % 4 == 0 else 1)
    ha = mix32_int(k1 ^ 1)
    hb = mix32_int(k1 ^ 2)
    a = (1 + L * (ha % (M // L))) % M
    b = hb % M
    while math.gcd(b, M) != 1:
        b = (b + 1) % M
    return a, b


def neighbourhood(g: int, M: int, a: int, b: int, kappa: int) -> list[int]:
    """[pi_1(g), ..., pi_kappa(g)] with pi_l = f^l (the identity is not used)."""
    out, h = [], g
    for _ in range(kappa):
        h = (a * h + b) % M
        out.append(h)
    return out


# --------------------------------------------------------------------------
# Within-block hashing (Alg. 1, the "hash (g,h,u,i) -> (r_i, sigma_i)" step)
# --------------------------------------------------------------------------
def block_key(k1: int, g: int, h: int, M: int) -> int:
    return mix32_int(k1 ^ mix32_int((g * M + h + C3) & _MASK))


def row_targets(bk, u, Br: int, s: int):
    """Destination rows and signs for local input rows ``u`` of one block.

    ``bk`` and ``u`` broadcast against each other.  Returns ``rows`` and
    ``signs`` with a trailing axis of length ``s``: the rows are the arithmetic
    progression shift + i*c (mod Br) with gcd(c, Br) = 1, hence distinct for
    s <= Br; sign i is +1 when bit i of the second hash word is clear.
    """
    bk = np.asarray(bk, dtype=np.uint32)
    u = np.asarray(u, dtype=np.uint32)
    h1 = mix32(bk ^ u)
    h2 = mix32(h1 ^ np.uint32(C2))
    shift = (h1 & np.uint32(0xFFFF)).astype(np.int64) % Br
    c = (h1 >> np.uint32(16)).astype(np.int64) % Br
    while True:
        bad = np.gcd(c, Br) != 1
        if not bad.any():
            break
        c = np.where(bad, (c + 1) % Br, c)
    i = np.arange(s, dtype=np.int64)
    rows = (shift[..., None] + i * c[..., None]) % Br
    bits = (h2[..., None] >> i.astype(np.uint32)) & np.uint32(1)
    signs = np.where(bits == 0, 1, -1).astype(np.int8)
    return rows, signs


# --------------------------------------------------------------------------
# Parameters and explicit construction of S
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Params:
    d: int
    k: int
    Bc: int
    Br: int
    kappa: int
    s: int

    @property
    def M(self) -> int:
        return self.k // self.Br

    @property
    def d_padded(self) -> int:
        """Input dimension rounded up to whole blocks (Section 4: the general case is handled
        by padding): S is the first d columns of the sketch of the zero-padded input."""
        return self.M * self.Bc

    def check(self) -> None:
        if min(self.d, self.k, self.Bc, self.Br, self.kappa, self.s) < 1:
            raise ValueError("all parameters must be positive")
        if self.k % self.Br:
            raise ValueError("Br must divide k")
        if -(-self.d // self.Bc) != self.k // self.Br:
            raise ValueError("ceil(d/Bc) must equal k/Br (square block grid)")
        if self.kappa > self.M:
            raise ValueError("kappa must not exceed M")
        if self.s > self.Br or self.s > 32 or self.Br > 65536:
            raise ValueError("need s <= min(Br, 32) and Br <= 65536")


def build_tables(p: Params, seed: int):
    """Nonzeros of S per column: global rows [d, kappa*s] and signs [d, kappa*s].

    Entry (col, (l-1)*s + i) belongs to the block (g, h) with h = col // Bc and
    pi_l(g) = h, and to the i-th update of that block.
    """
    p.check()
    M, Bc, Br, kappa, s = p.M, p.Bc, p.Br, p.kappa, p.s
    _, k1 = seed_keys(seed)
    a, b = wiring(M, k1)
    rows = np.empty((p.d_padded, kappa * s), dtype=np.int64)
    signs = np.empty((p.d_padded, kappa * s), dtype=np.int8)
    u = np.arange(Bc, dtype=np.uint32)
    g_all = np.arange(M, dtype=np.int64)
    h_l = g_all.copy()
    for l in range(1, kappa + 1):
        h_l = (a * h_l + b) % M  # pi_l(g) for every g
        inner = ((g_all * M + h_l + C3) & _MASK).astype(np.uint32)
        bk = mix32(np.uint32(k1) ^ mix32(inner))  # [M]
        r, sg = row_targets(bk[:, None], u[None, :], Br, s)  # [M, Bc, s]
        r = r + (g_all * Br)[:, None, None]
        # scatter block-row g to the column range of its input block h_l[g]
        cols = (h_l[:, None] * Bc + np.arange(Bc)[None, :]).reshape(-1)
        rows[cols, (l - 1) * s:l * s] = r.reshape(-1, s)
        signs[cols, (l - 1) * s:l * s] = sg.reshape(-1, s)
    return rows[:p.d], signs[:p.d]  # columns of the padding are dropped


def build_csc(p: Params, seed: int) -> sp.csc_matrix:
    """S as an explicit k x d CSC matrix in float64 (Section 4 definition)."""
    rows, signs = build_tables(p, seed)
    nnz_col = p.kappa * p.s
    data = signs.astype(np.float64).reshape(-1) / math.sqrt(nnz_col)
    indptr = np.arange(p.d + 1, dtype=np.int64) * nnz_col
    return sp.csc_matrix((data, rows.reshape(-1), indptr), shape=(p.k, p.d))


def apply(S: sp.csc_matrix, A) -> np.ndarray:
    """SA in float64 from the exact input values."""
    return np.asarray(S @ np.asarray(A, dtype=np.float64))


def apply_rows(S: sp.csc_matrix, G) -> np.ndarray:
    """The same map for vectors held as rows: out[i, :] = S G[i, :], i.e. out = G S^T (float64).
    (The layout of a per-example-gradient pipeline, Section 7 "GraSS for Data Attribution".)"""
    G64 = np.asarray(G, dtype=np.float64)
    return np.ascontiguousarray(np.asarray(S @ G64.T).T)


def dense_by_loops(p: Params, seed: int) -> np.ndarray:
    """S as a dense array, one scalar at a time (tiny sizes only).

    Walks output block, neighbour, local row and update index exactly in the
    order of Alg. 1, using only the scalar hash; serves as a brute-force check
    of the vectorised construction.
    """
    p.check()
    M, Bc, Br = p.M, p.Bc, p.Br
    _, k1 = seed_keys(seed)
    a, b = wiring(M, k1)
    S = np.zeros((p.k, p.d))
    val = 1.0 / math.sqrt(p.kappa * p.s)
    for g in range(M):
        for h in neighbourhood(g, M, a, b, p.kappa):
            bk = block_key(k1, g, h, M)
            for u in range(Bc):
                h1 = mix32_int(bk ^ u)
                h2 = mix32_int(h1 ^ C2)
                shift = (h1 & 0xFFFF) % Br
                c = (h1 >> 16) % Br
                while math.gcd(c, Br) != 1:
                    c = (c + 1) % Br
                if h * Bc + u >= p.d:  # padding column
                    continue
                for i in range(p.s):
                    r = (shift + i * c) % Br
                    sigma = 1.0 if ((h2 >> i) & 1) == 0 else -1.0
                    S[g * Br + r, h * Bc + u] += sigma * val
    return S


# --------------------------------------------------------------------------
# Quality read-outs (Section 3 Def. of block coherence, Section 6 Def. of
# neighbourhood coherence, Appendix G "OSE spectral error")
# --------------------------------------------------------------------------
def rel_fro_err(X, ref) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    num = np.linalg.norm(np.asarray(X, dtype=np.float64) - ref)
    return float(num / den) if den > 0 else float(num)


def ose_error(SQ) -> float:
    """|| (SQ)^T (SQ) - I ||_2 for an orthonormal Q."""
    SQ = np.asarray(SQ, dtype=np.float64)
    G = SQ.T @ SQ
    return float(np.linalg.norm(G - np.eye(G.shape[0]), 2))


def block_coherence(U, M: int) -> float:
    """M * max_h ||U^(h)||_2^2 over M contiguous row blocks."""
    U = np.asarray(U, dtype=np.float64)
    Bc = U.shape[0] // M
    return M * max(np.linalg.norm(U[h * Bc:(h + 1) * Bc], 2) ** 2 for h in range(M))


def nbr_coherence(U, M: int, a: int, b: int, kappa: int) -> float:
    """(M/kappa) * max_g ||U_N(g)||_2^2 with N(g) from the affine wiring."""
    U = np.asarray(U, dtype=np.float64)
    Bc = U.shape[0] // M
    best = 0.0
    for g in range(M):
        blocks = [U[h * Bc:(h + 1) * Bc] for h in neighbourhood(g, M, a, b, kappa)]
        best = max(best, np.linalg.norm(np.vstack(blocks), 2) ** 2)
    return M / kappa * best
