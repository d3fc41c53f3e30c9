"""Float64 CPU oracle for the dense Gaussian sketch S_ij ~ N(0, 1/k) (paper
Section 1: the canonical JL transform; Section 3: the canonical OSE example).

TEST INFRASTRUCTURE ONLY -- never imported by the product package.

The paper fixes only the distribution.  So that both sides can draw the same
matrix from a seed, entry (i, j) comes from a counter-based generator: two
24-bit uniforms hashed from the flat index i*d + j and the seed key, turned
into a standard normal by the Box-Muller transform, divided by sqrt(k) and
rounded to float32 (the stored matrix is float32).
"""
from __future__ import annotations

import math

import numpy as np

from .blockperm import C1, mix32, seed_keys


def gaussian_matrix(k: int, d: int, seed: int) -> np.ndarray:
    """The k x d sketch as float32 values held in a float64 array."""
    _, k1 = seed_keys(seed)
    idx = np.arange(k * d, dtype=np.uint64)
    lo = (idx & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    hi = (idx >> np.uint64(32)).astype(np.uint32)
    c = mix32(lo ^ mix32(hi ^ np.uint32(k1 ^ C1)))
    u1 = ((mix32(c ^ np.uint32(0x9E3779B9)) >> np.uint32(8)).astype(np.float64) + 1.0) / 16777216.0
    u2 = (mix32(c ^ np.uint32(0x85EBCA6B)) >> np.uint32(8)).astype(np.float64) / 16777216.0
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    S = (z / math.sqrt(k)).astype(np.float32)
    return S.astype(np.float64).reshape(k, d)


def apply(S: np.ndarray, A) -> np.ndarray:
    return S @ np.asarray(A, dtype=np.float64)
