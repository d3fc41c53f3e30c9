"""The five benchmark configurations and their seeded synthetic inputs.

This module serves the tests, the benchmark and the smoke check.  It holds no
arithmetic of the sketch itself: only shapes, parameters and random input
matrices.  The inputs stand in for the paper's workloads (Section 7: synthetic
Gaussian and low-rank matrices, sparse and LLM-weight matrices, per-example
gradients of a data-attribution pipeline), none of which ship with this
repository; shapes and value distributions follow them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Config:
    name: str
    dtype: torch.dtype
    d: int
    n: int
    k: int
    Bc: int
    Br: int
    s: int
    kappa: int
    sketch_seed: int = 0
    data_seed: int = 1
    chunk: int = 0  # > 0: columns are applied in chunks of this width

    @property
    def params(self):
        return (self.d, self.k, self.Bc, self.Br, self.kappa, self.s)

    @property
    def elt(self) -> int:
        return 4 if self.dtype == torch.float32 else 2

    @property
    def a_bytes(self) -> int:
        return self.d * self.n * self.elt


CONFIGS = {
    "tiny": Config("tiny", torch.float32, 4096, 512, 256, 512, 32, 4, 2),
    "mid": Config("mid", torch.float32, 16384, 16384, 1024, 1024, 64, 8, 4),
    "tall": Config("tall", torch.float32, 262144, 256, 4096, 2048, 32, 4, 4),
    "wide": Config("wide", torch.bfloat16, 65536, 8192, 4096, 2048, 128, 8, 4),
    "grad": Config("grad", torch.bfloat16, 4194304, 1024, 8192, 4096, 8, 2, 8, chunk=256),
}
MID_KAPPAS = (1, 2, 4, 8)
WIDE_NS = (1024, 2048, 4096, 8192)


def _gen(device, seed):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def gaussian(d, n, seed, device, dtype=torch.float32):
    return torch.randn((d, n), generator=_gen(device, seed), device=device, dtype=torch.float32).to(dtype)


def student_t3(d, n, seed, device, dtype=torch.bfloat16, slab=8192):
    """Student-t with 3 degrees of freedom scaled to unit variance (var = 3)."""
    g = _gen(device, seed)
    out = torch.empty((d, n), device=device, dtype=dtype)
    for r0 in range(0, d, slab):
        r1 = min(d, r0 + slab)
        z = torch.randn((r1 - r0, n), generator=g, device=device)
        chi = torch.randn((3, r1 - r0, n), generator=g, device=device).square_().sum(0)
        out[r0:r1] = (z / torch.sqrt(chi / 3.0) / math.sqrt(3.0)).to(dtype)
    return out


def laplace_lognormal(d, n, seed, device, dtype=torch.bfloat16, slab=65536):
    """Heavy-tailed synthetic per-example gradients: Laplace entries of unit
    variance, column j scaled by exp(z_j)/sqrt(d), z_j ~ N(0,1)."""
    g = _gen(device, seed)
    col = torch.exp(torch.randn(n, generator=g, device=device)) / math.sqrt(d)
    out = torch.empty((d, n), device=device, dtype=dtype)
    for r0 in range(0, d, slab):
        r1 = min(d, r0 + slab)
        u = torch.rand((r1 - r0, n), generator=g, device=device) - 0.5
        lap = -torch.sign(u) * torch.log1p(-2.0 * u.abs()).clamp_(min=-80.0) / math.sqrt(2.0)
        out[r0:r1] = (lap * col).to(dtype)
    return out


def coherent_tall(d, n, seed, device="cpu"):
    """U diag(sigma) V^T with sigma decaying 1 -> 1e-6, plus 16 rows scaled x1e3
    (high leverage).  Built in float64 on the host; returns (A64, row_ids)."""
    g = _gen("cpu", seed)
    U, _ = torch.linalg.qr(torch.randn((d, n), generator=g, dtype=torch.float64))
    V, _ = torch.linalg.qr(torch.randn((n, n), generator=g, dtype=torch.float64))
    sigma = torch.pow(10.0, -6.0 * torch.arange(n, dtype=torch.float64) / (n - 1))
    A = (U * sigma) @ V.T
    rows = torch.randperm(d, generator=g)[:16]
    A[rows] *= 1.0e3
    return A, rows


def make_input(cfg: Config, device, n: int | None = None):
    """The synthetic A of a configuration (optionally with another width n)."""
    n = cfg.n if n is None else n
    if cfg.name in ("tiny", "mid"):
        return gaussian(cfg.d, n, cfg.data_seed, device)
    if cfg.name == "tall":
        A, _ = coherent_tall(cfg.d, n, cfg.data_seed)
        return A.to(torch.float32).to(device)
    if cfg.name == "wide":
        return student_t3(cfg.d, n, cfg.data_seed, device)
    if cfg.name == "grad":
        return laplace_lognormal(cfg.d, n, cfg.data_seed, device)
    raise KeyError(cfg.name)
