"""Quality-versus-speed read-outs for the sketches of this library (paper Section 7 and
Appendix G "Metrics"): Gram-matrix error, OSE spectral error, sketch-and-ridge and
sketch-and-solve residuals, each next to the sketch's kernel time.

    python -m paper_2602_06071_amd.quality [--d 65536 --n 1024 --k 4096] [--data gaussian|lowrank]

The sketches run in the HIP library; the downstream linear algebra (Gram products, QR,
solves) is plain torch on the same device, in float64 so that the metric itself adds no
error of its own.  Inputs are synthetic (Gaussian, low-rank + noise, and a localized one whose energy sits in
a single input block: the case the wiring parameter kappa exists for) at the paper's shapes.
"""
from __future__ import annotations

import argparse
import json

import torch


# ---- metrics, exactly as Appendix G defines them ------------------------------------
def gram_error(A: torch.Tensor, SA: torch.Tensor) -> float:
    """|| (SA)^T (SA) - A^T A ||_F / || A^T A ||_F   (absolute if the denominator is 0)."""
    A, SA = A.double(), SA.double()
    G = A.T @ A
    den = torch.linalg.norm(G)
    num = torch.linalg.norm(SA.T @ SA - G)
    return float(num / den) if den > 0 else float(num)


def ose_error(SQ: torch.Tensor) -> float:
    """|| (SQ)^T (SQ) - I ||_2 for an orthonormal Q."""
    SQ = SQ.double()
    G = SQ.T @ SQ
    return float(torch.linalg.matrix_norm(G - torch.eye(G.shape[0], dtype=G.dtype, device=G.device), ord=2))


def ridge_residual(A, b, SA, Sb, lam: float) -> float:
    """x = argmin ||SA x - Sb||^2 + lam ||x||^2;  ||A x - b|| / ||b||  (absolute if b = 0)."""
    A, b, SA, Sb = A.double(), b.double(), SA.double(), Sb.double()
    n = SA.shape[1]
    x = torch.linalg.solve(SA.T @ SA + lam * torch.eye(n, dtype=SA.dtype, device=SA.device), SA.T @ Sb)
    nb = torch.linalg.norm(b)
    r = torch.linalg.norm(A @ x - b)
    return float(r / nb) if nb > 0 else float(r)


def lstsq_residual(A, b, SA, Sb) -> float:
    """x = argmin ||SA x - Sb||;  the same residual definition."""
    A, b, SA, Sb = A.double(), b.double(), SA.double(), Sb.double()
    x = torch.linalg.lstsq(SA, Sb).solution
    nb = torch.linalg.norm(b)
    r = torch.linalg.norm(A @ x - b)
    return float(r / nb) if nb > 0 else float(r)


# ---- synthetic inputs -----------------------------------------------------------------
def make_data(kind: str, d: int, n: int, seed: int, device):
    g = torch.Generator(device=device).manual_seed(seed)
    if kind == "gaussian":
        A = torch.randn((d, n), generator=g, device=device)
    elif kind == "lowrank":  # rank-32 signal + 1 % noise
        r = min(32, n)
        A = torch.randn((d, r), generator=g, device=device) @ torch.randn((r, n), generator=g, device=device)
        A = A / r ** 0.5 + 0.01 * torch.randn((d, n), generator=g, device=device)
    elif kind == "oneblock":  # all energy in the first d/128 rows: one input block at the default k and Br
        A = torch.zeros((d, n), device=device)
        A[: d // 128] = torch.randn((d // 128, n), generator=g, device=device)
    else:
        raise KeyError(kind)
    x_true = torch.randn((n, 1), generator=g, device=device)
    b = A @ x_true + 0.1 * torch.randn((d, 1), generator=g, device=device)
    return A, b


# ---- one method on one problem ----------------------------------------------------------
def evaluate(sk, A, b, lam=1e-2, reps=5):
    """Sketch A (timed: the dominant kernel, and the whole apply, on the n columns alone) and b (a second apply on
    a 4-column matrix holding b, so that the matrix-core path stays eligible), then the four
    metrics."""
    d, n = A.shape
    out = sk.apply(A)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        sk.apply(A, out)
    e1.record()
    torch.cuda.synchronize()
    apply_ms = e0.elapsed_time(e1) / reps  # whole apply, all its kernels, back to back
    sk.profile_begin(reps)
    for _ in range(reps):
        sk.apply(A, out)
    ms = sk.profile_end()
    b4 = torch.zeros((d, 4), device=A.device, dtype=A.dtype)
    b4[:, :1] = b
    SA, Sb = out, sk.apply(b4)[:, :1]
    Q = torch.linalg.qr(A.double()).Q
    SQ = sk.apply(Q.to(A.dtype).contiguous())
    return {
        "kernel_ms": sum(ms) / len(ms),
        "apply_ms": apply_ms,
        "gram_rel": gram_error(A, SA),
        "ose": ose_error(SQ),
        "ridge_resid": ridge_residual(A, b, SA, Sb, lam),
        "lstsq_resid": lstsq_residual(A, b, SA, Sb),
    }


def sweep(d, n, k, data, Bc=None, Br=None, s=2, kappas=(1, 2, 4), seed=0, device="cuda"):
    from . import binding as B
    A, b = make_data(data, d, n, 1, device)
    Br = Br or 32
    M = k // Br
    Bc = Bc or d // M
    res = {"problem": {"d": d, "n": n, "k": k, "data": data, "Bc": Bc, "Br": Br, "s": s}}
    x = torch.linalg.lstsq(A.double(), b.double()).solution
    res["unsketched_lstsq_resid"] = float(torch.linalg.norm(A.double() @ x - b.double()) / torch.linalg.norm(b.double()))
    for kappa in kappas:
        if kappa <= M:
            sk = B.Sketch(d, k, Bc, Br, kappa, s, seed=seed)
            res[f"blockperm_kappa{kappa}_s{s}"] = evaluate(sk, A, b)
    for name, kind, args in (
        ("plain_sjlt_scatter_s%d" % min(32, s * max(kappas)), B.KIND_SJLT_SCATTER,
         (d, k, d, k, 1, min(32, s * max(kappas)))),
        ("blockrow_kappa%d_s%d" % (max(kappas), s), B.KIND_BLOCKROW, (d, k, Bc, Br, min(max(kappas), M), s)),
        ("dense_gaussian", B.KIND_GAUSS_DENSE, (d, k, d, k, 1, 1)),
    ):
        try:
            res[name] = evaluate(B.Sketch(*args, seed=seed, kind=kind), A, b)
        except B.FlashSketchError as e:
            res[name] = {"error": str(e)}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--d", type=int, default=65536)
    ap.add_argument("--n", type=int, default=1024)
    ap.add_argument("--k", type=int, default=4096)
    ap.add_argument("--data", default="gaussian", choices=["gaussian", "lowrank", "oneblock"])
    ap.add_argument("--kappas", default="1,2,4", help="comma-separated wiring parameters to sweep")
    a = ap.parse_args()
    print(json.dumps(sweep(a.d, a.n, a.k, a.data, kappas=tuple(int(x) for x in a.kappas.split(","))), indent=1))


if __name__ == "__main__":
    main()
