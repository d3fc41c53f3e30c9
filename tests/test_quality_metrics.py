"""The quality read-outs (paper Appendix G, "Metrics"): the torch implementations against the
plain NumPy definitions on small problems (CPU), and a sanity sweep on the GPU."""
import numpy as np
import pytest
import torch

from oracle import blockperm as O
from paper_2602_06071_amd import quality as Q


def test_metric_definitions_against_numpy():
    rng = np.random.default_rng(0)
    p = O.Params(512, 64, 64, 8, 2, 2)
    S = O.build_csc(p, 1).toarray()
    A = rng.standard_normal((p.d, 6))
    b = rng.standard_normal((p.d, 1))
    SA, Sb = S @ A, S @ b
    tA, tb, tSA, tSb = (torch.from_numpy(x) for x in (A, b, SA, Sb))
    G = A.T @ A
    assert abs(Q.gram_error(tA, tSA) - np.linalg.norm(SA.T @ SA - G) / np.linalg.norm(G)) < 1e-12
    Qm = np.linalg.qr(A)[0]
    SQ = S @ Qm
    assert abs(Q.ose_error(torch.from_numpy(SQ)) - np.linalg.norm(SQ.T @ SQ - np.eye(6), 2)) < 1e-12
    assert abs(Q.ose_error(torch.from_numpy(SQ)) - O.ose_error(SQ)) < 1e-12
    lam = 0.3
    x = np.linalg.solve(SA.T @ SA + lam * np.eye(6), SA.T @ Sb)
    assert abs(Q.ridge_residual(tA, tb, tSA, tSb, lam) - np.linalg.norm(A @ x - b) / np.linalg.norm(b)) < 1e-12
    x = np.linalg.lstsq(SA, Sb, rcond=None)[0]
    assert abs(Q.lstsq_residual(tA, tb, tSA, tSb) - np.linalg.norm(A @ x - b) / np.linalg.norm(b)) < 1e-10
    # degenerate denominators fall back to absolute errors
    z = torch.zeros((p.d, 6), dtype=torch.float64)
    assert Q.gram_error(z, tSA) == pytest.approx(float(np.linalg.norm(SA.T @ SA)))
    assert Q.ridge_residual(tA, torch.zeros_like(tb), tSA, torch.zeros_like(tSb), lam) == 0.0


@pytest.mark.gpu
@pytest.mark.parametrize("data", ["gaussian", "lowrank"])
def test_quality_sweep_is_sane(data):
    res = Q.sweep(16384, 256, 2048, data, Br=32, s=2, kappas=(1, 4))
    gauss = res["dense_gaussian"]
    for name, r in res.items():
        if not isinstance(r, dict) or "gram_rel" not in r:
            continue
        print(name, r, flush=True)
        assert r["kernel_ms"] > 0
        if name.startswith("blockrow"):
            continue  # no subspace-embedding guarantee (Appendix D): only reported
        # JL-type sketches of the same k agree to a small factor on incoherent inputs
        assert r["gram_rel"] < 3.0 * gauss["gram_rel"] + 0.02, name
        assert r["ose"] < 1.0, name
        assert res["unsketched_lstsq_resid"] - 1e-9 <= r["lstsq_resid"] < 2.0 * res["unsketched_lstsq_resid"] + 0.05, name


@pytest.mark.gpu
@pytest.mark.parametrize("data", ["gaussian", "lowrank"])
@pytest.mark.parametrize("kappa", [1, 4])
def test_metrics_from_the_gpu_apply_match_the_oracles(data, kappa):
    """Appendix G "Metrics" on the BlockPerm rows of the 16384 x 256 sweep: the four figures the
    harness derives from the HIP apply (fp32) against the same figures derived, with plain NumPy
    formulas, from the oracle's float64 S A, S b and S Q on the same inputs.  The sketch is the
    same linear map on both sides, so they agree to fp32 accumulation error."""
    from paper_2602_06071_amd import binding as B
    d, n, k, Br, s, seed = 16384, 256, 2048, 32, 2, 0
    M = k // Br
    Bc = d // M
    A, b = Q.make_data(data, d, n, 1, "cuda")
    sk = B.Sketch(d, k, Bc, Br, kappa, s, seed=seed)
    got = Q.evaluate(sk, A, b, lam=1e-2)
    print(data, kappa, got, flush=True)
    # the oracle's side, all in float64 NumPy
    S = O.build_csc(O.Params(d, k, Bc, Br, kappa, s), seed)
    A64, b64 = A.cpu().double().numpy(), b.cpu().double().numpy()
    SA, Sb = O.apply(S, A64), O.apply(S, b64)
    G = A64.T @ A64
    want_gram = np.linalg.norm(SA.T @ SA - G) / np.linalg.norm(G)
    Q32 = torch.linalg.qr(A.double()).Q.to(A.dtype).cpu().double().numpy()   # the harness sketches fp32(Q)
    SQ = O.apply(S, Q32)
    want_ose = np.linalg.norm(SQ.T @ SQ - np.eye(n), 2)
    x = np.linalg.solve(SA.T @ SA + 1e-2 * np.eye(n), SA.T @ Sb)
    want_ridge = np.linalg.norm(A64 @ x - b64) / np.linalg.norm(b64)
    x = np.linalg.lstsq(SA, Sb, rcond=None)[0]
    want_lstsq = np.linalg.norm(A64 @ x - b64) / np.linalg.norm(b64)
    for name, want in (("gram_rel", want_gram), ("ose", want_ose), ("ridge_resid", want_ridge),
                       ("lstsq_resid", want_lstsq)):
        assert abs(got[name] - want) <= 1e-4 * abs(want), (name, got[name], want)
    sk.close()
