#!/usr/bin/env python3
"""Benchmark of the BlockPerm-SJLT sketch apply on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload grad] [--no-extra]

A step is one pass of the whole hot path over one batch of synthetic input: for
the default workload (the per-example-gradient configuration, 8 GiB bf16) that
is four fs_sketch_apply_ld calls on 256-column views of one resident matrix,
back to back on one stream.  Inputs are resident in HBM before the timed region.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import dataclasses
import functools
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E bandwidth
# HBM bytes per launch of the dominant kernel on the default workload, from the rocprofv3
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/blockperm_mfma_grad_bf16_chunk256.md
MEASURED_TRAFFIC = {("grad", "mfma"): (2_097_533 + 22_528) * 1024}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="grad", choices=["tiny", "mid", "tall", "wide", "grad"])
    ap.add_argument("--variant", default="auto", choices=["auto", "generic", "mfma"])
    ap.add_argument("--layout", default="cols", choices=["cols", "rows"],
                    help="cols: A is d x n, vectors are columns (the default, the metric's workload); "
                         "rows: the same data held n x d, vectors are rows (fs_sketch_apply_rows)")
    ap.add_argument("--ld-pad", type=int, default=64, help="rows layout: row stride = d + this many elements")
    ap.add_argument("--no-extra", action="store_true", help="skip the side measurements")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    return ap.parse_args()


def chunks_of(cfg):
    w = cfg.chunk if cfg.chunk else cfg.n
    return [(c, min(cfg.n, c + w)) for c in range(0, cfg.n, w)]


def run_steps(sk, A, out, cfg, steps, rows=False):
    for _ in range(steps):
        for c0, c1 in chunks_of(cfg):
            if rows:
                sk.apply_rows(A[c0:c1], out[c0:c1])
            else:
                sk.apply(A[:, c0:c1], out[:, c0:c1])


def time_workload(torch, B, cfg, A, variant, steps, warmup, kind=None, sketch_params=None, rows=False):
    """Wall-clock over `steps` steps plus HIP-event durations of the dominant kernel.
    rows: A is the n x d matrix of the examples-as-rows layout and out is n x k."""
    params = sketch_params or cfg.params
    sk = B.Sketch(*params, seed=cfg.sketch_seed, kind=B.KIND_BLOCKPERM if kind is None else kind)
    if kind is None:
        sk.set_variant({"auto": B.VARIANT_AUTO, "generic": B.VARIANT_GENERIC, "mfma": B.VARIANT_MFMA}[variant])
    out = torch.empty((cfg.n, cfg.k) if rows else (cfg.k, cfg.n), device=A.device, dtype=cfg.dtype)
    run_steps = functools.partial(globals()["run_steps"], rows=rows)
    run_steps(sk, A, out, cfg, warmup)
    torch.cuda.synchronize()
    # HIP-event brackets around the dominant kernel on the last two timed steps only: every
    # bracket costs ~2 us of queue time, so bracketing all launches would slow the timed region
    # (the host runs far ahead of the GPU, so creating the events mid-loop stalls nothing)
    n_brk = min(steps, 2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(sk, A, out, cfg, steps - n_brk)
    sk.profile_begin(n_brk * len(chunks_of(cfg)))
    run_steps(sk, A, out, cfg, n_brk)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms = sk.profile_end()
    used = sk.info().last_variant
    sk.close()
    return (t1 - t0) / steps, kernel_ms, used, out


def cpu_baseline(torch, cfg, A, budget_s=12.0, slice_cols=32):
    """The float64 oracle, as it stands, on a bounded sample of the same workload:
    the CSC product S @ A[:, cols] over leading column slices until ~budget_s of CPU
    time is spent (each slice is widened to float64 on the host first)."""
    from oracle import blockperm as O
    t0 = time.perf_counter()
    S = O.build_csc(O.Params(*cfg.params), cfg.sketch_seed)
    t_build = time.perf_counter() - t0
    t_apply, cols, outs = 0.0, 0, []
    while cols < cfg.n and t_apply < budget_s:
        c1 = min(cfg.n, cols + slice_cols)
        A_host = A[:, cols:c1].to("cpu").to(torch.float64).numpy()
        t0 = time.perf_counter()
        outs.append(O.apply(S, A_host))
        t_apply += time.perf_counter() - t0
        cols = c1
    import numpy as np
    Y = np.concatenate(outs, axis=1)
    gbps = cfg.d * cols * cfg.elt / t_apply / 1e9
    return {
        "value": gbps, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {cols} of {cfg.n} columns of the same A (all {cfg.d} rows), float64 CSC product "
                  f"{t_apply:.2f} s; building S as CSC took {t_build:.2f} s more and is not counted",
        "cols_per_s": cols / t_apply,
    }, Y, cols


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: the sketch apply shards over columns with no exchange step, "
              "so this build has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_06071_amd import binding as B
    from paper_2602_06071_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = "cuda:0"
    cfg = W.CONFIGS[args.workload]
    A = W.make_input(cfg, dev)
    torch.cuda.synchronize()

    rows = args.layout == "rows"
    if rows:  # the same values, one example per row, row stride d + ld_pad elements
        Gbuf = torch.empty((cfg.n, cfg.d + args.ld_pad), device=dev, dtype=cfg.dtype)
        Gbuf[:, :cfg.d].copy_(A.t())
        del A
        A = Gbuf[:, :cfg.d]
        torch.cuda.synchronize()
    sec_per_step, kernel_ms, used, out = time_workload(torch, B, cfg, A, args.variant, args.steps, args.warmup,
                                                       rows=rows)
    n_launch = len(chunks_of(cfg))
    cols_per_launch = cfg.n // n_launch
    # algorithmic bytes of one launch: read its columns of A once, write its columns of SA once
    alg_bytes = cols_per_launch * (cfg.d * cfg.elt + cfg.k * cfg.elt)
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    achieved = alg_bytes / avg_kernel_s / 1e9
    value = cfg.a_bytes / sec_per_step / 1e9

    rec = {
        "metric": "sketch-apply GB/s of A streamed",
        "value": value, "unit": "GB/s",
        "pct_hbm_peak": 100.0 * value / HBM_PEAK_GBPS,
        "cols_per_s": cfg.n / sec_per_step,
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.elt == 2 else "f32", "data": "synthetic",
        "config": {
            "workload": f"{cfg.name}: A {cfg.d}x{cfg.n} {'bf16' if cfg.elt == 2 else 'fp32'}, k={cfg.k}, "
                        f"Bc={cfg.Bc}, Br={cfg.Br}, s={cfg.s}, kappa={cfg.kappa}, "
                        f"{n_launch} launch(es) of {cols_per_launch} columns per step"
                        + (f"; held examples-as-rows ({cfg.n} x {cfg.d}, row stride d+{args.ld_pad})" if rows else ""),
            "variant": {1: "generic", 2: "mfma"}.get(used, str(used)),
            "accumulate": "fp32",
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": None if rows else MEASURED_TRAFFIC.get((cfg.name, {1: "generic", 2: "mfma"}.get(used))),
            "kernel_ms_avg": avg_kernel_s * 1e3, "launches_timed": len(kernel_ms),
            "algorithmic_bytes_per_launch": alg_bytes,
        },
    }

    if not args.no_cpu:
        from oracle import blockperm as O  # the CPU-baseline leg is the only user of the oracle here
        base, Y, cols = cpu_baseline(torch, cfg, A.t() if rows else A)
        got = out[:cols].t() if rows else out[:, :cols]
        err = O.rel_fro_err(got.to("cpu").to(torch.float64).numpy(), Y)
        rec["cpu_baseline"] = base
        rec["rel_fro_err_vs_oracle_on_sample"] = err

    if not args.no_extra and not rows:
        rec["extra"] = extra_measurements(torch, B, W, dev, cfg.name, with_oracle=not args.no_cpu)
        rec["extra"]["rows_layout"] = rows_layout_measurement(torch, B, cfg, A, out)
    print(json.dumps(rec))


def extra_measurements(torch, B, W, dev, skip, with_oracle):
    """Short side measurements on the other configurations (kernel time by HIP
    events, 5 launches each): the kappa sweep with the plain-SJLT scatter and
    dense-Gaussian reference points, the tall matrix, and the bf16 width sweep."""
    res = {}

    def one(cfg, A, **kw):
        try:
            _, ms, used, _ = time_workload(torch, B, cfg, A, "auto", 5, 2, **kw)
        except B.FlashSketchError as e:
            return {"error": str(e)}
        t = sum(ms) / len(ms) / 1e3
        return {"kernel_ms": t * 1e3, "GBps_A": cfg.a_bytes / len(chunks_of(cfg)) / t / 1e9,
                "variant": used}

    def cold(cfg, A, reps=5):
        """Kernel time of single applies, each after 2 GiB of unrelated writes have gone through the
        caches (L2 and the 256 MB Infinity Cache hold nothing of A or of the workspace)."""
        sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
        out = sk.apply(A)
        junk = torch.empty(1 << 29, device=dev, dtype=torch.float32)
        ms = []
        for i in range(reps):
            junk.fill_(float(i))
            sk.profile_begin(1)
            sk.apply(A, out)
            ms += sk.profile_end()
        sk.close()
        t = sum(ms) / len(ms) / 1e3
        return {"kernel_ms": t * 1e3, "GBps_A": cfg.a_bytes / t / 1e9}

    for name in ("tiny", "tall"):
        if name != skip:
            cfg = W.CONFIGS[name]
            A = W.make_input(cfg, dev)
            res[name] = one(cfg, A)
            if name == "tall":  # 256 MiB: about the size of the Infinity Cache, so also time it cold
                res["tall_cold"] = cold(cfg, A)
            del A
    if skip != "tall":
        res["tall_ose"] = tall_distortion(torch, B, W, dev, with_oracle)
    if skip != "mid":
        base = W.CONFIGS["mid"]
        A = W.make_input(base, dev)
        for kappa in W.MID_KAPPAS:
            res[f"mid_kappa{kappa}"] = one(dataclasses.replace(base, kappa=kappa), A)
        for s in (8, 32):
            res[f"mid_plain_sjlt_scatter_s{s}"] = one(
                base, A, kind=B.KIND_SJLT_SCATTER, sketch_params=(base.d, base.k, base.d, base.k, 1, s))
        res["mid_dense_gaussian"] = one(base, A, kind=B.KIND_GAUSS_DENSE)
        res["mid_blockrow"] = one(base, A, kind=B.KIND_BLOCKROW)  # gather variant, reads k*kappa*s rows
        del A
    if skip != "wide":
        base = W.CONFIGS["wide"]
        A = W.make_input(base, dev)
        for n in W.WIDE_NS:
            res[f"wide_n{n}"] = one(dataclasses.replace(base, n=n), A[:, :n].contiguous())
        del A
    return res


def rows_layout_measurement(torch, B, cfg, A, out, steps=10):
    """The same workload held examples-as-rows (G = A^T, n x d; out^T, n x k): fs_sketch_apply_rows
    on the same chunks of `chunk` examples, once with the packed row stride ld = d and once with
    ld = d + 64 elements (a power-of-two stride maps all rows of a tile to one HBM channel).  The
    result is compared with the column-layout output of the main measurement."""
    res = {}
    for pad in (64, 0):
        try:
            Gbuf = torch.empty((cfg.n, cfg.d + pad), device=A.device, dtype=A.dtype)
            G = Gbuf[:, :cfg.d]
            G.copy_(A.t())
            sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
            o = torch.empty((cfg.n, cfg.k), device=A.device, dtype=A.dtype)
            w = cfg.chunk if cfg.chunk else cfg.n

            def step():
                for c in range(0, cfg.n, w):
                    sk.apply_rows(G[c:c + w], o[c:c + w])
            step(); step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                step()
            torch.cuda.synchronize()
            t = (time.perf_counter() - t0) / steps
            diff = (o.t().float() - out.float()).norm() / out.float().norm()
            res[f"ld_d_plus_{pad}"] = {"ms_per_step": t * 1e3, "GBps_A": cfg.a_bytes / t / 1e9,
                                       "rel_diff_vs_column_layout": float(diff)}
            sk.close()
            del Gbuf, G, o
        except B.FlashSketchError as e:
            res[f"ld_d_plus_{pad}"] = {"error": str(e)}
    return res


def tall_distortion(torch, B, W, dev, with_oracle):
    """Subspace-embedding distortion ||(SQ)^T (SQ) - I||_2 of S on col(A) for the coherent tall
    matrix (Q from a float64 QR of A; Appendix G, "OSE spectral error"), from the GPU apply on
    fp32(Q).  With the CPU leg enabled the oracle's value for the same Q is reported beside it,
    and the block / neighbourhood coherence of Q that the paper's OSE bound is stated in."""
    import numpy as np
    cfg = W.CONFIGS["tall"]
    A64, _ = W.coherent_tall(cfg.d, cfg.n, cfg.data_seed)
    Q = np.linalg.qr(A64.numpy())[0]
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    SQ = sk.apply(torch.from_numpy(Q).to(torch.float32).to(dev)).cpu().double().numpy()
    i = sk.info()
    res = {"ose_error_gpu": float(np.linalg.norm(SQ.T @ SQ - np.eye(cfg.n), 2))}
    if with_oracle:
        from oracle import blockperm as O
        S = O.build_csc(O.Params(*cfg.params), cfg.sketch_seed)
        res.update(ose_error_oracle=O.ose_error(O.apply(S, Q)), mu_blk=O.block_coherence(Q, i.M),
                   mu_nbr=O.nbr_coherence(Q, i.M, i.a, i.b, cfg.kappa))
    return res


if __name__ == "__main__":
    main()
