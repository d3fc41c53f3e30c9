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
# FETCH_SIZE / WRITE_SIZE runs summarised in profiles/blockperm_mfma_grad_bf16_chunk256.md, with
# the kernel instantiation they were measured on (fs_info.last_kernel): reported only while the
# library still launches that instantiation for the workload, else null.
MEASURED_TRAFFIC = {
    "grad": ("mfma_kernel<bf16,2,1,2,in,4,4,1,-,->+reduce_planes", (2_097_533 + 22_528) * 1024),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="grad", choices=["tiny", "mid", "tall", "wide", "grad"])
    ap.add_argument("--kappa", type=int, default=0, help="override the workload's kappa (profiling runs of mid and wide)")
    ap.add_argument("--variant", default="auto", choices=["auto", "generic", "mfma"])
    ap.add_argument("--layout", default="cols", choices=["cols", "rows"],
                    help="cols: A is d x n, vectors are columns (the default, the metric's workload); "
                         "rows: the same data held n x d, vectors are rows (fs_sketch_apply_rows)")
    ap.add_argument("--ld-pad", type=int, default=64, help="rows layout: row stride = d + this many elements")
    ap.add_argument("--no-extra", action="store_true", help="skip the side measurements")
    ap.add_argument("--extras", default="", help="run only these side measurements (known: tall_cold)")
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


def time_workload(torch, B, cfg, A, variant, steps, warmup, kind=None, sketch_params=None, rows=False, brackets=2):
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
    # HIP-event brackets on the last 2 x `brackets` timed steps only: every recorded event costs a
    # few microseconds of queue time, so bracketing all launches would slow the timed region.
    # `brackets` steps bracket the whole apply (one pair around all its kernels, nothing in
    # between), the last `brackets` the dominant kernel alone.  (The host runs far ahead of the GPU, so creating the events
    # mid-loop stalls nothing.)
    n_brk = min(steps // 2, brackets)
    n_l = len(chunks_of(cfg))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(sk, A, out, cfg, steps - 2 * n_brk)
    apply_ms = []
    if n_brk:
        sk.profile_begin(n_brk * n_l, B.PROFILE_APPLY)
        run_steps(sk, A, out, cfg, n_brk)
        apply_ms = sk.profile_end(whole=True)[1]     # (waits for those steps)
        sk.profile_begin(n_brk * n_l, B.PROFILE_KERNEL)
        run_steps(sk, A, out, cfg, n_brk)
    else:
        sk.profile_begin(steps * n_l)
        run_steps(sk, A, out, cfg, steps)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kernel_ms, both = sk.profile_end(whole=True)
    apply_ms = apply_ms or both
    info = sk.info()
    sk.close()
    return Timing((t1 - t0) / steps, kernel_ms, apply_ms, info.last_variant, info.last_kernel.decode()), out


@dataclasses.dataclass
class Timing:
    sec_per_step: float      # wall clock
    kernel_ms: list          # HIP events around the dominant kernel of each bracketed apply
    apply_ms: list           # HIP events around everything each bracketed apply enqueued
    variant: int
    kernel: str              # fs_info.last_kernel

    @property
    def kernel_s(self):
        return sum(self.kernel_ms) / len(self.kernel_ms) / 1e3

    @property
    def apply_s(self):
        return sum(self.apply_ms) / len(self.apply_ms) / 1e3


_POOL_STATE = {}


def _pool_leg(j):
    """One worker's share of the all-core leg: the oracle's product on its own column slice."""
    from oracle import blockperm as O
    t0 = time.perf_counter()
    Y = O.apply(_POOL_STATE["S"], _POOL_STATE["slices"][j])
    return time.perf_counter() - t0, float(abs(Y).sum())


def cpu_baseline(torch, cfg, A, budget_s=10.0, slice_cols=32):
    """The float64 oracle, as it stands, on a bounded sample of the same workload, on the box's
    own host cores.  Leg 1, one core: the CSC product S @ A[:, cols] over leading column slices
    until ~budget_s of CPU time is spent (each slice is widened to float64 on the host first).
    Leg 2, all cores the process may run on (os.sched_getaffinity): one slice of the same width
    per core, each in a forked worker that runs the same single-threaded product (columns are
    independent, so sharding them is all there is to a parallel oracle); wall clock of the slowest.
    `value` is the all-core figure when that leg ran, else the one-core figure."""
    from oracle import blockperm as O
    import numpy as np
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
    Y = np.concatenate(outs, axis=1)
    one = cfg.d * cols * cfg.elt / t_apply / 1e9
    box_cores = len(os.sched_getaffinity(0))
    res = {
        "value": one, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": f"first {cols} of {cfg.n} columns of the same A (all {cfg.d} rows), float64 CSC product "
                  f"{t_apply:.2f} s on one core; building S as CSC took {t_build:.2f} s more and is not counted",
        "cols_per_s": cols / t_apply,
        "one_core": {"value": one, "cols_per_s": cols / t_apply, "seconds": t_apply, "columns": cols},
        "host_cores_available": box_cores,
    }
    # all-core leg: up to 64 columns per core (2 GiB of float64 each at d = 4 M), fewer when there
    # are not that many columns
    try:
        import multiprocessing as mp
        per_core = max(1, min(64, cfg.n // max(1, box_cores)))
        workers = min(box_cores, cfg.n // per_core)
        if workers >= 2:
            _POOL_STATE["S"] = S
            _POOL_STATE["slices"] = [A[:, j * per_core:(j + 1) * per_core].to("cpu").to(torch.float64).numpy()
                                     for j in range(workers)]
            ctx = mp.get_context("fork")  # the workers only run NumPy / SciPy code on inherited host arrays
            with ctx.Pool(workers) as pool:
                pool.map(_pool_leg, range(workers), chunksize=1)  # spin the workers up (untimed)
                t0 = time.perf_counter()
                legs = pool.map_async(_pool_leg, range(workers), chunksize=1).get(timeout=180)
                wall = time.perf_counter() - t0
            allc = cfg.d * per_core * workers * cfg.elt / wall / 1e9
            res.update({
                "value": allc, "cores": workers, "cols_per_s": per_core * workers / wall,
                "sample": res["sample"] + f"; all-core leg: {workers} forked workers x {per_core} columns each of the "
                          f"same A, {wall:.2f} s wall (slowest worker {max(t for t, _ in legs):.2f} s)",
                "all_cores": {"value": allc, "cores": workers, "seconds": wall, "columns": per_core * workers},
            })
            _POOL_STATE.clear()
    except Exception as e:  # the one-core leg stands on its own
        res["all_cores"] = {"error": f"{type(e).__name__}: {e}"}
    return res, Y, cols


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
    if args.kappa:
        import dataclasses
        cfg = dataclasses.replace(cfg, kappa=args.kappa)
    A = W.make_input(cfg, dev)
    torch.cuda.synchronize()

    rows = args.layout == "rows"
    if rows:  # the same values, one example per row, row stride d + ld_pad elements
        Gbuf = torch.empty((cfg.n, cfg.d + args.ld_pad), device=dev, dtype=cfg.dtype)
        Gbuf[:, :cfg.d].copy_(A.t())
        del A
        A = Gbuf[:, :cfg.d]
        torch.cuda.synchronize()
    tm, out = time_workload(torch, B, cfg, A, args.variant, args.steps, args.warmup, rows=rows)
    sec_per_step, used = tm.sec_per_step, tm.variant
    n_launch = len(chunks_of(cfg))
    cols_per_launch = cfg.n // n_launch
    # algorithmic bytes of one launch: read its columns of A once, write its columns of SA once
    alg_bytes = cols_per_launch * (cfg.d * cfg.elt + cfg.k * cfg.elt)
    a_bytes_launch = cols_per_launch * cfg.d * cfg.elt
    # The roofline figure divides by the time of EVERYTHING one apply enqueues (the kernel that
    # streams A and, where the output is written by a second kernel, that one too), so that the
    # bytes counted and the time counted belong together; the dominant kernel's own duration is
    # reported beside it (it is the one a rocprofv3 kernel trace shows).
    achieved = alg_bytes / tm.apply_s / 1e9
    value = cfg.a_bytes / sec_per_step / 1e9
    traffic = None
    if not rows and cfg.name in MEASURED_TRAFFIC and MEASURED_TRAFFIC[cfg.name][0] == tm.kernel:
        traffic = MEASURED_TRAFFIC[cfg.name][1]

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
            "traffic": traffic,
            "kernel": tm.kernel,
            "basis": "algorithmic bytes of one launch / HIP-event time of the whole apply (all its kernels)",
            "apply_ms_avg": tm.apply_s * 1e3,
            "kernel_ms_avg": tm.kernel_s * 1e3,
            "frac_dominant_kernel_reading_A": a_bytes_launch / tm.kernel_s / 1e9 / HBM_PEAK_GBPS,
            "launches_timed": len(tm.kernel_ms),
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
        only = set(args.extras.split(",")) if args.extras else None
        rec["extra"] = extra_measurements(torch, B, W, dev, cfg.name, with_oracle=not args.no_cpu, only=only)
        if only is not None:
            print(json.dumps(rec))
            return
        if cfg.name == "grad":
            rec["extra"].update(grad_side_measurements(torch, B, cfg, A, out))
        rec["extra"]["rows_layout"] = rows_layout_measurement(torch, B, cfg, A, out)
    print(json.dumps(rec))


def extra_measurements(torch, B, W, dev, skip, with_oracle, only=None):
    """Short side measurements on the other configurations (kernel time by HIP
    events, 5 launches each): the kappa sweep with the plain-SJLT scatter and
    dense-Gaussian reference points, the tall matrix, and the bf16 width sweep."""
    res = {}

    def one(cfg, A, **kw):
        """kernel_ms: the dominant kernel; apply_ms: everything the apply enqueues (zero-fills, plane
        reductions, conversions included); GBps_A and roofline_frac are computed from apply_ms."""
        try:
            # (enough warm-up for the clocks to settle: the matrix-core-bound shapes run 10-15 %
            # slower in their first few launches)
            tm, _ = time_workload(torch, B, cfg, A, "auto", 24, 8, brackets=8, **kw)
        except B.FlashSketchError as e:
            return {"error": str(e)}
        n_l = len(chunks_of(cfg))
        alg = (cfg.a_bytes + cfg.k * cfg.n * cfg.elt) / n_l
        return {"kernel_ms": tm.kernel_s * 1e3, "apply_ms": tm.apply_s * 1e3,
                "GBps_A": cfg.a_bytes / n_l / tm.apply_s / 1e9,
                "roofline_frac": alg / tm.apply_s / 1e9 / HBM_PEAK_GBPS,
                "variant": tm.variant, "kernel": tm.kernel}

    def cold(cfg, A, flush, reps=5):
        """Kernel time of single applies, each after 2 GiB of unrelated traffic has gone through the
        caches, so that L2 and the 256 MB Infinity Cache hold nothing of A or of the workspace.
        flush = "write": the 2 GiB are written (the caches are left full of DIRTY lines, which the
        apply's own fetches then have to push out to HBM first); flush = "read": they are only read
        (clean lines, dropped for free).  The difference between the two is the write-back, not the
        kernel."""
        sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
        out = sk.apply(A)
        junk = torch.empty(1 << 29, device=dev, dtype=torch.float32)
        junk.fill_(1.0)
        ms, ms_all = [], []
        for i in range(reps):
            if flush == "write":
                junk.fill_(float(i))
            else:
                junk.sum()
            sk.profile_begin(1)
            sk.apply(A, out)
            k_ms, a_ms = sk.profile_end(whole=True)
            ms += k_ms
            ms_all += a_ms
        sk.close()
        t = sum(ms_all) / len(ms_all) / 1e3
        return {"flush": "2 GiB of " + flush + "s", "kernel_ms": sum(ms) / len(ms), "apply_ms": t * 1e3,
                "GBps_A": cfg.a_bytes / t / 1e9,
                "roofline_frac": (cfg.a_bytes + cfg.k * cfg.n * cfg.elt) / t / 1e9 / HBM_PEAK_GBPS}

    if only is not None:  # --extras tall_cold: just that pair (profiling runs)
        assert only == {"tall_cold"}, "--extras knows: tall_cold"
        cfg = W.CONFIGS["tall"]
        A = W.make_input(cfg, dev)
        res["tall_cold"] = cold(cfg, A, "write")
        res["tall_cold_after_reads"] = cold(cfg, A, "read")
        return res
    for name in ("tiny", "tall"):
        if name != skip:
            cfg = W.CONFIGS[name]
            A = W.make_input(cfg, dev)
            res[name] = one(cfg, A)
            if name == "tall":  # 256 MiB: about the size of the Infinity Cache, so also time it cold
                res["tall_cold"] = cold(cfg, A, "write")
                res["tall_cold_after_reads"] = cold(cfg, A, "read")
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


def grad_side_measurements(torch, B, cfg, A, out, steps=10):
    """Two more views of the gradient workload.  (1) The prior-art plain-SJLT scatter at the same
    k on one 256-column chunk of the same A, at s nonzeros per column (equal s) and at kappa*s
    (equal nonzeros per column of S), whole apply (zero-fill, atomics, conversion).  (2) The same
    step on four separate packed d x 256 buffers (lda = 256), as a pipeline that hands over one
    chunk at a time would hold them, instead of column views of one d x 1024 matrix."""
    res = {}
    w = cfg.chunk
    chunk_cfg = dataclasses.replace(cfg, n=w, chunk=0)
    for s_nz in (cfg.s, cfg.s * cfg.kappa):
        try:
            tm, _ = time_workload(torch, B, chunk_cfg, A[:, :w], "auto", 3, 1, kind=B.KIND_SJLT_SCATTER,
                                  sketch_params=(cfg.d, cfg.k, cfg.d, cfg.k, 1, s_nz))
            res[f"grad_chunk_plain_sjlt_scatter_s{s_nz}"] = {
                "kernel_ms": tm.kernel_s * 1e3, "apply_ms": tm.apply_s * 1e3,
                "GBps_A": chunk_cfg.a_bytes / tm.apply_s / 1e9}
        except B.FlashSketchError as e:
            res[f"grad_chunk_plain_sjlt_scatter_s{s_nz}"] = {"error": str(e)}
    try:
        bufs = [A[:, c:c + w].contiguous() for c in range(0, cfg.n, w)]
        o = torch.empty_like(out)
        sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)

        def step():
            for j, buf in enumerate(bufs):
                sk.apply(buf, o[:, j * w:(j + 1) * w])
        step(); step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / steps
        sk.profile_begin(len(bufs))
        step()
        k_ms, a_ms = sk.profile_end(whole=True)
        res["grad_packed_chunks_lda256"] = {
            "ms_per_step": t * 1e3, "GBps_A": cfg.a_bytes / t / 1e9, "pct_hbm_peak": 100.0 * cfg.a_bytes / t / 1e9 / HBM_PEAK_GBPS,
            "kernel_ms": sum(k_ms) / len(k_ms), "apply_ms": sum(a_ms) / len(a_ms),
            "bit_identical_to_column_views": bool(torch.equal(o, out))}
        sk.close()
        del bufs, o
    except B.FlashSketchError as e:
        res["grad_packed_chunks_lda256"] = {"error": str(e)}
    # (3) What a library reduction reads per second from one CONTIGUOUS 2 GiB chunk (torch.max over
    # its int32 view: every byte read once, 8 bytes written): a reference point for the stream
    # rate of this machine, next to the 512-of-every-2048-bytes view the apply reads.
    try:
        flat = A[:, :w].contiguous().view(torch.int32)
        for _ in range(3):
            flat.max()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        torch.cuda.synchronize()
        ev[0].record()
        for _ in range(8):
            flat.max()
        ev[1].record()
        torch.cuda.synchronize()
        ms = ev[0].elapsed_time(ev[1]) / 8
        res["contiguous_chunk_read_by_torch_max"] = {"ms": ms, "GBps": chunk_cfg.a_bytes / ms / 1e6,
                                                     "pct_hbm_peak": 100.0 * chunk_cfg.a_bytes / ms / 1e6 / HBM_PEAK_GBPS}
        del flat
    except RuntimeError as e:
        res["contiguous_chunk_read_by_torch_max"] = {"error": str(e)}
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
