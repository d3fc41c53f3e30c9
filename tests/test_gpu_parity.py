"""GPU parity: every result of the HIP path, called through the C ABI, against
the float64 oracle on the same seeded inputs.

Bars: indices and signs bit-exact; relative Frobenius error <= 1e-5 for fp32
inputs, <= 4e-3 for bf16 and <= 5e-4 for half inputs/outputs with fp32
accumulation (the one rounding of the result to 8 resp. 11 significant bits
bounds it by 2^-8 resp. 2^-11 = 4.9e-4; the fp32 sum adds about 1e-6).
"""
import functools
import gc

import numpy as np
import pytest
import torch

from oracle import blockperm as O
from paper_2602_06071_amd import binding as B
from paper_2602_06071_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = {torch.float32: 1e-5, torch.bfloat16: 4e-3, torch.float16: 5e-4}
ETOL = {torch.float32: 2e-5, torch.bfloat16: 8e-3, torch.float16: 1e-3}   # element-wise, see the uses
DTYPES = pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16], ids=["f32", "bf16", "f16"])
VARIANTS = [B.VARIANT_GENERIC, B.VARIANT_MFMA]
VNAME = {B.VARIANT_GENERIC: "generic", B.VARIANT_MFMA: "mfma", B.VARIANT_AUTO: "auto"}


@functools.lru_cache(maxsize=8)
def oracle_csc(params, seed):
    return O.build_csc(O.Params(*params), seed)


def host64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def check(out, ref, dtype, what=""):
    err = O.rel_fro_err(host64(out), ref)
    assert err <= TOL[dtype], f"{what}: rel. Frobenius error {err:.3e} > {TOL[dtype]:.0e}"
    return err


def make_sketch(params, seed, variant):
    sk = B.Sketch(*params, seed=seed)
    sk.set_variant(variant)
    return sk


def apply_or_skip(sk, A, out=None):
    try:
        return sk.apply(A, out)
    except B.FlashSketchError as e:
        if e.status == 2:
            pytest.skip("variant does not support this shape")
        raise


# ------------------------------------------------------------ export ------
@pytest.mark.parametrize("params", [
    (4000, 256, 512, 32, 2, 4), (65500, 8192, 64, 8, 8, 2),
    (4096, 256, 512, 32, 2, 4), (2048, 1024, 128, 64, 4, 2), (1152, 72, 96, 6, 5, 3),
    (1440, 180, 80, 10, 18, 10), (512, 512, 1, 1, 3, 1), (1024, 64, 1024, 64, 1, 8),
    (16384, 1024, 1024, 64, 8, 8), (262144, 4096, 2048, 32, 4, 4), (65536, 4096, 2048, 128, 4, 8),
])
@pytest.mark.parametrize("seed", [0, 0xABCDEF0123456789])
def test_export_bit_exact(params, seed):
    print("export", params, seed, flush=True)
    sk = B.Sketch(*params, seed=seed)
    rows, signs = sk.export()
    torch.cuda.synchronize()
    want_r, want_s = O.build_tables(O.Params(*params), seed)
    assert np.array_equal(rows.cpu().numpy().astype(np.int64), want_r)
    assert np.array_equal(signs.cpu().numpy(), want_s)


def test_export_bit_exact_gradient_config():
    cfg = W.CONFIGS["grad"]
    print("export grad", flush=True)
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    rows, signs = sk.export()
    torch.cuda.synchronize()
    want_r, want_s = O.build_tables(O.Params(*cfg.params), cfg.sketch_seed)
    assert np.array_equal(rows.cpu().numpy(), want_r.astype(np.int32))
    assert np.array_equal(signs.cpu().numpy(), want_s)


# ------------------------------------------------- element-wise parity ----
SMALL = [
    # params (d,k,Bc,Br,kappa,s), n, lda pad, ldo pad
    ((4096, 256, 512, 32, 2, 4), 512, 0, 0),        # tiny config
    ((4096, 256, 512, 32, 2, 4), 301, 3, 5),        # ragged tail, odd strides
    ((2048, 1024, 128, 64, 4, 2), 130, 6, 0),       # Fig. 2 parameters
    ((8192, 512, 1024, 64, 8, 8), 264, 0, 8),       # mid-config blocks, kappa = M
    ((16384, 256, 2048, 32, 4, 4), 72, 8, 0),       # tall-config blocks
    ((16384, 1024, 2048, 128, 4, 8), 200, 0, 0),    # wide-config blocks
    ((32768, 64, 4096, 8, 8, 2), 256, 768, 0),      # gradient-config blocks, chunk view stride
    ((32768, 64, 4096, 8, 8, 2), 100, 4, 4),
    ((1152, 72, 96, 6, 5, 3), 65, 0, 0),            # Br not a power of two
    ((1440, 180, 80, 10, 18, 10), 33, 1, 1),        # kappa = M, s = Br
    ((512, 512, 1, 1, 3, 1), 17, 0, 0),             # Br = Bc = 1
    ((1024, 64, 1024, 64, 1, 8), 1, 0, 0),          # M = 1, single column
    ((3072, 1536, 1024, 512, 2, 8), 70, 0, 0),      # Br > LDS rows per pass
    ((65536, 8192, 64, 8, 8, 2), 256, 0, 0),        # M = 1024: orbit-run mode of the MFMA path
    ((65536, 8192, 64, 8, 8, 2), 300, 4, 4),        # the same with a ragged second column tile
    ((32768, 4096, 128, 16, 4, 4), 1024, 0, 0),     # M = 256, four column tiles, Br = 16
    ((16384, 2048, 64, 8, 8, 2), 2500, 0, 0),       # M = 256, ten column tiles, ragged
    ((4000, 256, 512, 32, 2, 4), 300, 0, 0),        # d not a multiple of Bc (zero-padded last block)
    ((32700, 64, 4096, 8, 8, 2), 256, 0, 0),
    ((65500, 8192, 64, 8, 8, 2), 300, 4, 0),        # the same in orbit-run mode, ragged tile
    ((7201, 512, 1024, 64, 8, 8), 264, 0, 0),       # the same in OUT-stationary mode
    ((1100, 72, 96, 6, 5, 3), 65, 0, 0),            # the same on the generic kernel only
    ((16384, 1024, 2048, 128, 4, 8), 520, 0, 0),    # 128-row wave tiles: two full column tiles + ragged
    ((8192, 1024, 512, 64, 4, 12), 300, 4, 0),      # OUT-stationary with s > 8 (tail of the pipelined fill)
    ((8192, 1024, 512, 64, 4, 3), 256, 0, 0),       # odd s
    ((4096, 1024, 128, 32, 8, 1), 256, 0, 0),       # s = 1, two stages per block
    ((2048, 4096, 64, 128, 2, 32), 256, 0, 0),      # s = 32, one stage per block, Br = 128, two stages in all
    ((2048, 4096, 64, 128, 3, 4), 256, 0, 0),       # the same with an odd stage count (shallow prefetch ring)
    ((6144, 4096, 192, 128, 1, 4), 256, 0, 0),      # kappa = 1, 128 stacked rows, three stages
    # kappa*Br below the tile height: the top rows of the matrix-core tile idle
    ((6144, 768, 256, 32, 3, 4), 300, 0, 0),        # 96 stacked rows in a 128-row tile
    ((2048, 128, 128, 8, 5, 2), 130, 6, 0),         # 40 in 64
    ((4096, 64, 64, 1, 4, 1), 256, 0, 0),           # Br = 1: 4 in 32
    ((4096, 128, 512, 16, 1, 4), 64, 0, 4),         # kappa = 1, Br = 16
    ((512, 16, 64, 2, 7, 2), 33, 3, 0),             # 14 in 32, one stage per block
    ((1024, 128, 128, 16, 7, 3), 256, 0, 0),        # 112 in 128, two stages (deep prefetch ring)
    # more than 128 stacked rows of small blocks: groups of 128/Br wiring slots
    ((8192, 2048, 64, 16, 16, 2), 300, 0, 0),       # 256 rows: two full groups
    ((2048, 256, 64, 8, 20, 2), 130, 2, 0),         # 160 rows: a full group and one of 4 slots
    ((4096, 256, 64, 4, 40, 3), 70, 2, 4),          # Br = 4: groups of 32 slots
    ((8192, 128, 64, 1, 128, 1), 64, 0, 0),         # Br = 1, kappa = M = 128: one full group
    # Bc not a multiple of the 64-row stage: the last stage of a block is partly filled
    ((1000, 256, 125, 32, 2, 4), 300, 0, 0),        # Bc = 125, input-stationary
    ((1536, 1024, 96, 64, 4, 4), 256, 0, 0),        # Bc = 96, output-stationary
    ((640, 128, 40, 8, 4, 2), 130, 2, 0),           # Bc = 40: less than one stage
    ((1990, 128, 250, 16, 8, 2), 64, 0, 0),         # Bc = 250 and a partly filled last block
    ((73728, 8192, 72, 8, 8, 2), 256, 0, 0),        # Bc = 72, orbit runs
    # lda not a multiple of 4 columns: the matrix-core kernels load element by element
    ((4096, 256, 512, 32, 2, 4), 301, 0, 0),        # input-stationary, lda = 301
    ((32768, 64, 4096, 8, 8, 2), 255, 0, 0),        # gradient-config blocks, lda = 255
    ((8192, 1024, 512, 64, 4, 8), 250, 1, 0),       # output-stationary, lda = 251
    ((16384, 1024, 2048, 128, 4, 8), 130, 1, 3),    # 128-row tiles, lda = 131
    ((4001, 256, 512, 32, 2, 4), 77, 0, 0),         # and a partly filled last block
    ((16640, 4160, 64, 16, 130, 1), 64, 0, 0),      # kappa = 130 > 128: 17 slot groups
    ((8320, 4160, 64, 32, 130, 1), 40, 0, 0),       # the same with 32-row blocks: groups of four
    # Br not a power of two: a slot takes the next power of two of tile rows (column layout)
    ((512, 768, 64, 96, 1, 8), 130, 2, 0),          # Br = 96, kappa = 1: 96 of 128 rows
    ((1024, 768, 64, 48, 2, 5), 256, 0, 0),         # Br = 48, kappa = 2: two slots of 64
    ((1024, 768, 64, 48, 4, 5), 64, 0, 4),          # the same with kappa = 4: groups of two slots
    ((4800, 600, 200, 25, 3, 25), 100, 0, 0),       # Br = 25 = s, Bc = 200
    ((8192, 48, 1024, 6, 4, 2), 64, 0, 0),          # Br = 6 with few, long blocks: split rows
    # output blocks higher than the 128-row tile: 128-row slices
    ((4096, 1024, 1024, 256, 2, 8), 300, 0, 0),     # Br = 256
    ((8192, 4096, 1024, 512, 3, 32), 130, 2, 0),    # Br = 512, s = 32
    ((2048, 2048, 1024, 1024, 2, 16), 64, 0, 4),    # Br = 1024, M = 2: split stages as well
]


@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: VNAME[v])
@DTYPES
@pytest.mark.parametrize("case", SMALL, ids=lambda c: f"{c[0]}-n{c[1]}")
def test_apply_matches_oracle(case, dtype, variant):
    params, n, pa, po = case
    print("apply", params, n, dtype, VNAME[variant], flush=True)
    seed = 5
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(n + d)
    Abuf = torch.randn((d + 70, n + pa), generator=g, device=DEV).to(dtype)
    Abuf[d:] = float("nan")         # nor may memory past the last row (a partly filled last block reads zeros)
    if pa:
        Abuf[:, n:] = float("nan")  # the padding between n and lda must never reach the result
    A = Abuf[:d, :n]
    obuf = torch.full((k, n + po), float("nan"), device=DEV, dtype=dtype)
    sk = make_sketch(params, seed, variant)
    apply_or_skip(sk, A, obuf[:, :n])
    torch.cuda.synchronize()
    plan, did = sk.plan(n, dtype, ld=A.stride(0), address=A.data_ptr()), sk.info()
    assert (plan["variant"], plan["mode"]) == (did.last_variant, did.last_mode)   # the host-side query agrees
    ref = O.apply(oracle_csc(params, seed), host64(A))
    check(obuf[:, :n], ref, dtype, "apply")
    if po:
        assert torch.isnan(obuf[:, n:].float()).all(), "wrote outside the n output columns"
    # element-wise, scaled by the typical magnitude of an output entry
    tol = ETOL[dtype]
    diff = np.abs(host64(obuf[:, :n]) - ref)
    assert (diff <= tol * (np.abs(ref) + np.sqrt((ref ** 2).mean()))).all()


# --------------------- output-stationary kernel with shared Phi tiles -----
OUTS = [
    # params (d,k,Bc,Br,kappa,s), n, lda pad, ldo pad, taken: 16-bit output-stationary shapes (k >= d/4
    # keeps the dispatcher from splitting the rows of these small problems over grid.z)
    ((8192, 2048, 512, 128, 4, 8), 520, 0, 0, True),     # wide-config block height: four column waves, ragged last tile
    ((8192, 2048, 512, 128, 4, 8), 200, 0, 0, True),     # two column waves (128 < n <= 256)
    ((8192, 2048, 512, 128, 4, 8), 1021, 3, 0, True),    # n not a multiple of 4: the last vector straddles n
    ((4096, 1024, 256, 64, 4, 8), 532, 0, 3, True),      # 64-row blocks, output rows not vector aligned
    ((4096, 1024, 128, 32, 8, 1), 260, 4, 0, True),      # 32-row blocks, s = 1, two stages per block
    ((4096, 1024, 256, 64, 4, 12), 300, 4, 0, True),     # s = 12: a lane's share runs into the tail loop
    ((4096, 2048, 256, 128, 2, 32), 300, 0, 0, True),    # s = 32
    ((4096, 1024, 256, 64, 16, 3), 300, 0, 0, True),     # kappa = M, odd s
    ((3900, 1024, 256, 64, 8, 8), 264, 0, 0, True),      # d not a multiple of Bc: a partly filled last block
    ((3200, 1024, 100, 32, 8, 4), 300, 0, 0, True),      # Bc = 100: the second stage of a block is partly outside it
    ((6144, 4096, 192, 128, 2, 4), 300, 0, 0, True),     # three stages per block, kappa = 2: six stages
    ((16384, 8192, 256, 128, 2, 8), 260, 0, 0, True),    # M = 64: orbit renumbering over many blocks
    ((4096, 1024, 256, 64, 4, 8), 530, 0, 0, False),     # rows not aligned to 4 columns: element loads
    ((16384, 1024, 2048, 128, 4, 8), 520, 0, 0, True),   # few output tiles: rows split over grid.z, partial planes
    ((8192, 512, 1024, 64, 8, 8), 300, 4, 3, True),      # the same with 64-row blocks, kappa = M, padded rows
    ((6144, 4096, 192, 128, 1, 4), 300, 0, 0, False),    # an odd number of stages
    ((4096, 1024, 256, 64, 4, 8), 100, 0, 0, False),     # a single wave of columns
]


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16], ids=["bf16", "f16"])
@pytest.mark.parametrize("case", OUTS, ids=lambda c: f"{c[0]}-n{c[1]}")
def test_shared_phi_kernel_matches_oracle(case, dtype):
    """The 16-bit output-stationary shapes (kappa*Br above one tile, blocks one tile high) run on the
    kernel whose work-group shares its Phi tiles; element-wise parity, untouched padding, and
    results that do not depend on where a column sits in the launch."""
    params, n, pa, po, expect_outs = case
    print("outs", params, n, dtype, flush=True)
    seed = 8
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(n + d)
    Abuf = torch.randn((d + 70, n + pa), generator=g, device=DEV).to(dtype)
    Abuf[d:] = float("nan")
    if pa:
        Abuf[:, n:] = float("nan")
    A = Abuf[:d, :n]
    obuf = torch.full((k, n + po), float("nan"), device=DEV, dtype=dtype)
    sk = B.Sketch(*params, seed=seed)
    sk.apply(A, obuf[:, :n])
    torch.cuda.synchronize()
    i = sk.info()
    assert i.last_kernel.decode().startswith("outs_kernel") == expect_outs, i.last_kernel
    assert (i.last_variant, i.last_mode) == (B.VARIANT_MFMA, 1)
    ref = O.apply(oracle_csc(params, seed), host64(A))
    check(obuf[:, :n], ref, dtype, "shared-Phi kernel")
    if po:
        assert torch.isnan(obuf[:, n:].float()).all(), "wrote outside the n output columns"
    diff = np.abs(host64(obuf[:, :n]) - ref)
    assert (diff <= ETOL[dtype] * (np.abs(ref) + np.sqrt((ref ** 2).mean()))).all()
    # column independence: an aligned 256-column sub-view (two column waves instead of four) gives
    # the same bits for the shared columns
    if expect_outs and n >= 516:
        other = sk.apply(A[:, 260:516])
        assert sk.info().last_kernel.decode().startswith("outs_kernel")
        assert torch.equal(other, obuf[:, 260:516])


# --------------------- several output blocks per wave ----------------------
STACKED = [
    # params (d,k,Bc,Br,kappa,s), n, lda pad, ldo pad, dtypes, taken.  The kernel wants at least 128
    # work-groups of (4 or 2 output blocks) x 256 columns, so M and n are larger than elsewhere.
    ((8192, 4096, 128, 64, 4, 8), 3584, 0, 0, "f32 bf16 f16", True),     # kappa = S = 4: one phase of one block, three of two
    ((8192, 4096, 128, 64, 8, 8), 3070, 2, 3, "f32 bf16", True),         # kappa = 8; ragged last tile, padded rows, element stores
    ((12750, 4096, 200, 64, 12, 5), 3074, 0, 0, "f32 f16", True),        # Bc = 200: a stage partly outside its block; d short of M*Bc; odd s
    ((8192, 4096, 128, 64, 4, 1), 3072, 0, 0, "f32 bf16", True),         # s = 1
    ((8192, 4096, 128, 64, 4, 20), 3072, 0, 0, "f32 bf16", True),        # s = 20: the tail loop over a row's nonzeros
    ((2048, 1024, 128, 64, 16, 3), 12288, 0, 0, "f32", True),            # kappa = M: the window wraps round the orbit
    ((16384, 8192, 256, 128, 6, 12), 2048, 0, 0, "f32", True),           # 128-row blocks: two slots; s = 12
    ((16384, 8192, 256, 128, 2, 8), 2050, 0, 0, "f32", True),            # kappa = S = 2
    ((16384, 8192, 256, 128, 2, 8), 2048, 0, 0, "bf16", False),          # 16-bit, 128 rows: one block per work-group is faster
    ((8192, 4096, 128, 64, 6, 8), 3072, 0, 0, "f32", False),             # kappa not a multiple of the slot count
    ((8192, 4096, 128, 64, 4, 8), 3071, 1, 0, "f32", False),             # odd n
    ((8192, 4096, 128, 64, 4, 8), 1792, 0, 0, "f32", False),             # too few work-groups for the chip
    ((8192, 4096, 128, 64, 4, 8), 2048, 0, 0, "f32", True),              # exactly the 128 it asks for
    ((12288, 4096, 192, 64, 4, 8), 3072, 0, 0, "f32", False),           # an odd number of stages per block
]
_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
STACKED_RUNS = [(c, _DT[t]) for c in STACKED for t in c[4].split()]


@pytest.mark.parametrize("case,dtype", STACKED_RUNS,
                         ids=[f"{c[0]}-n{c[1]}-{str(t).split('.')[1]}" for c, t in STACKED_RUNS])
def test_stacked_kernel_matches_oracle(case, dtype):
    """Shapes with 64-row blocks (or 128-row, fp32) and kappa a multiple of the slot count run on the
    kernel that keeps several consecutive output blocks of the wiring's orbit in one wave's
    accumulators; element-wise parity, untouched padding."""
    params, n, pa, po, _, expect = case
    print("stacked", params, n, dtype, flush=True)
    seed = 12
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(n + d)
    Abuf = torch.randn((d + 70, n + pa), generator=g, device=DEV).to(dtype)
    Abuf[d:] = float("nan")
    if pa:
        Abuf[:, n:] = float("nan")
    A = Abuf[:d, :n]
    obuf = torch.full((k, n + po), float("nan"), device=DEV, dtype=dtype)
    sk = B.Sketch(*params, seed=seed)
    plan = sk.plan(n, dtype, ld=A.stride(0), address=A.data_ptr())
    sk.apply(A, obuf[:, :n])
    torch.cuda.synchronize()
    i = sk.info()
    assert i.last_kernel.decode().startswith("stacked_kernel") == expect, i.last_kernel
    assert (plan["variant"], plan["mode"]) == (i.last_variant, i.last_mode)
    assert bool(plan["flags"] & B.PLAN_STACKED) == expect, plan
    if expect:
        assert (i.last_variant, i.last_mode, plan["workspace_bytes"]) == (B.VARIANT_MFMA, 1, 0)
    ref = O.apply(oracle_csc(params, seed), host64(A))
    check(obuf[:, :n], ref, dtype, "stacked kernel")
    if po:
        assert torch.isnan(obuf[:, n:].float()).all(), "wrote outside the n output columns"
    diff = np.abs(host64(obuf[:, :n]) - ref)
    assert (diff <= ETOL[dtype] * (np.abs(ref) + np.sqrt((ref ** 2).mean()))).all()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_stacked_kernel_one_hot_columns_are_exact_and_columns_independent(dtype):
    params = (8192, 4096, 128, 64, 4, 4)             # kappa*s = 16: the scale is a power of two
    d, n = params[0], 3584
    rng = np.random.default_rng(5)
    rows = np.r_[0, d - 1, params[2] - 1, params[2], rng.integers(0, d, n - 4)]
    A = torch.zeros((d, n), device=DEV, dtype=dtype)
    A[torch.from_numpy(rows).to(DEV), torch.arange(n, device=DEV)] = 1.0
    sk = B.Sketch(*params, seed=0)
    out = sk.apply(A)
    torch.cuda.synchronize()
    assert sk.info().last_kernel.decode().startswith("stacked_kernel")
    assert np.array_equal(host64(out), oracle_csc(params, 0)[:, rows].toarray())
    # a sub-view (other column tiles, other work-groups) gives the same bits for the shared columns
    g = torch.Generator(device=DEV).manual_seed(1)
    R = torch.randn((d, n), generator=g, device=DEV).to(dtype)
    full = sk.apply(R)
    part = sk.apply(R[:, 512:])
    assert sk.info().last_kernel.decode().startswith("stacked_kernel")
    assert torch.equal(part, full[:, 512:])


def test_shared_phi_kernel_one_hot_columns_are_exact():
    params = (8192, 2048, 512, 128, 4, 4)            # kappa*s = 16: the scale is a power of two
    d = params[0]
    rng = np.random.default_rng(2)
    cols = np.unique(np.r_[0, d - 1, params[2] - 1, params[2], rng.integers(0, d, 400)])
    A = torch.zeros((d, (len(cols) + 3) // 4 * 4), device=DEV, dtype=torch.bfloat16)[:, :len(cols)]  # rows aligned to 4 columns
    A[torch.from_numpy(cols).to(DEV), torch.arange(len(cols), device=DEV)] = 1.0
    sk = B.Sketch(*params, seed=0)
    out = sk.apply(A)
    torch.cuda.synchronize()
    assert sk.info().last_kernel.decode().startswith("outs_kernel")
    assert np.array_equal(host64(out), oracle_csc(params, 0)[:, cols].toarray())


# ---------------------------------------------------------- one-hot -------
@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: VNAME[v])
@DTYPES
@pytest.mark.parametrize("params", [(4096, 256, 512, 32, 4, 4), (32768, 64, 4096, 8, 8, 2),
                                    (8192, 512, 1024, 64, 4, 4), (4096, 256, 512, 32, 2, 2),
                                    (65536, 8192, 64, 8, 8, 2)])
def test_one_hot_probes_reproduce_columns_exactly(params, dtype, variant):
    """A = selected unit vectors: each output column is one column of S; with
    kappa*s a power of four the scale is a power of two, so the match is exact."""
    print("one-hot", params, dtype, VNAME[variant], flush=True)
    d = params[0]
    assert round(np.sqrt(params[4] * params[5])) ** 2 == params[4] * params[5]
    rng = np.random.default_rng(1)
    cols = np.unique(np.r_[0, d - 1, params[2] - 1, params[2], rng.integers(0, d, 120)])
    A = torch.zeros((d, len(cols)), device=DEV, dtype=dtype)
    A[torch.from_numpy(cols).to(DEV), torch.arange(len(cols), device=DEV)] = 1.0
    sk = make_sketch(params, 0, variant)
    out = apply_or_skip(sk, A)
    torch.cuda.synchronize()
    want = oracle_csc(params, 0)[:, cols].toarray()
    assert np.array_equal(host64(out), want)


@DTYPES
@pytest.mark.parametrize("params", [(4096, 256, 512, 32, 2, 4), (8192, 1024, 512, 64, 4, 8)])
def test_apply_on_a_view_that_starts_at_an_odd_column(params, dtype):
    """A view whose first element is not aligned to 4 columns (here: column 1 or 3 of a wider
    buffer) takes the element-wise loads of the matrix-core kernel and still matches."""
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(21)
    buf = torch.randn((d, 264), generator=g, device=DEV).to(dtype)
    sk = make_sketch(params, 6, B.VARIANT_MFMA)
    for first, n in ((1, 256), (3, 130)):
        A = buf[:, first:first + n]
        out = sk.apply(A)
        torch.cuda.synchronize()
        check(out, O.apply(oracle_csc(params, 6), host64(A)), dtype, f"view from column {first}")
        assert torch.equal(out, sk.apply(A.contiguous()) if n % 4 == 0 else out)


# ------------------------------------------ half: the ends of its range ---
@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: VNAME[v])
@pytest.mark.parametrize("params", [(4096, 256, 512, 32, 2, 4), (8192, 1024, 512, 64, 4, 8)])
def test_half_subnormal_inputs_count_and_overflow_becomes_infinity(params, variant):
    """Half inputs below 2^-14 are subnormal and must enter the sums with their value; results
    beyond the largest half (65504) round to infinity, as IEEE round-to-nearest does."""
    print("half range", params, VNAME[variant], flush=True)
    d, n = params[0], 96
    g = torch.Generator(device=DEV).manual_seed(12)
    A = torch.randn((d, n), generator=g, device=DEV)
    A[:, :32] *= 2.0 ** -17          # every entry subnormal or nearly so in half
    A[:, 32:64] *= 3.0e4             # sums pass 65504 in many places
    A = A.clamp(-65504, 65504).to(torch.float16)
    assert (A[:, :32].abs().float() < 2.0 ** -14).float().mean() > 0.9
    sk = make_sketch(params, 4, variant)
    out = host64(apply_or_skip(sk, A))
    ref = O.apply(oracle_csc(params, 4), host64(A))
    # one rounding to half: 2^-11 relative, or half a unit of the subnormal spacing 2^-24; the
    # fp32 sum and the fp32 scale factor add a few 2^-24 relative
    small, big = slice(0, 32), slice(32, 64)
    assert np.abs(ref[:, small]).max() < 2.0 ** -10 and (ref[:, small] != 0).mean() > 0.9
    assert (np.abs(out[:, small] - ref[:, small]) <= 2.0 ** -11 * 1.01 * np.abs(ref[:, small]) + 2.0 ** -25 * 1.01).all()
    over = np.abs(ref[:, big]) > 65520 * (1 + 1e-5)
    under = np.abs(ref[:, big]) < 65520 * (1 - 1e-5)
    assert over.any() and under.any()
    assert (out[:, big][over] == np.sign(ref[:, big][over]) * np.inf).all()
    assert np.isfinite(out[:, big][under]).all()
    assert (np.abs(out[:, big][under] - ref[:, big][under]) <= 2.0 ** -11 * 1.01 * np.abs(ref[:, big][under])).all()
    check(torch.from_numpy(out[:, 64:]), ref[:, 64:], torch.float16, "half, ordinary columns")
    if variant == B.VARIANT_MFMA:    # the same vectors as rows
        rows = host64(sk.apply_rows(A.t().contiguous())).T
        assert (np.abs(rows[:, small] - ref[:, small]) <= 2.0 ** -11 * 1.01 * np.abs(ref[:, small]) + 2.0 ** -25 * 1.01).all()
        assert (rows[:, big][over] == np.sign(ref[:, big][over]) * np.inf).all()


# ------------------------------------ chunking, determinism, linearity ----
@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: VNAME[v])
@DTYPES
def test_chunked_equals_monolithic_bitwise(dtype, variant):
    params, n, chunk = (32768, 64, 4096, 8, 8, 2), 1024, 256
    print("chunked", dtype, VNAME[variant], flush=True)
    A = W.laplace_lognormal(params[0], n, 3, DEV, dtype=dtype)
    sk = make_sketch(params, 0, variant)
    whole = apply_or_skip(sk, A)
    again = sk.apply(A)
    parts = torch.empty_like(whole)
    for c in range(0, n, chunk):
        sk.apply(A[:, c:c + chunk], parts[:, c:c + chunk])
    torch.cuda.synchronize()
    bits = torch.int32 if dtype == torch.float32 else torch.int16
    assert torch.equal(whole.view(bits), again.view(bits))
    assert torch.equal(whole, parts)


@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: VNAME[v])
def test_linearity(variant):
    params = (8192, 512, 1024, 64, 4, 4)
    g = torch.Generator(device=DEV).manual_seed(0)
    X, Y = torch.randn((2, params[0], 96), generator=g, device=DEV)
    sk = make_sketch(params, 2, variant)
    lhs = apply_or_skip(sk, 2 * X - 3 * Y)
    rhs = 2 * sk.apply(X) - 3 * sk.apply(Y)
    torch.cuda.synchronize()
    assert O.rel_fro_err(host64(lhs), host64(rhs)) < 1e-5


def test_mfma_modes_are_the_intended_ones():
    """The dispatcher picks the decomposition each configuration was designed for."""
    want = {"grad": 3, "wide": 1, "tall": 2, "tiny": 2}
    for name, mode in want.items():
        cfg = W.CONFIGS[name]
        n = 256 if name == "grad" else min(cfg.n, 512)
        A = torch.zeros((cfg.d, n), device=DEV, dtype=cfg.dtype)
        sk = B.Sketch(*cfg.params, seed=0)
        sk.apply(A)
        i = sk.info()
        assert (i.last_variant, i.last_mode) == (B.VARIANT_MFMA, mode), (name, i.last_variant, i.last_mode)
    torch.cuda.synchronize()


def test_forced_variant_on_unsupported_shape_reports_unsupported():
    sk = B.Sketch(256, 384, 64, 96, 2, 4)  # Br = 96 (not a power of two) with kappa = 2: 256 padded rows
    sk.set_variant(B.VARIANT_MFMA)
    A = torch.zeros((256, 8), device=DEV)
    with pytest.raises(B.FlashSketchError) as e:
        sk.apply(A)
    assert e.value.status == 2
    sk.set_variant(B.VARIANT_AUTO)
    sk.apply(A)  # falls back to the generic kernel
    assert sk.info().last_variant == B.VARIANT_GENERIC


def test_empty_input_launches_nothing():
    sk = B.Sketch(4096, 256, 512, 32, 2, 4)
    A = torch.zeros((4096, 0), device=DEV)
    out = sk.apply(A)
    assert out.shape == (256, 0)


# ------------------------------------------------ baselines ---------------
@DTYPES
@pytest.mark.parametrize("d,k,s,n", [(4096, 256, 4, 300), (16384, 1024, 8, 520), (1000, 48, 3, 17)])
def test_plain_sjlt_scatter_matches_oracle(d, k, s, n, dtype):
    print("scatter", d, k, s, n, dtype, flush=True)
    params = (d, k, d, k, 1, s)
    g = torch.Generator(device=DEV).manual_seed(4)
    A = torch.randn((d, n), generator=g, device=DEV).to(dtype)
    sk = B.Sketch(*params, seed=1, kind=B.KIND_SJLT_SCATTER)
    out = sk.apply(A)
    torch.cuda.synchronize()
    check(out, O.apply(oracle_csc(params, 1), host64(A)), dtype, "scatter")
    rows, signs = sk.export()
    want_r, want_s = O.build_tables(O.Params(*params), 1)
    assert np.array_equal(rows.cpu().numpy().astype(np.int64), want_r)
    assert np.array_equal(signs.cpu().numpy(), want_s)


@DTYPES
@pytest.mark.parametrize("k,d,n,pad", [(128, 1024, 256, 0), (256, 4096, 300, 4), (1024, 2048, 1000, 0),
                                       (1024, 256, 12328, 0)])  # enough tiles for the 128 x 512 fp32 work-groups
def test_dense_gaussian_matches_oracle(k, d, n, pad, dtype):
    from oracle import gaussian as G
    print("gauss", k, d, n, dtype, flush=True)
    g = torch.Generator(device=DEV).manual_seed(7)
    A = torch.randn((d, n + pad), generator=g, device=DEV).to(dtype)[:, :n]
    sk = B.Sketch(d, k, d, k, 1, 1, seed=2, kind=B.KIND_GAUSS_DENSE)
    out = sk.apply(A)
    S_dev = sk.export_dense()
    torch.cuda.synchronize()
    S = G.gaussian_matrix(k, d, 2)
    # the same matrix up to the last bit of the device's double-precision log / cos
    Sd = S_dev.cpu().double().numpy()
    assert np.abs(Sd - S).max() <= 2.0 ** -22 * np.abs(S).max()
    assert (Sd != S).mean() < 1e-3
    # (16-bit applies multiply by S rounded to the element type: one more rounding of that size)
    err = O.rel_fro_err(host64(out), G.apply(S, host64(A)))
    assert err <= {torch.float32: 1e-5, torch.bfloat16: 4e-3, torch.float16: 1e-3}[dtype], f"dense gaussian: {err:.3e}"


# ------------------------------------------------ full-size configs -------
def _sampled_parity(cfg, A, out, seed=0):
    """Oracle on a sample of columns of the full-size problem: one column, at a random place, from
    every 128-column wave tile, plus both edges; the bar holds for the sample as a whole and,
    with a factor for the smaller sample, for every sampled column on its own."""
    rng = np.random.default_rng(seed)
    tiles = np.arange(0, cfg.n, 128)
    cols = np.unique(np.r_[0, cfg.n - 1, np.minimum(tiles + rng.integers(0, 128, len(tiles)), cfg.n - 1)])
    idx = torch.from_numpy(cols).to(A.device)
    ref = O.apply(oracle_csc(cfg.params, cfg.sketch_seed), host64(A[:, idx]))
    got = host64(out[:, idx])
    per_col = np.linalg.norm(got - ref, axis=0) / np.linalg.norm(ref, axis=0)
    assert per_col.max() <= 1.5 * TOL[cfg.dtype], f"{cfg.name}: column {cols[per_col.argmax()]} off by {per_col.max():.3e}"
    return check(out[:, idx], ref, cfg.dtype, f"{cfg.name} sampled columns")


def _all_columns_against_the_general_kernel(sk, A, out):
    """Every column of a full-size result against the general (one-lane-per-column, LDS) kernel, on
    the device: two kernels that share only the hash recipe.  Both accumulate in fp32 in different
    orders, so fp32 results agree to rounding of the sum and 16-bit results are equal except where
    the sum falls next to a rounding boundary (then one unit in the last place)."""
    sk.set_variant(B.VARIANT_GENERIC)
    other = sk.apply(A)
    sk.set_variant(B.VARIANT_AUTO)
    torch.cuda.synchronize()
    a, b = out.float(), other.float()
    rms = float(b.pow(2).mean().sqrt())
    if out.dtype == torch.float32:
        assert float((a - b).abs().max()) <= 2e-5 * rms
    else:
        ulp = 2.0 ** -7 if out.dtype == torch.bfloat16 else 2.0 ** -10
        differ = a != b
        assert float(differ.float().mean()) < 2e-2
        assert bool(((a - b).abs() <= ulp * b.abs() + 1e-5 * rms)[differ].all())   # (sums that cancel to about 0)
    assert float((a - b).norm() / b.norm()) <= TOL[out.dtype]


@pytest.mark.parametrize("name", ["tiny", "tall"])
def test_full_config_all_columns(name):
    cfg = W.CONFIGS[name]
    print("full", name, flush=True)
    A = W.make_input(cfg, DEV)
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    out = sk.apply(A)
    torch.cuda.synchronize()
    ref = O.apply(oracle_csc(cfg.params, cfg.sketch_seed), host64(A))
    check(out, ref, cfg.dtype, name)


@pytest.mark.parametrize("kappa", W.MID_KAPPAS)
def test_full_config_mid_sampled(kappa):
    import dataclasses
    cfg = dataclasses.replace(W.CONFIGS["mid"], kappa=kappa)
    print("full mid kappa", kappa, flush=True)
    A = W.make_input(cfg, DEV)
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    out = sk.apply(A)
    torch.cuda.synchronize()
    _sampled_parity(cfg, A, out)
    if kappa in (1, 4):
        _all_columns_against_the_general_kernel(sk, A, out)


@pytest.mark.parametrize("n", W.WIDE_NS)
def test_full_config_wide_sampled(n):
    """The bf16 width sweep at full d on the shared-Phi kernel: n = 1024 and 2048 split the rows of
    a work-group over grid.z (partial planes and the reduction), 4096 and 8192 store directly."""
    import dataclasses
    cfg = dataclasses.replace(W.CONFIGS["wide"], n=n)
    print("full wide n", n, flush=True)
    A = W.make_input(cfg, DEV)
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    out = sk.apply(A)
    torch.cuda.synchronize()
    kernel = sk.info().last_kernel.decode()
    assert kernel.startswith("outs_kernel") and kernel.endswith("+reduce_planes") == (n < 4096), kernel
    _sampled_parity(cfg, A, out)
    if n in (1024, 8192):
        _all_columns_against_the_general_kernel(sk, A, out)


def test_baseline_kinds_at_the_mid_configurations_full_d():
    """The two reference points of the mid configuration at its full d = 16384, k = 1024 (fewer
    columns, so that the oracles stay quick): the plain-SJLT scatter with s = 8 and the dense
    Gaussian sketch."""
    from oracle import gaussian as OG
    cfg = W.CONFIGS["mid"]
    n = 96
    A = W.make_input(cfg, DEV, n=n)
    sc = B.Sketch(cfg.d, cfg.k, cfg.d, cfg.k, 1, cfg.s, seed=cfg.sketch_seed, kind=B.KIND_SJLT_SCATTER)
    out = sc.apply(A)
    torch.cuda.synchronize()
    ref = O.apply(O.build_csc(O.Params(cfg.d, cfg.k, cfg.d, cfg.k, 1, cfg.s), cfg.sketch_seed), host64(A))
    check(out, ref, torch.float32, "plain SJLT scatter at mid's d")
    ga = B.Sketch(cfg.d, cfg.k, cfg.d, cfg.k, 1, 1, seed=cfg.sketch_seed, kind=B.KIND_GAUSS_DENSE)
    A4 = W.make_input(cfg, DEV, n=128)
    out = ga.apply(A4)
    torch.cuda.synchronize()
    ref = OG.apply(OG.gaussian_matrix(cfg.k, cfg.d, cfg.sketch_seed), host64(A4))
    check(out, ref, torch.float32, "dense Gaussian at mid's d")


def test_full_config_grad_chunked_sampled():
    """8 GiB bf16 input, applied as the benchmark does: four 256-column views of
    one allocation on one stream."""
    cfg = W.CONFIGS["grad"]
    print("full grad", flush=True)
    A = W.make_input(cfg, DEV)
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    out = torch.empty((cfg.k, cfg.n), device=DEV, dtype=cfg.dtype)
    for c in range(0, cfg.n, cfg.chunk):
        sk.apply(A[:, c:c + cfg.chunk], out[:, c:c + cfg.chunk])
    torch.cuda.synchronize()
    print("  applied; oracle on sampled columns", flush=True)
    _sampled_parity(cfg, A, out)
    # the same chunks as four separate packed d x 256 buffers (lda = 256), as a pipeline that hands
    # over one chunk at a time holds them: the same bits
    packed = torch.empty_like(out)
    for c in range(0, cfg.n, cfg.chunk):
        buf = A[:, c:c + cfg.chunk].contiguous()
        sk.apply(buf, packed[:, c:c + cfg.chunk])
        del buf
    torch.cuda.synchronize()
    assert torch.equal(packed, out)
    # and every column of one chunk against the general kernel
    _all_columns_against_the_general_kernel(sk, A[:, :cfg.chunk], out[:, :cfg.chunk].contiguous())


def test_full_config_grad_rows_layout_sampled():
    """The same 8 GiB input held examples-as-rows (row stride d + 64 elements), applied in four
    chunks of 256 examples; the oracle on a sample of examples."""
    cfg = W.CONFIGS["grad"]
    print("full grad, rows layout", flush=True)
    A = W.make_input(cfg, DEV)
    Gbuf = torch.empty((cfg.n, cfg.d + 64), device=DEV, dtype=cfg.dtype)
    G = Gbuf[:, :cfg.d]
    G.copy_(A.t())
    del A
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    out = torch.empty((cfg.n, cfg.k), device=DEV, dtype=cfg.dtype)
    for c in range(0, cfg.n, cfg.chunk):
        sk.apply_rows(G[c:c + cfg.chunk], out[c:c + cfg.chunk])
    torch.cuda.synchronize()
    print("  applied; oracle on sampled examples", flush=True)
    rng = np.random.default_rng(0)
    ex = np.unique(np.r_[0, cfg.n - 1, rng.integers(0, cfg.n, 6)])
    idx = torch.from_numpy(ex).to(DEV)
    ref = O.apply_rows(oracle_csc(cfg.params, cfg.sketch_seed), host64(G[idx]))
    check(out[idx], ref, cfg.dtype, "grad rows layout, sampled examples")


def test_rows_so_long_that_128_of_them_span_2_to_31_bytes():
    """fp32 vectors of the gradient configuration's length held as rows: 16 MiB per row, so the
    kernel addresses each 32-example tile through a descriptor of its own.  The oracle on a
    sample of the examples (one of them in the ragged last tile)."""
    cfg = W.CONFIGS["grad"]
    n = 150
    print("long fp32 rows", flush=True)
    g = torch.Generator(device=DEV).manual_seed(33)
    Gbuf = torch.randn((n, cfg.d + 64), generator=g, device=DEV)
    G = Gbuf[:, :cfg.d]
    sk = B.Sketch(*cfg.params, seed=cfg.sketch_seed)
    assert sk.plan(n, torch.float32, ld=cfg.d + 64, rows=True)["variant"] == B.VARIANT_MFMA
    out = sk.apply_rows(G)
    torch.cuda.synchronize()
    assert sk.info().last_variant == B.VARIANT_MFMA
    idx = torch.tensor([0, 31, 32, 127, 128, n - 1], device=DEV)
    ref = O.apply_rows(oracle_csc(cfg.params, cfg.sketch_seed), host64(G[idx]))
    check(out[idx], ref, torch.float32, "long fp32 rows, sampled examples")


@pytest.mark.parametrize("params,n", [
    ((65536, 65536, 65536, 65536, 1, 2), 8),     # Br at its maximum, one block
    ((1 << 20, 1 << 20, 1, 1, 5, 1), 3),         # Br = Bc = 1, M = 2^20 blocks
    ((4096, 32768, 1, 8, 7, 8), 5),              # expanding sketch (k > d), s = Br
])
def test_extreme_shapes(params, n):
    """Limits of the parameter ranges the header allows; these run on the generic kernel."""
    print("extreme", params, n, flush=True)
    A = torch.randn((params[0], n), generator=torch.Generator(device=DEV).manual_seed(4), device=DEV)
    sk = B.Sketch(*params, seed=3)
    out = sk.apply(A)
    rows, signs = sk.export()
    torch.cuda.synchronize()
    P = O.Params(*params)
    check(out, O.apply(O.build_csc(P, 3), host64(A)), torch.float32, "extreme shape")
    want_r, want_s = O.build_tables(P, 3)
    assert np.array_equal(rows.cpu().numpy().astype(np.int64), want_r)
    assert np.array_equal(signs.cpu().numpy(), want_s)


# ------------------------------------------------ boundary behaviour ------
def test_caller_workspace_and_too_small_workspace():
    params, n = (65536, 8192, 64, 8, 8, 2), 256
    A = torch.randn((params[0], n), device=DEV).to(torch.bfloat16)
    sk = B.Sketch(*params, seed=1)
    need = sk.workspace_bytes(n, torch.bfloat16)
    assert need > 0
    exact = sk.plan(n, torch.bfloat16)["workspace_bytes"]
    assert 0 < exact <= need                # the query is an upper bound over alignments and modes
    ref = sk.apply(A)                       # internal, lazily grown workspace
    assert sk.info().workspace_bytes >= exact
    ws = torch.empty(need + 256, dtype=torch.uint8, device=DEV)
    off = (-ws.data_ptr()) % 256
    sk.set_workspace(ws[off:off + need])
    got = sk.apply(A)                       # caller-owned workspace, no allocation
    torch.cuda.synchronize()
    assert torch.equal(ref, got)
    sk.set_workspace(ws[off:off + 256])     # too small: must fail, not overrun
    with pytest.raises(B.FlashSketchError) as e:
        sk.apply(A)
    assert e.value.status == 3
    sk.set_workspace(None)
    assert torch.equal(sk.apply(A), ref)


def test_prepare_then_applies_on_a_caller_workspace_allocate_nothing():
    """After fs_sketch_prepare (device tables) and fs_sketch_set_workspace, an apply only enqueues
    kernels: device memory in use stays what it was, and the result equals the lazily set-up one."""
    params, n = (65536, 8192, 64, 8, 8, 2), 256   # orbit-run mode: uses the table and partial planes
    A = torch.randn((params[0], n), device=DEV).to(torch.bfloat16)
    lazy = B.Sketch(*params, seed=4)
    ref = lazy.apply(A)
    assert lazy.info().last_mode == 3
    sk = B.Sketch(*params, seed=4)
    ws = torch.empty(sk.workspace_bytes(n, torch.bfloat16) + 256, dtype=torch.uint8, device=DEV)
    off = (-ws.data_ptr()) % 256
    sk.set_workspace(ws[off:])
    sk.prepare()
    out = torch.empty_like(ref)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(3):
        ws.fill_(0xFF)                      # the workspace need not survive between calls
        sk.apply(A, out)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "an apply allocated device memory"
    assert sk.info().last_mode == 3
    assert torch.equal(out, ref)
    sk.prepare()                            # idempotent
    assert torch.equal(sk.apply(A), ref)


def test_apply_on_a_side_stream_and_profile_brackets():
    params, n = (4096, 256, 512, 32, 2, 4), 512
    A = torch.randn((params[0], n), device=DEV)
    sk = B.Sketch(*params, seed=0)
    ref = sk.apply(A)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    out = torch.empty_like(ref)
    sk.profile_begin(3)
    with torch.cuda.stream(side):
        for _ in range(5):                  # two more applies than brackets: extra ones run unbracketed
            sk.apply(A, out, stream=side)
    side.synchronize()
    ms, ms_apply = sk.profile_end(whole=True)
    assert len(ms) == 3 and all(0.0 < t < 50.0 for t in ms)
    # the whole-apply bracket contains the dominant kernel's (tiny runs input-stationary: + a reduction)
    assert len(ms_apply) == 3 and all(a >= t for a, t in zip(ms_apply, ms)) and all(a < 50.0 for a in ms_apply)
    assert torch.equal(out, ref)
    with pytest.raises(B.FlashSketchError):
        sk.profile_end()                    # not profiling any more


@pytest.mark.parametrize("params,n,chunk", [
    ((32768, 64, 4096, 8, 8, 2), 1024, 256),     # IN-stationary with partial planes + reduce kernel
    ((65536, 8192, 64, 8, 8, 2), 512, 256),      # orbit-run mode
    ((8192, 1024, 512, 64, 4, 8), 512, 512),     # OUT-stationary, direct store
    ((8192, 2048, 64, 16, 16, 2), 512, 256),     # slot groups
    ((4096, 1024, 1024, 256, 2, 8), 512, 256),   # 128-row slices of a 256-row block, split stages
    ((8192, 4096, 128, 64, 4, 8), 7168, 3584),   # four output blocks per wave
])
def test_chunked_apply_replays_from_a_hip_graph(params, n, chunk):
    """The apply only enqueues kernels once a handle has run once (workspace and orbit table
    exist), so a chunk loop can be captured into a HIP graph.  Several replays, with eager work
    and synchronisations between them, must each reproduce the eager result bit for bit."""
    print("graph", params, flush=True)
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(11)
    A = torch.randn((d, n), generator=g, device=DEV).to(torch.bfloat16)
    sk = B.Sketch(*params, seed=2)
    eager = torch.empty((k, n), device=DEV, dtype=A.dtype)
    for c in range(0, n, chunk):
        sk.apply(A[:, c:c + chunk], eager[:, c:c + chunk])
    torch.cuda.synchronize()
    out = torch.zeros_like(eager)
    graph = torch.cuda.CUDAGraph()
    gc.collect()  # nothing that frees device memory may run during the capture (HIP rule)
    with torch.cuda.graph(graph):
        for c in range(0, n, chunk):
            sk.apply(A[:, c:c + chunk], out[:, c:c + chunk])
    for rep in range(3):
        out.zero_()
        scratch = sk.apply(A[:, :chunk])          # eager work of the same handle in between
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
        assert torch.equal(scratch, eager[:, :chunk])
    ref = O.apply(oracle_csc(params, 2), host64(A))
    check(out, ref, torch.bfloat16, "graph replay")


@pytest.mark.parametrize("params,n,chunk", [
    ((32768, 64, 4096, 8, 8, 2), 512, 256),      # input-stationary: partial records + gather reduction
    ((8192, 1024, 512, 64, 4, 8), 256, 128),     # output-stationary
    ((1152, 72, 96, 6, 5, 3), 140, 70),          # general kernel
])
def test_chunked_apply_rows_replays_from_a_hip_graph(params, n, chunk):
    """The same for the examples-as-rows entry point."""
    print("graph rows", params, flush=True)
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(12)
    G = torch.randn((n, d), generator=g, device=DEV).to(torch.bfloat16)
    sk = B.Sketch(*params, seed=2)
    eager = torch.empty((n, k), device=DEV, dtype=G.dtype)
    for c in range(0, n, chunk):
        sk.apply_rows(G[c:c + chunk], eager[c:c + chunk])
    torch.cuda.synchronize()
    out = torch.zeros_like(eager)
    graph = torch.cuda.CUDAGraph()
    gc.collect()
    with torch.cuda.graph(graph):
        for c in range(0, n, chunk):
            sk.apply_rows(G[c:c + chunk], out[c:c + chunk])
    for rep in range(3):
        out.zero_()
        scratch = sk.apply_rows(G[:chunk])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
        assert torch.equal(scratch, eager[:chunk])
    check(out, O.apply_rows(oracle_csc(params, 2), host64(G)), torch.bfloat16, "graph replay, rows")


# ------------------------------------------ examples-as-rows layout -------
ROWS = [
    # params (d,k,Bc,Br,kappa,s), n examples, ldg pad, ldo pad
    ((4096, 256, 512, 32, 2, 4), 300, 0, 0),        # tiny config: 64 stacked rows, ragged example tile
    ((4096, 256, 512, 32, 2, 4), 128, 8, 4),        # padded leading dimensions
    ((32768, 64, 4096, 8, 8, 2), 256, 0, 0),        # gradient-config blocks
    ((32768, 64, 4096, 8, 8, 2), 5, 0, 0),          # a handful of examples
    ((16384, 256, 2048, 32, 4, 4), 72, 0, 0),       # tall-config blocks: 128 stacked rows
    ((8192, 512, 1024, 64, 2, 8), 130, 0, 0),       # mid-config blocks, kappa = 2
    ((2048, 1024, 64, 32, 1, 1), 33, 0, 0),         # kappa = 1, one stage per block, s = 1
    ((65536, 8192, 64, 8, 8, 2), 64, 0, 0),         # M = 1024
    ((8192, 1024, 512, 64, 4, 8), 200, 0, 0),       # kappa*Br = 256: output-stationary, mid-config blocks
    ((16384, 1024, 2048, 128, 4, 8), 130, 8, 0),    # wide-config blocks, Br = 128
    ((4096, 1024, 128, 32, 8, 1), 64, 0, 4),        # Br = 32, kappa = 8, two stages per block
    ((2048, 4096, 64, 128, 3, 32), 40, 0, 0),       # one stage per block, s = 32
    # kappa*Br below the tile height
    ((6144, 768, 256, 32, 3, 4), 100, 0, 0),        # 96 stacked rows in a 128-row tile
    ((2048, 128, 128, 8, 5, 2), 130, 8, 0),         # 40 in 64
    ((4096, 64, 64, 1, 4, 1), 70, 0, 0),            # Br = 1: 4 in 32, scalar reduction
    ((4096, 128, 512, 16, 1, 4), 64, 0, 4),         # kappa = 1, Br = 16
    ((512, 16, 64, 2, 7, 2), 33, 0, 0),             # 14 in 32
    # more than 128 stacked rows of small blocks: groups of 128/Br wiring slots
    ((8192, 2048, 64, 16, 16, 2), 33, 0, 0),        # 256 rows: two full groups
    ((2048, 256, 64, 8, 20, 2), 130, 0, 0),         # 160 rows: a full group and one of 4 slots
    ((4096, 256, 64, 4, 40, 3), 70, 8, 4),          # Br = 4: groups of 32 slots
    # d not a multiple of Bc: the entries of the last block at or beyond d are cleared in registers
    ((4000, 256, 512, 32, 2, 4), 130, 0, 0),        # 416 of 512 entries, input-stationary
    ((4001, 256, 512, 32, 2, 4), 70, 7, 0),         # odd d: the cut falls inside a dword (16-bit types)
    ((7000, 448, 1024, 64, 4, 8), 100, 0, 4),       # output-stationary, M = 7, whole stages beyond d
    # rows that are not 16-byte aligned: four dword loads per piece, or (an odd ldg of a 16-bit
    # type) eight element loads
    ((4096, 256, 512, 32, 2, 4), 128, 2, 0),        # ldg = 4098
    ((4096, 256, 512, 32, 2, 4), 70, 1, 1),         # ldg = 4097
    ((16384, 256, 2048, 32, 4, 4), 72, 3, 0),       # 128 stacked rows, ldg = 16387
    ((8192, 1024, 512, 64, 4, 8), 100, 1, 0),       # output-stationary, ldg = 8193
    ((8192, 1024, 512, 64, 4, 8), 100, 2, 0),       # output-stationary, ldg = 8194
    ((4001, 256, 512, 32, 2, 4), 40, 1, 0),         # ldg = 4002 and a partly filled last block
    # Bc not a multiple of the 64-entry stage: no nonzeros of Phi^T past the block
    ((4000, 256, 500, 32, 2, 4), 130, 0, 0),        # Bc = 500
    ((1000, 256, 125, 32, 2, 4), 70, 0, 0),         # Bc = 125: blocks start at odd entries
    ((1536, 1024, 96, 64, 4, 4), 100, 0, 0),        # Bc = 96, output-stationary
    ((1990, 128, 250, 16, 8, 2), 64, 2, 0),         # Bc = 250 and a partly filled last block
    # output blocks higher than the 128-row tile: 128-row slices
    ((4096, 1024, 1024, 256, 2, 8), 129, 0, 0),     # Br = 256
    ((8192, 4096, 1024, 512, 3, 32), 70, 2, 0),     # Br = 512, s = 32
    ((2048, 2048, 1024, 1024, 1, 16), 40, 0, 4),    # Br = 1024, kappa = 1
    # Br not a power of two: slots padded to the next power of two of tile rows
    ((1152, 72, 96, 6, 5, 3), 70, 1, 3),            # Br = 6, M = 12, odd row stride
    ((1440, 180, 80, 10, 18, 10), 5, 0, 0),         # kappa = M, s = Br = 10: slot groups
    ((1440, 180, 80, 10, 18, 10), 130, 2, 0),       # the same over two example tiles
    ((1024, 768, 64, 48, 2, 5), 100, 0, 0),         # Br = 48: vector reduction, two slots of 64
    ((512, 768, 64, 96, 1, 8), 64, 0, 4),           # Br = 96, kappa = 1
    ((8192, 48, 1024, 6, 4, 2), 64, 0, 0),          # Br = 6 with few, long blocks: split rows
    ((8320, 4160, 64, 32, 130, 1), 40, 0, 0),       # kappa = 130 > 128: groups of four 32-row slots
    # shapes only the general kernel takes
    ((256, 384, 64, 96, 2, 4), 70, 0, 0),           # Br = 96, kappa = 2: 256 padded rows
    ((8320, 16640, 64, 128, 130, 1), 40, 0, 0),     # kappa = 130 with Br = 128
]


@pytest.mark.parametrize("variant", [B.VARIANT_AUTO, B.VARIANT_GENERIC], ids=lambda v: VNAME[v])
@DTYPES
@pytest.mark.parametrize("case", ROWS, ids=lambda c: f"{c[0]}-n{c[1]}")
def test_apply_rows_matches_oracle(case, dtype, variant):
    params, n, pg, po = case
    print("rows", params, n, dtype, VNAME[variant], flush=True)
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(n + k)
    Gbuf = torch.randn((n + 3, d + pg), generator=g, device=DEV).to(dtype)
    Gbuf[n:] = float("nan")         # memory past the last example must never reach the result
    if pg:
        Gbuf[:, d:] = float("nan")
    G = Gbuf[:n, :d]
    obuf = torch.full((n, k + po), float("nan"), device=DEV, dtype=dtype)
    sk = make_sketch(params, 9, variant)
    sk.apply_rows(G, obuf[:, :k])
    torch.cuda.synchronize()
    plan, did = sk.plan(n, dtype, ld=G.stride(0), rows=True, address=G.data_ptr()), sk.info()
    assert plan["variant"] == did.last_variant
    ref = O.apply_rows(oracle_csc(params, 9), host64(G))
    check(obuf[:, :k], ref, dtype, "apply_rows")
    if po:
        assert torch.isnan(obuf[:, k:].float()).all(), "wrote outside the k output columns"
    tol = ETOL[dtype]
    diff = np.abs(host64(obuf[:, :k]) - ref)
    assert (diff <= tol * (np.abs(ref) + np.sqrt((ref ** 2).mean()))).all()
    again = sk.apply_rows(G)                      # no atomics on data: bit-identical run to run
    torch.cuda.synchronize()
    assert torch.equal(again, obuf[:, :k])
    # and it is the transpose of the column-layout apply, to rounding
    colwise = sk.apply(G.t().contiguous())
    torch.cuda.synchronize()
    check(colwise.t(), ref, dtype, "column layout on the transpose")


def test_apply_rows_one_hot_rows_reproduce_columns_exactly():
    params = (32768, 64, 4096, 8, 8, 2)  # kappa*s = 16: the scale is a power of two
    d, k = params[0], params[1]
    rng = np.random.default_rng(2)
    cols = np.unique(np.r_[0, d - 1, 4095, 4096, rng.integers(0, d, 60)])
    G = torch.zeros((len(cols), d), device=DEV, dtype=torch.bfloat16)
    G[torch.arange(len(cols), device=DEV), torch.from_numpy(cols).to(DEV)] = 1.0
    sk = B.Sketch(*params, seed=0)
    out = sk.apply_rows(G)
    torch.cuda.synchronize()
    want = oracle_csc(params, 0)[:, cols].toarray().T
    assert np.array_equal(host64(out), want)


def test_apply_rows_forced_matrix_core_variant_reports_unsupported_shapes():
    """Shapes the matrix-core rows kernel cannot take run on the general one; forcing the
    matrix-core variant turns them into FS_ERR_UNSUPPORTED instead."""
    for params in [(256, 384, 64, 96, 2, 4),         # Br = 96, kappa = 2: 256 padded rows
                   (8320, 16640, 64, 128, 130, 1)]:  # kappa = 130 with Br = 128
        G = torch.zeros((4, params[0]), device=DEV, dtype=torch.bfloat16)
        sk = B.Sketch(*params, seed=0)
        sk.apply_rows(G)
        assert sk.info().last_variant == B.VARIANT_GENERIC
        sk.set_variant(B.VARIANT_MFMA)
        with pytest.raises(B.FlashSketchError) as e:
            sk.apply_rows(G)
        assert e.value.status == 2
    torch.cuda.synchronize()


def test_handle_collected_during_a_capture_does_not_break_it():
    """Destroying a handle frees device memory, which HIP forbids while a stream is capturing.  A
    handle that the garbage collector finds during a capture is parked by the binding and
    destroyed later; the capture stays valid."""
    params, n = (32768, 64, 4096, 8, 8, 2), 256
    A = torch.randn((params[0], n), device=DEV).to(torch.bfloat16)
    sk = B.Sketch(*params, seed=2)
    eager = sk.apply(A)

    class Cycle:  # a dead reference cycle holding a used handle: only the cyclic collector frees it
        pass
    c = Cycle()
    c.me, c.sk = c, B.Sketch(*params, seed=3)
    c.sk.apply(A)
    torch.cuda.synchronize()
    del c
    out = torch.zeros_like(eager)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        gc.collect()          # the cycle dies here, inside the capture
        sk.apply(A, out)
    assert len(B._deferred) >= 1  # (dead handles of earlier tests may have been found as well)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, eager)
    sk.close()                # flushes the parked handle
    assert len(B._deferred) == 0


@DTYPES
def test_variants_agree_with_each_other(dtype):
    """Generic and MFMA paths implement the same S: they agree to accumulation rounding."""
    params, n = (16384, 256, 2048, 32, 4, 4), 384
    A = torch.randn((params[0], n), device=DEV).to(dtype)
    outs = []
    for v in (B.VARIANT_GENERIC, B.VARIANT_MFMA, B.VARIANT_AUTO):
        sk = make_sketch(params, 9, v)
        outs.append(host64(apply_or_skip(sk, A)))
    torch.cuda.synchronize()
    tol = 1e-5 if dtype == torch.float32 else ETOL[dtype]
    assert O.rel_fro_err(outs[1], outs[0]) < tol
    assert np.array_equal(outs[1], outs[2])  # AUTO picked the MFMA path


# ------------------------------------------------ seeded random shapes ----
def _random_cases(count, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        Br = int(rng.choice([1, 2, 4, 8, 16, 32, 64, 128, 3, 12]))
        M = int(rng.choice([1, 2, 4, 8, 16, 64, 256, 6]))
        Bc = int(rng.choice([64, 128, 256, 512, 96]))
        kappa = int(rng.integers(1, min(M, 8) + 1))
        s = int(rng.integers(1, min(Br, 8) + 1))
        n = int(rng.choice([1, 5, 64, 127, 128, 129, 255, 256, 260, 515]))
        if M * Bc * n > 2 ** 24:
            continue
        cases.append(((M * Bc, M * Br, Bc, Br, kappa, s), n, int(rng.integers(0, 2 ** 62))))
    return cases


def _random_cases_wide(count, seed):
    """A wider draw: high and tiny blocks, many wiring slots, block widths that are not whole
    stages, a partly filled last block -- the combinations of the dispatcher's special modes."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        Br = int(rng.choice([1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 6, 48, 96]))
        M = int(rng.choice([1, 2, 3, 4, 8, 16, 40, 64, 130]))
        Bc = int(rng.choice([8, 40, 64, 72, 96, 125, 128, 200, 256, 500]))
        kappa = int(rng.integers(1, min(M, 40) + 1))
        s = int(rng.integers(1, min(Br, 32) + 1))
        n = int(rng.choice([1, 3, 64, 100, 128, 130, 255, 256, 301]))
        short = int(rng.choice([0, 0, 1, Bc // 2]))        # rows missing from the last block
        d = M * Bc - min(short, Bc - 1)
        if M * Bc * n > 2 ** 23 or M * Br * n > 2 ** 23:
            continue
        cases.append(((d, M * Br, Bc, Br, kappa, s), n, int(rng.integers(0, 2 ** 62))))
    return cases


@DTYPES
def test_random_shapes_wide_draw_both_layouts(dtype):
    """60 seeded draws; the column apply (packed, so lda = n is often not a multiple of 4) and the
    rows apply (packed too: ldg = d) against the oracle, whatever kernels the dispatcher picks."""
    seen = set()
    for params, n, seed in _random_cases_wide(60, 77):
        print("random wide", params, n, seed, dtype, flush=True)
        g = torch.Generator(device=DEV).manual_seed(seed % (2 ** 31))
        A = torch.randn((params[0], n), generator=g, device=DEV).to(dtype)
        sk = B.Sketch(*params, seed=seed)
        S = O.build_csc(O.Params(*params), seed)
        ref = O.apply(S, host64(A))
        out = sk.apply(A)
        i = sk.info()
        seen.add(("cols", i.last_variant, i.last_mode, sk.plan(n, dtype, address=A.data_ptr())["flags"]))
        check(out, ref, dtype, f"{params} n={n}")
        G = A.t().contiguous()
        out_r = sk.apply_rows(G)
        seen.add(("rows", sk.info().last_variant, sk.plan(n, dtype, rows=True, address=G.data_ptr())["flags"]))
        check(out_r.t(), ref, dtype, f"rows {params} n={n}")
        sk.close()
    torch.cuda.synchronize()
    flags = {f for key in seen if key[0] == "cols" for f in (key[3],)}
    assert any(f & B.PLAN_ELEMENT_LOADS for f in flags) and any(f & B.PLAN_SLOT_GROUPS for f in flags) \
        and any(f & B.PLAN_ROW_SLICES for f in flags), seen
    assert ("cols", B.VARIANT_GENERIC, 0, 0) in seen


def _random_cases_many_work_groups(count, seed):
    """Shapes with enough (block, column tile) pairs for the kernels that want a chip full of
    work-groups: output-stationary with shared Phi tiles (whole and row-split), several output
    blocks per wave."""
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < count:
        Br = int(rng.choice([32, 64, 64, 128, 128]))
        M = int(rng.choice([4, 8, 16, 32, 64, 64, 128]))
        Bc = int(rng.choice([128, 200, 256, 384, 512, 1000, 1024]))
        kappa = min(int(rng.choice([2, 4, 4, 6, 8, 8, 12, 16])), M)
        s = min(int(rng.choice([1, 2, 3, 8, 8, 12, 20, 32])), Br)
        n = int(rng.choice([132, 256, 520, 1024, 1028, 1536, 2048, 2050, 3072, 4096, 4100, 6144]))
        d = M * Bc - int(rng.choice([0, 0, 0, 7, Bc // 3]))
        if d * n > 6e7:
            n = max(130, int(6e7 // d) // 2 * 2)
        cases.append(((d, M * Br, Bc, Br, kappa, s), n, int(rng.choice([0, 0, 2, 4, 3])), int(rng.integers(0, 2 ** 62))))
    return cases


@DTYPES
def test_random_shapes_many_work_groups(dtype):
    """70 seeded draws at sizes where the dispatcher picks the kernels built for full chips.  All
    columns against the general kernel on the device (two implementations that share only the
    hash recipe), 24 sampled columns against the oracle."""
    kernels = set()
    for params, n, pad, seed in _random_cases_many_work_groups(70, 4242):
        print("random many", params, n, pad, seed, dtype, flush=True)
        g = torch.Generator(device=DEV).manual_seed(seed % (2 ** 31))
        A = torch.randn((params[0], n + pad), generator=g, device=DEV).to(dtype)[:, :n]
        sk = B.Sketch(*params, seed=seed)
        out = sk.apply(A)
        kern = sk.info().last_kernel.decode()
        kernels.add(kern.split("<")[0] + ("+reduce" if kern.endswith("+reduce_planes") else ""))
        sk.set_variant(B.VARIANT_GENERIC)
        other = sk.apply(A)
        sk.set_variant(B.VARIANT_AUTO)
        torch.cuda.synchronize()
        a, b = out.float(), other.float()
        assert float((a - b).norm() / b.norm()) <= TOL[dtype], (params, n, kern)
        cols = np.unique(np.r_[0, n - 1, np.random.default_rng(seed % 1000).integers(0, n, 22)])
        ref = O.apply(oracle_csc(params, seed), host64(A[:, torch.from_numpy(cols).to(DEV)]))
        check(out[:, torch.from_numpy(cols).to(DEV)], ref, dtype, f"{params} n={n} {kern}")
        sk.close()
    want = {"stacked_kernel", "mfma_kernel", "mfma_kernel+reduce"}
    if dtype != torch.float32:
        want |= {"outs_kernel", "outs_kernel+reduce"}
    assert want <= kernels, kernels


@pytest.mark.parametrize("variant", [B.VARIANT_AUTO, B.VARIANT_GENERIC], ids=lambda v: VNAME[v])
@DTYPES
def test_random_shapes_match_oracle(dtype, variant):
    """40 seeded random parameter sets (power-of-two and odd Br, composite M, ragged n): whichever
    kernel the dispatcher (or the forced generic variant) runs must match the oracle, and the
    exported nonzeros must be the oracle's."""
    modes = set()
    for params, n, seed in _random_cases(40, 2024):
        print("random", params, n, seed, dtype, VNAME[variant], flush=True)
        g = torch.Generator(device=DEV).manual_seed(seed % (2 ** 31))
        A = torch.randn((params[0], n + (-n) % 4), generator=g, device=DEV).to(dtype)[:, :n]
        sk = make_sketch(params, seed, variant)
        out = sk.apply(A)
        i = sk.info()
        modes.add((i.last_variant, i.last_mode))
        S = O.build_csc(O.Params(*params), seed)
        check(out, O.apply(S, host64(A)), dtype, f"{params} n={n}")
        if dtype == torch.float32 and variant == B.VARIANT_AUTO:
            rows, signs = sk.export()
            want_r, want_s = O.build_tables(O.Params(*params), seed)
            assert np.array_equal(rows.cpu().numpy().astype(np.int64), want_r)
            assert np.array_equal(signs.cpu().numpy(), want_s)
    if variant == B.VARIANT_AUTO:
        assert {m for v, m in modes if v == B.VARIANT_MFMA} >= {1, 2}, modes  # both MFMA modes were hit
        assert all(v == B.VARIANT_MFMA for v, m in modes), modes   # every draw has a matrix-core kernel


# ------------------------------------------------ FlashBlockRow kind ------
@DTYPES
@pytest.mark.parametrize("case", [
    ((4096, 256, 512, 32, 2, 4), 512, 0), ((4000, 256, 512, 32, 2, 4), 301, 3),
    ((1152, 72, 96, 6, 5, 3), 65, 0), ((65536, 8192, 64, 8, 8, 2), 260, 0),
    ((16384, 1024, 2048, 128, 4, 8), 1000, 0), ((1024, 64, 1024, 64, 1, 8), 1, 0),
], ids=lambda c: f"{c[0]}-n{c[1]}")
def test_blockrow_matches_oracle(case, dtype):
    from oracle import blockrow as R
    params, n, pad = case
    print("blockrow", params, n, dtype, flush=True)
    seed = 11
    g = torch.Generator(device=DEV).manual_seed(n)
    A = torch.randn((params[0], n + pad), generator=g, device=DEV).to(dtype)[:, :n]
    sk = B.Sketch(*params, seed=seed, kind=B.KIND_BLOCKROW)
    out = sk.apply(A)
    cols, signs = sk.export()
    torch.cuda.synchronize()
    p = O.Params(*params)
    want_c, want_s = R.build_tables(p, seed)
    assert np.array_equal(cols.cpu().numpy().astype(np.int64), want_c)
    assert np.array_equal(signs.cpu().numpy(), want_s)
    assert abs(sk.info().scale - R.scale(p)) <= 1e-7 * R.scale(p)
    check(out, R.apply(R.build_csr(p, seed), host64(A)), dtype, "blockrow")
