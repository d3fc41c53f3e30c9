"""Host-only checks of the dispatcher through fs_sketch_plan: which kernel, which work
decomposition and how much workspace an apply would use.  Nothing is launched, so these run
without a GPU; tests/test_gpu_parity.py checks that the applies do what the plan says."""
import ctypes as C

import pytest
import torch

from paper_2602_06071_amd import binding as B
from paper_2602_06071_amd import workloads as W

GENERIC, MFMA = B.VARIANT_GENERIC, B.VARIANT_MFMA
OUT, IN, RUNS = 1, 2, 3
EL, SL, GR, SP, ST = B.PLAN_ELEMENT_LOADS, B.PLAN_ROW_SLICES, B.PLAN_SLOT_GROUPS, B.PLAN_SPLIT, B.PLAN_STACKED


def plan(params, n, dtype, **kw):
    sk = B.Sketch(*params)
    try:
        return sk.plan(n, dtype, **kw)
    finally:
        sk.close()


def test_the_five_configurations_take_the_decompositions_they_were_designed_for():
    want = {"grad": (RUNS, 0), "wide": (OUT, 0), "tall": (IN, SP), "tiny": (IN, SP)}
    for name, (mode, flags) in want.items():
        cfg = W.CONFIGS[name]
        n = cfg.chunk or cfg.n
        p = plan(cfg.params, n, cfg.dtype, ld=cfg.n)
        assert (p["variant"], p["mode"], p["flags"]) == (MFMA, mode, flags), (name, p)
    # mid: output-stationary throughout (kappa = 2: the planes would cost more than the re-read); from
    # kappa = 4 on with four output blocks per wave
    for kappa, flags in ((1, 0), (2, 0), (4, ST), (8, ST)):
        cfg = W.CONFIGS["mid"]
        params = cfg.params[:4] + (kappa,) + cfg.params[5:]
        p = plan(params, cfg.n, cfg.dtype)
        assert (p["variant"], p["mode"], p["flags"], p["workspace_bytes"]) == (MFMA, OUT, flags, 0), (kappa, p)
    # the gradient chunk: three merged planes of 8192 x 256 floats
    assert plan(W.CONFIGS["grad"].params, 256, torch.bfloat16, ld=1024)["workspace_bytes"] == 3 * 8192 * 256 * 4


@pytest.mark.parametrize("params,n,kw,want", [
    ((6144, 768, 256, 32, 3, 4), 300, {}, (MFMA, IN, None)),             # 96 stacked rows in a 128-row tile
    ((4096, 64, 64, 1, 4, 1), 256, {}, (MFMA, IN, None)),                # Br = 1
    ((8192, 2048, 64, 16, 16, 2), 300, {}, (MFMA, IN, GR)),              # two groups of 8 slots
    ((4096, 256, 64, 4, 40, 3), 72, {}, (MFMA, IN, GR)),                 # groups of 32 slots
    ((65536, 4096, 4096, 256, 4, 8), 2048, {}, (MFMA, OUT, SL | SP)),    # 128-row slices, split stages
    ((65536, 4096, 8192, 512, 4, 8), 8192, {}, (MFMA, OUT, SL)),
    ((1000, 256, 125, 32, 2, 4), 300, {}, (MFMA, IN, None)),             # Bc = 125
    ((4096, 256, 512, 32, 2, 4), 301, {}, (MFMA, IN, EL | SP)),          # lda = 301
    ((4096, 256, 512, 32, 2, 4), 300, {"address": 258}, (MFMA, IN, EL | SP)),   # A not aligned to 4 columns
    ((1152, 72, 96, 6, 5, 3), 65, {}, (MFMA, IN, None)),                 # Br = 6: slots of 8 tile rows
    ((1440, 180, 80, 10, 18, 10), 36, {}, (MFMA, IN, GR)),               # Br = 10: slots of 16, groups of 8
    ((256, 384, 64, 96, 2, 4), 64, {}, (GENERIC, 0, 0)),                 # Br = 96, kappa = 2: 256 padded rows
    ((16640, 4160, 64, 16, 130, 1), 64, {}, (MFMA, IN, GR)),             # kappa = 130: 17 groups of 8 slots
    ((8320, 16640, 64, 128, 130, 1), 64, {}, (GENERIC, 0, 0)),           # kappa = 130 with Br = 128
])
def test_column_layout_dispatch(params, n, kw, want):
    p = plan(params, n, torch.bfloat16, **kw)
    assert (p["variant"], p["mode"]) == want[:2], p
    if want[2] is not None:
        assert p["flags"] == want[2], p
    if p["variant"] == GENERIC:
        assert p["workspace_bytes"] == 0


@pytest.mark.parametrize("params,n,dtype,kw,want", [
    ((4194304, 8192, 4096, 8, 8, 2), 256, torch.bfloat16, {"ld": 4194304 + 64}, (MFMA, IN, 0)),
    ((4194304, 8192, 4096, 8, 8, 2), 256, torch.bfloat16, {"ld": 4194304 + 2}, (MFMA, IN, EL)),
    ((4194304, 8192, 4096, 8, 8, 2), 256, torch.bfloat16, {"ld": 4194304 + 1}, (MFMA, IN, EL)),
    ((2097152, 8192, 2048, 8, 8, 2), 256, torch.float32, {"ld": 2097152 + 1}, (MFMA, IN, EL)),
    ((4194304, 8192, 4096, 8, 8, 2), 256, torch.float32, {"ld": 4194304 + 64}, (MFMA, IN, 0)),
    ((16777216, 8192, 16384, 8, 8, 2), 64, torch.float32, {}, (GENERIC, 0, 0)),   # 34 rows span 2^31 bytes
    ((8192, 1024, 512, 64, 4, 8), 200, torch.float32, {}, (MFMA, OUT, 0)),
    ((4096, 1024, 1024, 256, 2, 8), 129, torch.float32, {}, (MFMA, OUT, SL)),
    ((8192, 2048, 64, 16, 16, 2), 33, torch.float32, {}, (MFMA, IN, GR)),
    ((1000, 256, 125, 32, 2, 4), 70, torch.bfloat16, {}, (MFMA, IN, EL)),      # blocks start at odd entries
    ((1000, 256, 125, 32, 2, 4), 70, torch.float32, {}, (MFMA, IN, EL)),       # 500-byte blocks: dword loads
    ((1152, 72, 96, 6, 5, 3), 70, torch.float32, {}, (MFMA, IN, 0)),          # Br = 6: slots of 8 tile rows
    ((256, 384, 64, 96, 2, 4), 70, torch.float32, {}, (GENERIC, 0, 0)),       # 256 padded rows
])
def test_rows_layout_dispatch(params, n, dtype, kw, want):
    p = plan(params, n, dtype, rows=True, **kw)
    assert (p["variant"], p["mode"], p["flags"] & ~SP) == want, p


def test_plan_honours_the_forced_variant_and_reports_errors():
    sk = B.Sketch(4096, 256, 512, 32, 2, 4)
    assert sk.plan(64, torch.float32)["variant"] == MFMA
    sk.set_variant(GENERIC)
    assert sk.plan(64, torch.float32) == {"variant": GENERIC, "mode": 0, "flags": 0, "workspace_bytes": 0}
    sk.set_variant(B.VARIANT_AUTO)
    L, h = B.lib, sk._h
    v = C.c_int32()
    a = C.c_void_p(256)
    assert L.fs_sketch_plan(None, a, 64, 64, 0, 0, C.byref(v), None, None, None) == 1
    assert L.fs_sketch_plan(h, None, 64, 64, 0, 0, C.byref(v), None, None, None) == 1      # NULL A
    assert L.fs_sketch_plan(h, a, 63, 64, 0, 0, C.byref(v), None, None, None) == 1         # lda < n
    assert L.fs_sketch_plan(h, a, 4095, 64, 0, 1, C.byref(v), None, None, None) == 1       # ldg < d
    assert L.fs_sketch_plan(h, a, 64, 64, 9, 0, C.byref(v), None, None, None) == 1         # unknown dtype
    assert L.fs_sketch_plan(h, a, 64, 64, 0, 2, C.byref(v), None, None, None) == 1         # rows is 0 or 1
    assert L.fs_sketch_plan(h, C.c_void_p(258), 64, 64, 0, 0, C.byref(v), None, None, None) == 1   # fp32 at 258
    assert L.fs_sketch_plan(h, a, 64, 0, 0, 0, C.byref(v), None, None, None) == 0 and v.value == GENERIC  # n = 0
    assert L.fs_sketch_plan(h, a, 64, 64, 0, 0, None, None, None, None) == 0               # every result optional
    sk.close()
    odd = B.Sketch(256, 384, 64, 96, 2, 4)   # Br = 96 with kappa = 2: no matrix-core kernel
    odd.set_variant(MFMA)
    with pytest.raises(B.FlashSketchError) as e:
        odd.plan(8, torch.float32)
    assert e.value.status == 2
    odd.close()
    sc = B.Sketch(4096, 256, 4096, 256, 1, 4, kind=B.KIND_SJLT_SCATTER)
    assert sc.plan(100, torch.bfloat16) == {"variant": GENERIC, "mode": 0, "flags": 0, "workspace_bytes": 256 * 100 * 4}
    with pytest.raises(B.FlashSketchError) as e:
        sc.plan(100, torch.bfloat16, rows=True)
    assert e.value.status == 2
    sc.close()


@pytest.mark.parametrize("params,n,dtype,kw,stacked", [
    ((16384, 1024, 1024, 64, 4, 8), 16384, torch.float32, {}, True),      # mid
    ((16384, 1024, 1024, 64, 4, 8), 16384, torch.bfloat16, {}, True),     # 64-row blocks: 16-bit too
    ((16384, 2048, 1024, 128, 2, 8), 16384, torch.float32, {}, True),     # 128-row blocks, fp32: two per wave
    ((65536, 4096, 2048, 128, 4, 8), 8192, torch.bfloat16, {}, False),    # wide: 16-bit 128-row blocks stay with one block per work-group
    ((16384, 1024, 1024, 64, 6, 8), 16384, torch.float32, {}, False),     # kappa not a multiple of the 4 slots
    ((16384, 1024, 1024, 64, 2, 8), 16384, torch.float32, {}, False),     # fewer permutations than slots
    ((16384, 1024, 1024, 64, 4, 8), 16383, torch.float32, {"ld": 16384}, False),  # odd n
    ((16384, 1024, 1024, 64, 4, 8), 16384, torch.float32, {"address": 260}, False),  # A not aligned to 2 columns
    ((16384, 1024, 1024, 64, 4, 8), 8192, torch.float32, {}, True),       # 4 groups x 32 column tiles: the 128 work-groups it asks for
    ((16384, 1024, 1024, 64, 4, 8), 7936, torch.float32, {}, False),      # 4 x 31: too few
    ((12288, 4096, 192, 64, 4, 8), 4096, torch.float32, {}, False),       # three 64-row stages per block
    ((8192, 2048, 128, 32, 8, 8), 4096, torch.float32, {}, False),        # 32-row blocks
])
def test_the_kernel_with_several_output_blocks_per_wave_takes_the_shapes_it_says(params, n, dtype, kw, stacked):
    p = plan(params, n, dtype, **kw)
    assert bool(p["flags"] & ST) == stacked, p
    if stacked:
        assert (p["variant"], p["mode"], p["workspace_bytes"]) == (MFMA, OUT, 0), p
