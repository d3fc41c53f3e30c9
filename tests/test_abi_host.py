"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, rejects bad arguments before touching HIP, and its host-side
seed -> wiring derivation agrees with the oracle's integers."""
import ctypes as C
import os
import re

import pytest

from oracle import blockperm as O
from paper_2602_06071_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "flashsketch.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fs_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(B.lib, n), n
    assert sorted(B.SYMBOLS) == names


def _create(*args, kind=B.KIND_BLOCKPERM):
    h = C.c_void_p()
    st = B.lib.fs_sketch_create_kind(C.byref(h), kind, *args)
    return st, h


@pytest.mark.parametrize("args", [
    (0, 256, 512, 32, 2, 4, 0),       # d < 1
    (4096, 0, 512, 32, 2, 4, 0),      # k < 1
    (4096, 256, 500, 32, 2, 4, 0),    # ceil(d/Bc) = 9 != k/Br = 8
    (4096, 256, 512, 48, 2, 4, 0),    # Br does not divide k
    (4096, 256, 512, 64, 2, 4, 0),    # d/Bc != k/Br
    (3584, 256, 512, 32, 2, 4, 0),    # one whole block short of a square grid
    (4096, 256, 512, 32, 9, 4, 0),    # kappa > M
    (4096, 256, 512, 32, 0, 4, 0),    # kappa < 1
    (4096, 256, 512, 32, 2, 0, 0),    # s < 1
    (4096, 256, 512, 32, 2, 33, 0),   # s > 32 (and > Br)
    (4096, 64, 512, 8, 2, 9, 0),      # s > Br
    (262144, 262144, 2, 2, 1, 3, 0),  # s > Br
    (1 << 25, 1 << 25, 1, 1, 1, 1, 0),  # M > 2^24
])
def test_create_rejects_bad_params(args):
    st, h = _create(*args)
    assert st == 1 and not h.value
    # the oracle rejects the same parameter sets
    with pytest.raises(ValueError):
        p = O.Params(*args[:6])
        p.check()
        if p.M > (1 << 24):
            raise ValueError("M too large for the library")


def test_create_null_out_and_bad_kind():
    assert B.lib.fs_sketch_create(None, 4096, 256, 512, 32, 2, 4, 0) == 1
    st, _ = _create(4096, 256, 512, 32, 2, 4, 0, kind=7)
    assert st == 1
    st, _ = _create(4096, 256, 512, 32, 2, 4, 0, kind=B.KIND_SJLT_SCATTER)  # needs M = 1
    assert st == 1
    st, _ = _create(1000, 64, 1024, 64, 1, 4, 0, kind=B.KIND_SJLT_SCATTER)  # Bc > d: a padded block
    assert st == 1
    st, h = _create(4096, 256, 4096, 256, 1, 4, 0, kind=B.KIND_SJLT_SCATTER)
    assert st == 0
    assert B.lib.fs_sketch_destroy(h) == 0
    assert B.lib.fs_sketch_destroy(None) == 1


@pytest.mark.parametrize("cfg", [
    (4096, 256, 512, 32, 2, 4), (16384, 1024, 1024, 64, 8, 8), (262144, 4096, 2048, 32, 4, 4),
    (65536, 4096, 2048, 128, 4, 8), (4194304, 8192, 4096, 8, 8, 2), (1152, 72, 96, 6, 5, 3),
    (4000, 256, 512, 32, 2, 4), (3585, 256, 512, 32, 2, 4),
    (1440, 180, 80, 10, 18, 10), (512, 512, 1, 1, 3, 1), (1024, 64, 1024, 64, 1, 8),
])
@pytest.mark.parametrize("seed", [0, 1, 0xDEADBEEF12345678])
def test_host_wiring_matches_oracle(cfg, seed):
    sk = B.Sketch(*cfg, seed=seed)
    i = sk.info()
    p = O.Params(*cfg)
    k0, k1 = O.seed_keys(seed)
    a, b = O.wiring(p.M, k1)
    assert (i.key0, i.key1, i.M, i.a, i.b) == (k0, k1, p.M, a, b)
    if p.M > 1:
        assert (i.a * i.a_inv) % p.M == 1
    assert abs(i.scale - (cfg[4] * cfg[5]) ** -0.5) < 1e-7
    assert (i.d, i.k, i.Bc, i.Br, i.kappa, i.s) == cfg
    sk.close()


def test_apply_argument_errors_before_any_hip_call():
    sk = B.Sketch(4096, 256, 512, 32, 2, 4)
    h = sk._h
    buf = C.c_void_p(4096)  # never dereferenced: every call below must fail or no-op first
    L = B.lib
    assert L.fs_sketch_apply(None, buf, 8, 8, buf, 0, None) == 1
    assert L.fs_sketch_apply(h, buf, 8, 0, buf, 0, None) == 0          # n = 0: nothing to do
    assert L.fs_sketch_apply(h, None, 8, 8, buf, 0, None) == 1         # NULL A
    assert L.fs_sketch_apply(h, buf, 8, 8, None, 0, None) == 1         # NULL out
    assert L.fs_sketch_apply(h, buf, 7, 8, buf, 0, None) == 1          # lda < n
    assert L.fs_sketch_apply(h, buf, 8, -1, buf, 0, None) == 1         # n < 0
    assert L.fs_sketch_apply(h, buf, 8, 8, buf, 5, None) == 1          # unknown dtype
    assert L.fs_sketch_apply_ld(h, buf, 8, 8, buf, 7, 0, None) == 1    # ldo < n
    assert L.fs_sketch_apply(h, C.c_void_p(4098), 8, 8, buf, 0, None) == 1  # misaligned fp32
    assert L.fs_sketch_export(h, None, buf, None) == 1
    assert L.fs_sketch_set_variant(h, 9) == 1
    assert L.fs_sketch_set_workspace(h, C.c_void_p(4096 + 8), 64) == 1  # not 256-aligned
    assert L.fs_sketch_set_workspace(h, None, 64) == 1
    assert L.fs_sketch_info(h, None) == 1
    out = C.c_size_t(123)
    assert L.fs_sketch_workspace_bytes(h, 0, 0, C.byref(out)) == 0 and out.value == 0
    assert L.fs_sketch_workspace_bytes(h, -1, 0, C.byref(out)) == 1
    assert L.fs_status_string(0) == b"ok" and L.fs_status_string(1) == b"invalid argument"
    # examples-as-rows entry point: G is n x 4096 (ldg >= d), out is n x 256 (ldo >= k)
    assert L.fs_sketch_apply_rows(None, buf, 4096, 8, buf, 256, 0, None) == 1
    assert L.fs_sketch_apply_rows(h, buf, 4096, 0, buf, 256, 0, None) == 0    # n = 0
    assert L.fs_sketch_apply_rows(h, None, 4096, 8, buf, 256, 0, None) == 1   # NULL G
    assert L.fs_sketch_apply_rows(h, buf, 4096, 8, None, 256, 0, None) == 1   # NULL out
    assert L.fs_sketch_apply_rows(h, buf, 4095, 8, buf, 256, 0, None) == 1    # ldg < d
    assert L.fs_sketch_apply_rows(h, buf, 4096, 8, buf, 255, 0, None) == 1    # ldo < k
    assert L.fs_sketch_apply_rows(h, buf, 4096, -1, buf, 256, 0, None) == 1   # n < 0
    assert L.fs_sketch_apply_rows(h, buf, 4096, 8, buf, 256, 7, None) == 1    # unknown dtype
    assert L.fs_sketch_set_variant(h, B.VARIANT_MFMA) == 0                    # (AUTO would run the general kernel)
    assert L.fs_sketch_apply_rows(h, C.c_void_p(4097), 4096, 8, buf, 256, 1, None) == 1   # G not element aligned
    assert L.fs_sketch_rows_workspace_bytes(h, 8, 0, C.byref(out)) == 0
    one_set = 2 * 8 * 256 * 4                                                 # kappa planes of n x k floats
    assert out.value >= one_set and out.value % one_set == 0                  # times the row split
    assert L.fs_sketch_rows_workspace_bytes(h, -1, 0, C.byref(out)) == 1
    sk.close()
    big = B.Sketch(4096, 6144, 64, 96, 2, 4)                                  # Br = 96, kappa = 2: 256 padded rows
    big.set_variant(B.VARIANT_MFMA)
    assert L.fs_sketch_apply_rows(big._h, buf, 4096, 8, buf, 6144, 0, None) == 2
    big.close()
