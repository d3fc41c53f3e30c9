"""fs_sketch_apply_static (the entry point for callers that cannot allocate device memory)
against fs_sketch_apply_ld, through the C ABI: same kernels on the library's static device
array instead of an allocated workspace, so the outputs must be bit-identical (the bar of the
parity tests for integer work, and for floating point with the same summation order); the
existing entry point is itself checked against the float64 oracle here and in
test_gpu_parity.py.  Each case makes two calls in a row on the shared array, the second with a
smaller input, with a different handle's call in between."""
import numpy as np
import pytest
import torch

from oracle import blockperm as O
from paper_2602_06071_amd import binding as B
from paper_2602_06071_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"
TOL = {torch.float32: 1e-5, torch.bfloat16: 4e-3, torch.float16: 5e-4}


def host64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


CASES = [
    # params (d,k,Bc,Br,kappa,s), dtype, n first, n second, expected mode (fs_info.last_mode)
    ((65536, 8192, 64, 8, 8, 2), torch.bfloat16, 300, 100, 3),   # orbit runs: planes + table, ragged tile
    ((4096, 256, 512, 32, 2, 4), torch.float32, 512, 77, 2),      # input-stationary: planes + reduction
    ((32768, 64, 4096, 8, 8, 2), torch.float16, 256, 64, 2),      # gradient-shaped blocks, row splits
    ((8192, 1024, 512, 64, 4, 8), torch.float32, 520, 130, 1),    # output-stationary: table only
    ((4096, 6144, 64, 96, 2, 4), torch.bfloat16, 65, 9, 0),       # general kernel: no scratch at all
    ((8192, 4096, 128, 64, 4, 8), torch.float32, 3584, 3072, 1),  # four output blocks per wave: table only
]


@pytest.mark.parametrize("params,dtype,n1,n2,mode", CASES)
def test_static_apply_equals_allocating_apply(params, dtype, n1, n2, mode):
    print("static", params, dtype, n1, n2, flush=True)
    d, k = params[0], params[1]
    g = torch.Generator(device=DEV).manual_seed(21)
    A = torch.randn((d, n1 + 8), generator=g, device=DEV).to(dtype)[:, :n1]    # padded lda
    sk = B.Sketch(*params, seed=5)
    other = B.Sketch(65536, 8192, 64, 8, 8, 2, seed=9)                          # another wiring on the same array
    A_other = torch.randn((65536, 256), generator=g, device=DEV).to(torch.bfloat16)
    want1 = sk.apply(A)
    assert sk.info().last_mode == mode
    want2 = sk.apply(A[:, :n2])
    want_other = other.apply(A_other)
    S = O.build_csc(O.Params(*params), 5)
    err = O.rel_fro_err(host64(want1), O.apply(S, host64(A)))
    assert err <= TOL[dtype], f"allocating apply vs oracle: {err:.3e}"
    got1 = torch.full((k, n1 + 3), float("nan"), device=DEV, dtype=dtype)      # padded ldo, poisoned
    got2 = torch.full((k, n2), float("nan"), device=DEV, dtype=dtype)
    got_other = torch.empty_like(want_other)
    # the first call in a process makes the runtime load the library's static array onto this
    # device (33 MiB, once, kept until the process ends); the calls after it must leave the amount
    # of free device memory alone
    sk.apply_static(A[:, :4], got2[:, :4])
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    sk.apply_static(A, got1[:, :n1])
    assert sk.info().last_mode == mode
    other.apply_static(A_other, got_other)       # overwrites planes and table with another sketch's
    sk.apply_static(A[:, :n2], got2)             # second call, smaller input, stale contents around
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0, "the static entry point changed the amount of free device memory"
    assert torch.equal(got1[:, :n1], want1)
    assert torch.isnan(got1[:, n1:].float()).all()   # ldo padding untouched
    assert torch.equal(got2, want2)
    assert torch.equal(got_other, want_other)
    sk.close()
    other.close()


def test_static_apply_scatter_kind_uses_the_array_as_accumulator():
    d, k, s, n1, n2 = 4096, 256, 4, 96, 40
    A = torch.randn((d, n1), device=DEV).to(torch.bfloat16)
    sk = B.Sketch(d, k, d, k, 1, s, seed=3, kind=B.KIND_SJLT_SCATTER)
    ref = O.apply(O.build_csc(O.Params(d, k, d, k, 1, s), 3), host64(A))
    for n in (n1, n2):                               # float atomics: order differs run to run, so compare with the oracle
        out = torch.empty((k, n), device=DEV, dtype=torch.bfloat16)
        sk.apply_static(A[:, :n], out)
        torch.cuda.synchronize()
        assert O.rel_fro_err(host64(out), ref[:, :n]) <= TOL[torch.bfloat16]
    sk.close()


def test_static_apply_rejects_what_does_not_fit_and_bad_arguments():
    cfg = W.CONFIGS["tall"]                          # 16 planes of 4096 x 256 floats = 64 MiB
    sk = B.Sketch(*cfg.params, seed=0)
    n = 256
    need = sk.plan(n, torch.float32)["workspace_bytes"]
    assert need > B.STATIC_SCRATCH_BYTES
    A = torch.zeros((cfg.d, n), device=DEV)
    out = torch.full((cfg.k, n), 7.0, device=DEV)
    with pytest.raises(B.FlashSketchError) as e:
        sk.apply_static(A, out)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert (out == 7.0).all()                        # nothing was launched
    n_fit = 64                                       # 16 planes x 4096 x 64 floats = 16 MiB
    assert sk.plan(n_fit, torch.float32)["workspace_bytes"] <= B.STATIC_SCRATCH_BYTES
    A[:, :n_fit].normal_()
    got = torch.empty((cfg.k, n_fit), device=DEV)
    sk.apply_static(A[:, :n_fit], got)
    assert torch.equal(got, sk.apply(A[:, :n_fit].contiguous()))
    L = B.lib
    p = A.data_ptr()
    assert L.fs_sketch_apply_static(None, p, n, n, out.data_ptr(), n, 0, None) == 1
    assert L.fs_sketch_apply_static(sk._h, None, n, n, out.data_ptr(), n, 0, None) == 1
    assert L.fs_sketch_apply_static(sk._h, p, n - 1, n, out.data_ptr(), n, 0, None) == 1
    assert L.fs_sketch_apply_static(sk._h, p, n, n, out.data_ptr(), n, 9, None) == 1
    assert L.fs_sketch_apply_static(sk._h, p, n, 0, out.data_ptr(), n, 0, None) == 0
    sk.close()
