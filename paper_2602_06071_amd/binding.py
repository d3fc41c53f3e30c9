"""ctypes binding of include/flashsketch.h: same names, argument marshalling only.

PyTorch supplies device memory (``tensor.data_ptr()``) and the HIP stream
(``torch.cuda.current_stream().cuda_stream``); nothing is computed here.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # must precede the CDLL: the library binds to the HIP runtime torch has loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.environ.get("FLASHSKETCH_LIB") or os.path.join(_HERE, "libflashsketch.so")

FS_F32, FS_BF16, FS_F16 = 0, 1, 2
KIND_BLOCKPERM, KIND_SJLT_SCATTER, KIND_GAUSS_DENSE, KIND_BLOCKROW = 0, 1, 2, 3
VARIANT_AUTO, VARIANT_GENERIC, VARIANT_MFMA = 0, 1, 2

SYMBOLS = [
    "fs_sketch_create", "fs_sketch_create_kind", "fs_sketch_apply", "fs_sketch_apply_ld",
    "fs_sketch_export", "fs_sketch_export_dense", "fs_sketch_info", "fs_sketch_workspace_bytes",
    "fs_sketch_set_workspace", "fs_sketch_set_variant", "fs_sketch_destroy", "fs_status_string",
    "fs_sketch_profile_begin", "fs_sketch_profile_end",
    "fs_sketch_apply_rows", "fs_sketch_rows_workspace_bytes", "fs_sketch_plan", "fs_sketch_prepare",
    "fs_sketch_apply_static",
]
STATIC_SCRATCH_BYTES = 32 << 20
PROFILE_KERNEL, PROFILE_APPLY = 1, 2
PLAN_ELEMENT_LOADS, PLAN_ROW_SLICES, PLAN_SLOT_GROUPS, PLAN_SPLIT, PLAN_STACKED = 1, 2, 4, 8, 16


class FlashSketchError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {lib.fs_status_string(status).decode()} (fs_status {status})")


class fs_info(C.Structure):
    _fields_ = [
        ("d", C.c_int64), ("k", C.c_int64),
        ("Bc", C.c_int32), ("Br", C.c_int32), ("kappa", C.c_int32), ("s", C.c_int32),
        ("M", C.c_int32), ("a", C.c_int32), ("b", C.c_int32), ("a_inv", C.c_int32),
        ("key0", C.c_uint32), ("key1", C.c_uint32),
        ("scale", C.c_float),
        ("kind", C.c_int32), ("variant", C.c_int32), ("last_variant", C.c_int32), ("last_mode", C.c_int32),
        ("last_hip_error", C.c_int32),
        ("workspace_bytes", C.c_uint64),
        ("last_kernel", C.c_char * 64),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(lib_path):
        raise ImportError(
            f"{lib_path} is missing: build it with `python -m paper_2602_06071_amd.build` "
            "(there is no CPU fallback)")
    L = C.CDLL(lib_path)
    vp, i64, i32, u64 = C.c_void_p, C.c_int64, C.c_int32, C.c_uint64
    L.fs_sketch_create.argtypes = [C.POINTER(vp), i64, i64, i32, i32, i32, i32, u64]
    L.fs_sketch_create_kind.argtypes = [C.POINTER(vp), C.c_int, i64, i64, i32, i32, i32, i32, u64]
    L.fs_sketch_apply.argtypes = [vp, vp, i64, i64, vp, C.c_int, vp]
    L.fs_sketch_apply_ld.argtypes = [vp, vp, i64, i64, vp, i64, C.c_int, vp]
    L.fs_sketch_apply_static.argtypes = [vp, vp, i64, i64, vp, i64, C.c_int, vp]
    L.fs_sketch_apply_rows.argtypes = [vp, vp, i64, i64, vp, i64, C.c_int, vp]
    L.fs_sketch_rows_workspace_bytes.argtypes = [vp, i64, C.c_int, C.POINTER(C.c_size_t)]
    i32p = C.POINTER(C.c_int32)
    L.fs_sketch_plan.argtypes = [vp, vp, i64, i64, C.c_int, C.c_int32, i32p, i32p, i32p, C.POINTER(C.c_size_t)]
    L.fs_sketch_export.argtypes = [vp, vp, vp, vp]
    L.fs_sketch_export_dense.argtypes = [vp, vp, vp]
    L.fs_sketch_info.argtypes = [vp, C.POINTER(fs_info)]
    L.fs_sketch_workspace_bytes.argtypes = [vp, i64, C.c_int, C.POINTER(C.c_size_t)]
    L.fs_sketch_set_workspace.argtypes = [vp, vp, C.c_size_t]
    L.fs_sketch_set_variant.argtypes = [vp, C.c_int]
    L.fs_sketch_destroy.argtypes = [vp]
    L.fs_sketch_profile_begin.argtypes = [vp, i32, i32]
    L.fs_sketch_profile_end.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(i32)]
    L.fs_sketch_prepare.argtypes = [vp, vp]
    for name in SYMBOLS:
        getattr(L, name).restype = C.c_int
    L.fs_status_string.argtypes = [C.c_int]
    L.fs_status_string.restype = C.c_char_p
    return L


lib = _load()


def _check(st: int, what: str) -> None:
    if st != 0:
        raise FlashSketchError(st, what)


_DTYPE_CODES = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FS_F32
    if t.dtype == torch.bfloat16:
        return FS_BF16
    if t.dtype == torch.float16:
        return FS_F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


_deferred: list = []  # handles whose destruction was postponed (see Sketch.__del__)


def _capturing() -> bool:
    try:
        return torch.cuda.is_available() and torch.cuda.is_current_stream_capturing()
    except Exception:
        return False


def _flush_deferred() -> None:
    if _deferred and not _capturing():
        while _deferred:
            lib.fs_sketch_destroy(_deferred.pop())


class Sketch:
    """Owns one fs_sketch_t.  Methods map one-to-one onto the C entry points."""

    def __init__(self, d, k, Bc, Br, kappa, s, seed=0, kind=KIND_BLOCKPERM):
        self._h = C.c_void_p()
        _flush_deferred()
        _check(lib.fs_sketch_create_kind(C.byref(self._h), kind, d, k, Bc, Br, kappa, s, seed),
               "fs_sketch_create_kind")
        self.d, self.k = d, k
        self._ws_keepalive = None

    def close(self) -> None:
        """Destroy the handle (frees its device memory).  Also flushes handles whose destruction
        the garbage collector had to postpone."""
        _flush_deferred()
        if self._h:
            lib.fs_sketch_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        # Freeing device memory is not allowed while a stream is being captured into a HIP graph
        # (it invalidates the capture), and the garbage collector may run at any time: if a
        # capture is under way the handle is parked and destroyed by the next close() / Sketch().
        try:
            if self._h:
                if _capturing():
                    _deferred.append(self._h)
                    self._h = C.c_void_p()
                else:
                    self.close()
        except Exception:  # interpreter shutdown: modules may already be gone
            pass

    def info(self) -> fs_info:
        out = fs_info()
        _check(lib.fs_sketch_info(self._h, C.byref(out)), "fs_sketch_info")
        return out

    def set_variant(self, v: int) -> None:
        _check(lib.fs_sketch_set_variant(self._h, v), "fs_sketch_set_variant")

    def workspace_bytes(self, n: int, dtype: torch.dtype) -> int:
        out = C.c_size_t()
        code = _DTYPE_CODES[dtype]
        _check(lib.fs_sketch_workspace_bytes(self._h, n, code, C.byref(out)), "fs_sketch_workspace_bytes")
        return out.value

    def set_workspace(self, buf: torch.Tensor | None) -> None:
        if buf is None:
            _check(lib.fs_sketch_set_workspace(self._h, None, 0), "fs_sketch_set_workspace")
        else:
            _check(lib.fs_sketch_set_workspace(self._h, buf.data_ptr(), buf.numel() * buf.element_size()),
                   "fs_sketch_set_workspace")
        self._ws_keepalive = buf

    def profile_begin(self, max_launches: int, scope: int = PROFILE_KERNEL | PROFILE_APPLY) -> None:
        self._prof_cap = max_launches
        _check(lib.fs_sketch_profile_begin(self._h, max_launches, scope), "fs_sketch_profile_begin")

    def profile_end(self, whole: bool = False):
        """Milliseconds of each bracketed dominant-kernel launch since profile_begin; with
        `whole`, also of each whole apply (everything it enqueued): (kernel_ms, apply_ms)."""
        ms = (C.c_float * self._prof_cap)()
        ms_apply = (C.c_float * self._prof_cap)()
        cnt = C.c_int32()
        _check(lib.fs_sketch_profile_end(self._h, ms, ms_apply, C.byref(cnt)), "fs_sketch_profile_end")
        kernel = [float(ms[i]) for i in range(cnt.value)]
        if whole:
            return kernel, [float(ms_apply[i]) for i in range(cnt.value)]
        return kernel

    def prepare(self, stream=None) -> None:
        _check(lib.fs_sketch_prepare(self._h, _stream_ptr(stream)), "fs_sketch_prepare")

    def apply(self, A: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        """out = S @ A for a 2-D row-major view A (unit column stride)."""
        if A.dim() != 2 or A.shape[0] != self.d or A.stride(1) != 1 and A.shape[1] > 1:
            raise ValueError("A must be d x n with contiguous rows")
        n = A.shape[1]
        if out is None:
            out = torch.empty((self.k, n), dtype=A.dtype, device=A.device)
        if out.shape != (self.k, n) or out.dtype != A.dtype or (out.stride(1) != 1 and n > 1):
            raise ValueError("out must be k x n, same dtype, contiguous rows")
        _check(lib.fs_sketch_apply_ld(self._h, A.data_ptr(), A.stride(0), n, out.data_ptr(),
                                      out.stride(0), _dtype_code(A), _stream_ptr(stream)),
               "fs_sketch_apply_ld")
        return out

    def apply_static(self, A: torch.Tensor, out: torch.Tensor, stream=None) -> torch.Tensor:
        """out = S @ A through fs_sketch_apply_static (no allocation: out must be given)."""
        if A.dim() != 2 or A.shape[0] != self.d or A.stride(1) != 1 and A.shape[1] > 1:
            raise ValueError("A must be d x n with contiguous rows")
        n = A.shape[1]
        if out.shape != (self.k, n) or out.dtype != A.dtype or (out.stride(1) != 1 and n > 1):
            raise ValueError("out must be k x n, same dtype, contiguous rows")
        _check(lib.fs_sketch_apply_static(self._h, A.data_ptr(), A.stride(0), n, out.data_ptr(),
                                          out.stride(0), _dtype_code(A), _stream_ptr(stream)),
               "fs_sketch_apply_static")
        return out

    def apply_rows(self, G: torch.Tensor, out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
        """out (n x k) = G @ S^T for a 2-D row-major G (n x d, unit column stride): every row of G
        is one vector to sketch."""
        if G.dim() != 2 or G.shape[1] != self.d or G.stride(1) != 1:
            raise ValueError("G must be n x d with contiguous rows")
        n = G.shape[0]
        if out is None:
            out = torch.empty((n, self.k), dtype=G.dtype, device=G.device)
        if out.shape != (n, self.k) or out.dtype != G.dtype or out.stride(1) != 1:
            raise ValueError("out must be n x k, same dtype, contiguous rows")
        _check(lib.fs_sketch_apply_rows(self._h, G.data_ptr(), G.stride(0) if n > 1 else max(G.stride(0), self.d),
                                        n, out.data_ptr(), out.stride(0) if n > 1 else max(out.stride(0), self.k),
                                        _dtype_code(G), _stream_ptr(stream)),
               "fs_sketch_apply_rows")
        return out

    def plan(self, n: int, dtype: torch.dtype, ld: int | None = None, rows: bool = False,
             address: int = 256) -> dict:
        """Which kernel an apply of n vectors would launch (host-only; nothing runs).  `ld` is the
        leading dimension (default: packed), `address` stands for the data pointer: only its
        alignment matters."""
        if ld is None:
            ld = self.d if rows else n
        v, m, f, w = C.c_int32(), C.c_int32(), C.c_int32(), C.c_size_t()
        _check(lib.fs_sketch_plan(self._h, C.c_void_p(address), ld, n, _DTYPE_CODES[dtype], int(rows),
                                  C.byref(v), C.byref(m), C.byref(f), C.byref(w)), "fs_sketch_plan")
        return {"variant": v.value, "mode": m.value, "flags": f.value, "workspace_bytes": w.value}

    def rows_workspace_bytes(self, n: int, dtype: torch.dtype) -> int:
        out = C.c_size_t()
        code = _DTYPE_CODES[dtype]
        _check(lib.fs_sketch_rows_workspace_bytes(self._h, n, code, C.byref(out)),
               "fs_sketch_rows_workspace_bytes")
        return out.value

    def export(self, device="cuda", stream=None):
        i = self.info()
        lead = i.k if i.kind == KIND_BLOCKROW else i.d  # BLOCKROW is stored by output row
        nnz = lead * i.kappa * i.s
        rows = torch.empty(nnz, dtype=torch.int32, device=device)
        signs = torch.empty(nnz, dtype=torch.int8, device=device)
        _check(lib.fs_sketch_export(self._h, rows.data_ptr(), signs.data_ptr(), _stream_ptr(stream)),
               "fs_sketch_export")
        return rows.view(lead, i.kappa * i.s), signs.view(lead, i.kappa * i.s)

    def export_dense(self, device="cuda", stream=None) -> torch.Tensor:
        S = torch.empty((self.k, self.d), dtype=torch.float32, device=device)
        _check(lib.fs_sketch_export_dense(self._h, S.data_ptr(), _stream_ptr(stream)),
               "fs_sketch_export_dense")
        return S
