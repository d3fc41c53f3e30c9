"""Choosing the block sizes (Br, Bc) of a BlockPerm-SJLT for given (d, k, kappa).

The paper treats (Br, Bc) as tuned template parameters (Appendix C, "Tuning").  This helper
encodes what the kernels of this library prefer, in that order:

  1. kappa*Br in {64, 32, 128} (in this order: measured 5-10 % apart on HBM-bound shapes, 64 also
     being the shape with the orbit-run merge): the input-stationary matrix-core path, which
     reads A once; then any other power-of-two Br with kappa*Br <= 128 (the stacked rows sit in
     a 32-, 64- or 128-row tile with its top rows idle), fullest tile first;
  2. Br in {128, 64, 32}: the output-stationary matrix-core path (A read kappa times);
  3. Br in {16, 8, 4, 2, 1} with kappa*Br > 128: input-stationary in groups of 128/Br wiring
     slots (A read once per group);
  4. any other Br dividing k, closest to 32 first.  The column-layout matrix-core kernel still
     takes it input-stationary when Br padded to the next power of two keeps kappa slots within
     128 tile rows (or Br <= 64 padded, in slot groups); otherwise the general kernel runs.  The
     path named for such a Br is what fs_sketch_plan reports for a packed 256-column call.

subject to the sketch's own constraints: Br | k, M = k/Br = ceil(d/Bc), kappa <= M, s <= Br.
For a given Br, Bc is the smallest multiple of 64 with ceil(d/Bc) = M when there is one (whole
64-row stages, aligned block starts), else ceil(d/M): the matrix-core kernels take any Bc,
the last stage of a block partly filled.  It only does integer arithmetic on shapes;
nothing here touches the sketch's hash or values.
"""
from __future__ import annotations


def _bc_for(d: int, M: int, multiple: int):
    """Smallest Bc that is a multiple of `multiple` with ceil(d / Bc) == M, or None."""
    bc = -(-d // M)                      # ceil(d / M): the smallest Bc with ceil(d/Bc) <= M
    bc = -(-bc // multiple) * multiple   # round up
    return bc if -(-d // bc) == M else None


def _planned_path(d, k, bc, br, kappa, s) -> str:
    """The path the library's dispatcher would take (host-only query; nothing is launched)."""
    import torch

    from . import binding as B
    sk = B.Sketch(d, k, bc, br, kappa, s)
    try:
        p = sk.plan(256, torch.bfloat16)
    finally:
        sk.close()
    if p["variant"] != B.VARIANT_MFMA:
        return "generic"
    if p["flags"] & B.PLAN_SLOT_GROUPS:
        return "grouped"
    return "out" if p["mode"] == 1 else "in"


def suggest_blocks(d: int, k: int, kappa: int, s: int = 2):
    """Return (Bc, Br, path) with path in {"in", "out", "grouped", "generic"}, or raise ValueError when no
    block grid satisfies the constraints (e.g. kappa > k)."""
    if min(d, k, kappa, s) < 1:
        raise ValueError("d, k, kappa, s must be positive")

    def ok(br):
        if br < s or br > 65536 or k % br:
            return False
        M = k // br
        return kappa <= M <= (1 << 24) and M <= d

    def fill(br):                        # share of the matrix-core tile the stacked rows use
        rw = kappa * br
        return rw / (32 if rw <= 32 else 64 if rw <= 64 else 128)

    exact = [r // kappa for r in (64, 32, 128) if r % kappa == 0]
    partial = sorted((b for b in (128, 64, 32, 16, 8, 4, 2, 1) if kappa * b <= 128 and b not in exact),
                     key=lambda b: (-fill(b), -b))
    grouped = [b for b in (16, 8, 4, 2, 1) if kappa * b > 128]
    for path, cands in (("in", exact + partial), ("out", [128, 64, 32]), ("grouped", grouped)):
        for br in cands:
            if br >= 1 and (br & (br - 1)) == 0 and ok(br):
                bc = _bc_for(d, k // br, 64) or _bc_for(d, k // br, 1)
                if bc is not None:
                    return bc, br, path
    for br in sorted((b for b in range(1, min(k, 65536) + 1) if k % b == 0), key=lambda b: abs(b - 32)):
        if ok(br):
            bc = _bc_for(d, k // br, 64) or _bc_for(d, k // br, 1)
            if bc is not None:
                return bc, br, _planned_path(d, k, bc, br, kappa, s)
    raise ValueError(f"no block grid for d={d}, k={k}, kappa={kappa}, s={s}")
