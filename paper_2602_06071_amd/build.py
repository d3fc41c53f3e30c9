"""Builds libflashsketch.so for gfx950 with hipcc, in-tree, next to this file.

    python -m paper_2602_06071_amd.build [--force] [--define NAME]... [--output PATH]

--define adds -DNAME to every compile (the kernels' FS_ABLATE_* switches); with --output the
objects go to a folder next to PATH and the library to PATH, and the in-tree library is left alone
(load such a library with FLASHSKETCH_LIB=PATH).

Each csrc/*.hip file is compiled to an object of its own (so an edit recompiles
one file) and the objects are linked into one shared library with the C ABI
declared in include/flashsketch.h.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflashsketch.so")

ARCH = "gfx950"
# Packed-fp32 VALU forms are kept off for every device translation unit.
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}", "-munsafe-fp-atomics",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _stale(src: str, obj: str, headers: list[str]) -> bool:
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(f) > t for f in [src, __file__] + headers)


def build(force: bool = False, verbose: bool = True, defines: tuple = (), output: str | None = None) -> str:
    global OBJ, LIB
    if output:
        LIB = os.path.abspath(output)
        OBJ = os.path.join(os.path.dirname(LIB), "_build")
        force = True
    os.makedirs(OBJ, exist_ok=True)
    cc = hipcc()
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(HERE, "..", "include", "flashsketch.h"))
    srcs = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    jobs = []
    for f in srcs:
        src = os.path.join(CSRC, f)
        obj = os.path.join(OBJ, f[:-4] + ".o")
        if force or _stale(src, obj, headers):
            jobs.append((src, obj))

    def compile_one(job):
        src, obj = job
        cmd = [cc, *FLAGS, *[f"-D{d}" for d in defines], "-c", src, "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        return src, r

    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        for src, r in ex.map(compile_one, jobs):
            # the host pass does not know the packed-fp32 feature name: drop that note
            err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            if verbose and (err.strip() or r.returncode):
                sys.stderr.write(err + "\n")
            if r.returncode:
                raise RuntimeError(f"hipcc failed on {src}")
            if verbose:
                print(f"[build] compiled {os.path.basename(src)}")
    objs = [os.path.join(OBJ, f[:-4] + ".o") for f in srcs]
    if jobs or not os.path.exists(LIB):
        cmd = [cc, "-shared", "-fPIC", f"--offload-arch={ARCH}", "-o", LIB, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode:
            sys.stderr.write(r.stderr)
            raise RuntimeError("link failed")
        if verbose:
            print(f"[build] linked {LIB}")
    return LIB


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser()
    ap.add_argument("--force", action="store_true")
    ap.add_argument("--define", action="append", default=[])
    ap.add_argument("--output")
    a = ap.parse_args()
    build(force=a.force, defines=tuple(a.define), output=a.output)
