"""Builds libkvp.so (hand-written HIP for gfx950) in-tree with hipcc.

Every csrc/*.hip becomes one object under _build/ (compiled in parallel, recompiled when the file or
any header is newer; `force` recompiles everything), then the objects are linked into libkvp.so.
"""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libkvp.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fno-fast-math", "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def headers():
    return sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(ROOT, "include", "kvp.h")]


def _newer(path: str, than: float) -> bool:
    return os.path.getmtime(path) > than


def build_library(verbose: bool = False, force: bool = True, jobs: int = 8) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        stale = force or not os.path.exists(obj)
        if not stale:
            t = os.path.getmtime(obj)
            stale = _newer(src, t) or any(_newer(h, t) for h in headers())
        if stale:
            todo.append([hipcc, *HIPCC_FLAGS, *inc, "-c", "-o", obj, src])

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)

    with ThreadPoolExecutor(max_workers=max(1, min(jobs, os.cpu_count() or 1))) as ex:
        list(ex.map(run, todo))
    if todo or not os.path.exists(LIB):
        run([hipcc, *HIPCC_FLAGS, "-shared", "-o", LIB, *objs])
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(_newer(d, t) for d in sources() + headers())


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True, force="--force" in sys.argv))
