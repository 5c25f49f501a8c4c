"""Builds the C-ABI library (libfedrag.so) for gfx950 with hipcc, in-tree.

Every source is compiled to an object of its own (in parallel) under `_build/` and the objects are linked into the
shared library; force=False recompiles only the sources that are newer than their objects."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ_DIR = os.path.join(_HERE, "_build")
LIB_PATH = os.path.join(_HERE, "libfedrag.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 arithmetic is kept off for the device code (scalar fp32 ops only)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]
_NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(_HERE, "..", "include", "*.h"))


def _obj_of(src: str) -> str:
    return os.path.join(OBJ_DIR, os.path.splitext(os.path.basename(src))[0] + ".o")


def _obj_stale(src: str) -> bool:
    obj = _obj_of(src)
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    return any(os.path.getmtime(p) > t for p in [src] + _headers())


def is_stale() -> bool:
    if not os.path.exists(LIB_PATH):
        return True
    t = os.path.getmtime(LIB_PATH)
    return any(os.path.getmtime(p) > t for p in sources() + _headers())


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if _NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)


def build_library(force: bool = True, verbose: bool = False, extra_flags=(), jobs: int = 8) -> str:
    """Compile every HIP source and link libfedrag.so.  force=False skips objects (and the link) that are newer
    than their sources and headers."""
    if not force and not is_stale():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    todo = [s for s in sources() if force or extra_flags or _obj_stale(s)]
    cmds = [[hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-c", s, "-o", _obj_of(s)] for s in todo]
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(cmds) or 1))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + [_obj_of(s) for s in sources()],
         verbose)
    return LIB_PATH


if __name__ == "__main__":
    import sys
    print(build_library(force="--incremental" not in sys.argv, verbose=True))
