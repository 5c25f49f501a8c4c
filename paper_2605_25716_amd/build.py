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


PROBES_SRC = os.path.join(CSRC, "probes", "rate_probes.hip")
PROBES_LIB = os.path.join(_HERE, "libfedrag_probes.so")


def build_probes(force: bool = True, verbose: bool = False) -> str:
    """The reference-rate kernels of bench.py (plain copy, plain read, bare MFMA loop) as a library of their own."""
    if not force and os.path.exists(PROBES_LIB) and os.path.getmtime(PROBES_LIB) >= os.path.getmtime(PROBES_SRC):
        return PROBES_LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    _run([hipcc] + HIPCC_FLAGS + ["-shared", "-o", PROBES_LIB, PROBES_SRC], verbose)
    return PROBES_LIB


SAN_DIR = os.path.join(OBJ_DIR, "san")
SAN_FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer",
             # host code only: each -fsanitize= goes directly behind an -Xarch_host (the device side has no sanitizer)
             "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined"]


def build_host_check(c_driver: str, force: bool = False, verbose: bool = False, jobs: int = 8) -> str:
    """The library's sources with their HOST code under AddressSanitizer + UndefinedBehaviorSanitizer, linked with a
    C driver into one executable (returned path).  Used by the CPU tests to walk the argument checks, the key-run
    planner and the workspace queries; the driver makes no call that reaches a kernel launch."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    os.makedirs(SAN_DIR, exist_ok=True)
    exe = os.path.join(SAN_DIR, os.path.splitext(os.path.basename(c_driver))[0])
    deps = sources() + _headers() + [c_driver, os.path.abspath(__file__)]
    if not force and os.path.exists(exe) and all(os.path.getmtime(d) <= os.path.getmtime(exe) for d in deps):
        return exe
    obj = lambda s_: os.path.join(SAN_DIR, os.path.splitext(os.path.basename(s_))[0] + ".o")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + SAN_FLAGS
    cmds = [[hipcc] + flags + ["-c", s_, "-o", obj(s_)] for s_ in sources()]
    include = os.path.join(_HERE, "..", "include")
    cmds.append([clang, "-std=c99", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-I", include, "-c", c_driver, "-o", obj(c_driver)])
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(cmds)))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc, "--offload-arch=gfx950", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
          "-o", exe] + [obj(s_) for s_ in sources()] + [obj(c_driver)], verbose)
    return exe


if __name__ == "__main__":
    import sys
    print(build_library(force="--incremental" not in sys.argv, verbose=True))
    print(build_probes(force="--incremental" not in sys.argv, verbose=True))
