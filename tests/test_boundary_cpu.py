"""Host-side logic of the C-ABI library, runnable without a GPU: the library loads, exports every symbol the
header declares, and every argument error is reported before any HIP call is made (so fake, never
dereferenced pointers are safe here: each call below must fail validation)."""
import ctypes
import os
import re
import subprocess

import pytest

from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import build as fbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
A = 0x10000  # fake 16-byte aligned "device pointers"; validation never dereferences them


@pytest.fixture(scope="module")
def lib():
    fbuild.build_library(force=False)
    return fb.load()


def shape(B=2, Hq=8, Hkv=2, d=128, dt=fb.BF16):
    return fb.Shape(B, Hq, Hkv, d, dt)


def P(x):
    return ctypes.c_void_p(x)


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "fedrag.h")).read()
    declared = set(re.findall(r"\b(fedrag_[a-z_0-9]+)\s*\(", header))
    assert declared == set(fb.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert fb.version() >= 100
    for code in range(7):
        assert fb.status_string(code) and fb.status_string(code) != "unknown status"
    assert fb.status_string(99) == "unknown status"


def test_scramble_kv_validation(lib):
    s = shape()
    f = lib.fedrag_scramble_kv
    ok_args = lambda: [ctypes.byref(s), 64, P(A), P(2 * A), P(3 * A), P(4 * A), P(5 * A), 1, P(6 * A), P(7 * A), None]
    a = ok_args(); a[0] = None
    assert f(*a) == fb.ERR_NULL
    for i in (2, 3, 4, 5, 8, 9):
        a = ok_args(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    a = ok_args(); a[1] = -1
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[7] = 3          # n_perm neither 1 nor B
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[8] = P(A)       # K_out aliases K
    assert f(*a) == fb.ERR_ALIAS
    a = ok_args(); a[9] = P(A + 256)  # V_out overlaps K
    assert f(*a) == fb.ERR_ALIAS
    a = ok_args(); a[2] = P(A + 4)   # misaligned
    assert f(*a) == fb.ERR_ALIAS
    bad = shape(Hq=6, Hkv=4); a = ok_args(); a[0] = ctypes.byref(bad)
    assert f(*a) == fb.ERR_SHAPE
    bad = shape(d=96); a = ok_args(); a[0] = ctypes.byref(bad)
    assert f(*a) == fb.ERR_UNSUPPORTED
    bad = shape(dt=7); a = ok_args(); a[0] = ctypes.byref(bad)
    assert f(*a) == fb.ERR_UNSUPPORTED


def test_scramble_q_and_unscramble_validation(lib):
    s = shape()
    assert lib.fedrag_scramble_q(ctypes.byref(s), 4, None, P(A), None, P(2 * A), None) == fb.ERR_NULL
    assert lib.fedrag_scramble_q(ctypes.byref(s), -4, P(A), P(2 * A), None, P(3 * A), None) == fb.ERR_SHAPE
    assert lib.fedrag_scramble_q(ctypes.byref(s), 4, P(A), P(2 * A), None, P(A), None) == fb.ERR_ALIAS
    assert lib.fedrag_scramble_q(ctypes.byref(s), 4, P(A), P(2 * A), P(3 * A + 2), P(4 * A), None) == fb.ERR_ALIAS
    assert lib.fedrag_unscramble(ctypes.byref(s), 4, P(A), None, None, P(2 * A), None) == fb.ERR_NULL
    assert lib.fedrag_unscramble(ctypes.byref(s), 4, P(A), P(3 * A), None, P(A + 16), None) == fb.ERR_ALIAS
    bad = shape(d=32)
    assert lib.fedrag_unscramble(ctypes.byref(bad), 4, P(A), P(3 * A), None, P(2 * A), None) == fb.ERR_UNSUPPORTED


def test_structured_calls_validation(lib):
    s = shape()
    key = fb.StructuredKey(A, 2 * A, 3 * A, 4 * A)
    kq = ctypes.byref(key)
    f = lib.fedrag_scramble_kv_structured
    ok_args = lambda: [ctypes.byref(s), 64, P(5 * A), P(6 * A), kq, kq, P(7 * A), 1, P(8 * A), P(9 * A), None]
    for i in (0, 2, 3, 4, 5, 8, 9):
        a = ok_args(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    for field in ("scale_in", "perm_in", "perm_out", "scale_out"):
        bad = fb.StructuredKey(A, 2 * A, 3 * A, 4 * A)
        setattr(bad, field, None)
        a = ok_args(); a[5] = ctypes.byref(bad)
        assert f(*a) == fb.ERR_NULL
        setattr(bad, field, A + 2)            # misaligned key array
        assert f(*a) == fb.ERR_ALIAS
    a = ok_args(); a[1] = -1
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[7] = 3
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[8] = P(5 * A)           # K_out aliases K
    assert f(*a) == fb.ERR_ALIAS
    bad = shape(d=96); a = ok_args(); a[0] = ctypes.byref(bad)
    assert f(*a) == fb.ERR_UNSUPPORTED
    g = lib.fedrag_scramble_q_structured
    assert g(ctypes.byref(s), 4, P(A), None, None, P(2 * A), None) == fb.ERR_NULL
    assert g(ctypes.byref(s), 4, None, kq, None, P(2 * A), None) == fb.ERR_NULL
    assert g(ctypes.byref(s), 4, P(5 * A), kq, None, P(5 * A), None) == fb.ERR_ALIAS
    assert g(ctypes.byref(s), -1, P(5 * A), kq, None, P(6 * A), None) == fb.ERR_SHAPE
    u = lib.fedrag_unscramble_structured
    assert u(ctypes.byref(s), 4, P(5 * A), None, None, P(6 * A), None) == fb.ERR_NULL
    assert u(ctypes.byref(s), 4, P(5 * A), kq, P(7 * A + 1), P(6 * A), None) == fb.ERR_ALIAS
    assert u(ctypes.byref(s), 4, P(5 * A), kq, None, P(5 * A + 16), None) == fb.ERR_ALIAS
    # zero rows: accepted without touching a device
    assert g(ctypes.byref(s), 0, P(5 * A), kq, None, P(6 * A), None) == fb.OK
    assert u(ctypes.byref(s), 0, P(5 * A), kq, None, P(6 * A), None) == fb.OK


def test_local_attn_and_unpermute_lse_validation(lib):
    s = shape()
    f = lib.fedrag_local_attn
    ok_args = lambda: [ctypes.byref(s), 64, 256, P(A), P(2 * A), P(3 * A), ctypes.c_float(0.1), P(4 * A), P(5 * A),
                       None, 0, None]
    for i in (0, 3, 4, 5, 7, 8):
        a = ok_args(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    a = ok_args(); a[1] = 300                 # more queries than local tokens
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[6] = ctypes.c_float(0.0)
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[3] = P(A + 8)
    assert f(*a) == fb.ERR_ALIAS
    a = ok_args(); a[1] = 1; a[2] = 1 << 20   # one decoding query over a long local cache: split path, no workspace
    assert f(*a) == fb.ERR_WORKSPACE
    a = ok_args(); a[1] = 0; a[2] = 0
    assert f(*a) == fb.OK
    u = lib.fedrag_unpermute_lse
    assert u(ctypes.byref(s), 4, None, None, P(A), None) == fb.ERR_NULL
    assert u(ctypes.byref(s), 4, P(A), None, P(A), None) == fb.ERR_ALIAS
    assert u(ctypes.byref(s), 4, P(A), P(3 * A + 2), P(2 * A), None) == fb.ERR_ALIAS
    assert u(ctypes.byref(s), -1, P(A), None, P(2 * A), None) == fb.ERR_SHAPE
    assert u(ctypes.byref(s), 0, P(A), None, P(2 * A), None) == fb.OK


def test_partial_attn_varlen_validation(lib):
    s = shape()
    f = lib.fedrag_partial_attn_varlen
    ok_args = lambda: [ctypes.byref(s), 64, 256, P(A), P(2 * A), P(3 * A), P(6 * A), None, ctypes.c_float(0.1), P(4 * A),
                       P(5 * A), None, 0, None]
    for i in (0, 3, 4, 5, 6, 9, 10):
        a = ok_args(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    a = ok_args(); a[6] = P(6 * A + 2)        # misaligned lengths
    assert f(*a) == fb.ERR_ALIAS
    a = ok_args(); a[7] = P(7 * A + 1)        # misaligned query lengths
    assert f(*a) == fb.ERR_ALIAS
    a = ok_args(); a[2] = -1
    assert f(*a) == fb.ERR_SHAPE
    a = ok_args(); a[1] = 1; a[2] = 1 << 20   # split path needs the workspace
    assert f(*a) == fb.ERR_WORKSPACE
    a = ok_args(); a[1] = 0
    assert f(*a) == fb.OK


def test_codec_validation(lib):
    for f in (lib.fedrag_quantize_rows, lib.fedrag_dequantize_rows):
        ok = lambda: [100, 128, fb.BF16, 8, P(A), P(4 * A), P(8 * A), None]
        for i in (4, 5, 6):
            a = ok(); a[i] = None
            assert f(*a) == fb.ERR_NULL
        a = ok(); a[0] = -1
        assert f(*a) == fb.ERR_SHAPE
        a = ok(); a[1] = 96
        assert f(*a) == fb.ERR_UNSUPPORTED
        a = ok(); a[3] = 5
        assert f(*a) == fb.ERR_UNSUPPORTED
        a = ok(); a[2] = 9
        assert f(*a) == fb.ERR_UNSUPPORTED
        a = ok(); a[6] = P(8 * A + 4)          # params need 8-byte alignment
        assert f(*a) == fb.ERR_ALIAS
        a = ok(); a[5] = P(A + 256)            # codes inside X
        assert f(*a) == fb.ERR_ALIAS
        a = ok(); a[0] = 0
        assert f(*a) == fb.OK


def test_scramble_kv_quantized_validation(lib):
    s = shape()
    f = lib.fedrag_scramble_kv_quantized
    ok = lambda: [ctypes.byref(s), 64, P(A), P(2 * A), P(3 * A), P(4 * A), P(5 * A), 1, 8, P(6 * A), P(7 * A), P(8 * A),
                  P(9 * A), None]
    for i in (0, 2, 3, 4, 5, 9, 10, 11, 12):
        a = ok(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    a = ok(); a[8] = 6
    assert f(*a) == fb.ERR_UNSUPPORTED
    s32 = shape(dt=fb.F32); a = ok(); a[0] = ctypes.byref(s32)
    assert f(*a) == fb.ERR_UNSUPPORTED
    a = ok(); a[9] = P(A)                       # codes over the input
    assert f(*a) == fb.ERR_ALIAS
    a = ok(); a[11] = P(6 * A)                  # both code buffers the same
    assert f(*a) == fb.ERR_ALIAS
    a = ok(); a[10] = P(7 * A + 4)              # params need 8-byte alignment
    assert f(*a) == fb.ERR_ALIAS
    a = ok(); a[7] = 3
    assert f(*a) == fb.ERR_SHAPE
    key = fb.StructuredKey(A, 2 * A, 3 * A, 4 * A)
    g = lib.fedrag_scramble_kv_structured_quantized
    okg = lambda: [ctypes.byref(s), 64, P(10 * A), P(11 * A), ctypes.byref(key), ctypes.byref(key), None, 0, 4,
                   P(6 * A), P(7 * A), P(8 * A), P(9 * A), None]
    a = okg(); a[4] = None
    assert g(*a) == fb.ERR_NULL
    a = okg(); a[8] = 16
    assert g(*a) == fb.ERR_UNSUPPORTED
    a = okg(); a[1] = 0
    assert g(*a) == fb.OK


def test_partial_attn_validation_and_workspace(lib):
    s = shape(B=16, Hq=32, Hkv=8)
    need = lib.fedrag_partial_attn_workspace_bytes(ctypes.byref(s), 1, 8192)
    assert need > 0 and need % 4 == 0
    f = lib.fedrag_partial_attn
    base = lambda: [ctypes.byref(s), 1, 8192, P(A), P(2 * A), P(3 * A), ctypes.c_float(0.088), P(4 * A), P(5 * A),
                    P(6 * A), need, None]
    a = base(); a[10] = need - 1
    assert f(*a) == fb.ERR_WORKSPACE
    a = base(); a[9] = None
    assert f(*a) == fb.ERR_WORKSPACE
    a = base(); a[3] = None
    assert f(*a) == fb.ERR_NULL
    a = base(); a[4] = None
    assert f(*a) == fb.ERR_NULL
    a = base(); a[7] = None
    assert f(*a) == fb.ERR_NULL
    a = base(); a[2] = -5
    assert f(*a) == fb.ERR_SHAPE
    for bad_scale in (float("nan"), float("inf"), 0.0, -0.1):
        a = base(); a[6] = ctypes.c_float(bad_scale)
        assert f(*a) == fb.ERR_SHAPE
    a = base(); a[3] = P(A + 8)
    assert f(*a) == fb.ERR_ALIAS
    # workspace query: prefill-shaped and fp32 problems need none; bad shapes report 0
    assert lib.fedrag_partial_attn_workspace_bytes(ctypes.byref(s), 2048, 16384) == 0
    s32 = shape(dt=fb.F32)
    assert lib.fedrag_partial_attn_workspace_bytes(ctypes.byref(s32), 1, 8192) == 0
    assert lib.fedrag_partial_attn_workspace_bytes(ctypes.byref(shape(d=100)), 1, 8192) == 0
    # splits x rows x (d + 1) floats
    rows = 16 * 32
    assert need % (rows * 129 * 4) == 0 and 2 <= need // (rows * 129 * 4) <= 64


def test_merge_and_invert_perm_validation(lib):
    s = shape()
    f = lib.fedrag_lse_merge
    assert f(ctypes.byref(s), 1, 0, P(A), P(2 * A), P(3 * A), P(4 * A), None) == fb.ERR_SHAPE
    assert f(ctypes.byref(s), 1, 2, None, P(2 * A), P(3 * A), P(4 * A), None) == fb.ERR_NULL
    assert f(ctypes.byref(s), 1, 2, P(A), P(2 * A), P(A), P(4 * A), None) == fb.ERR_ALIAS
    assert f(ctypes.byref(s), 1, 2, P(A), P(2 * A), P(3 * A), P(2 * A), None) == fb.ERR_ALIAS
    g = lib.fedrag_invert_perm
    assert g(None, 4, P(A), None) == fb.ERR_NULL
    assert g(P(A), -1, P(2 * A), None) == fb.ERR_SHAPE
    assert g(P(A), 8, P(A + 16), None) == fb.ERR_ALIAS


def test_zero_sized_problems_are_ok_without_a_device(lib):
    # nothing to do: returns OK before any launch
    s = shape(B=0)
    assert lib.fedrag_scramble_q(ctypes.byref(s), 4, P(A), P(2 * A), None, P(3 * A), None) == fb.OK
    s = shape()
    assert lib.fedrag_scramble_q(ctypes.byref(s), 0, P(A), P(2 * A), None, P(3 * A), None) == fb.OK
    assert lib.fedrag_invert_perm(P(A), 0, P(2 * A), None) == fb.OK


def test_binding_refuses_cpu_tensors(lib):
    import torch
    q = torch.zeros(1, 2, 1, 64)
    with pytest.raises(ValueError):
        fb.fedrag_scramble_q(q, torch.zeros(2, 64, 64))


def test_workspace_size_of_prefill_shapes(lib):
    """Few query tiles and many keys: the keys are cut into runs, the workspace holds one fp32 partial per run
    (256 compute units assumed without a GPU).  Enough query tiles to fill the chip: no workspace."""
    def need(B, Hq, Hkv, d, Lq, L, dt=fb.BF16):
        s = fb.make_shape(B, Hq, Hkv, d, dt)
        return int(lib.fedrag_partial_attn_workspace_bytes(ctypes.byref(s), Lq, L))
    # 8 KV heads x 2 tiles of the 4 x 128 rows of a group = 16 workgroups, 64 tiles -> 16 runs of 4 tiles
    assert need(1, 32, 8, 128, 128, 4096) == 16 * 32 * 128 * (128 + 1) * 4
    # 2 workgroups, 24 tiles -> runs of at least 4 tiles -> 6 runs
    assert need(1, 4, 2, 128, 70, 1500) == 6 * 4 * 70 * (128 + 1) * 4
    # fewer than 8 tiles: one run
    assert need(1, 4, 2, 128, 70, 256) == 0
    # the prefill benchmark shape (256 workgroups) and fp32 storage: no runs
    assert need(1, 32, 8, 128, 2048, 16384) == 0
    assert need(1, 4, 2, 128, 70, 1500, fb.F32) == 0


def test_partial_attn_shards_validation_and_workspace(lib):
    s = shape(B=1, Hq=32, Hkv=8)
    n = 2
    Ls = (ctypes.c_int64 * n)(4096, 4096)
    Kp = (ctypes.c_void_p * n)(2 * A, 3 * A)
    Vp = (ctypes.c_void_p * n)(4 * A, 5 * A)
    need = lib.fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(s), 1, n, Ls)
    # 8 units, 256 compute units: 32 runs of 256 keys wanted, a run is at least 512 keys: 8 runs per shard
    assert need == 16 * 32 * (128 + 1) * 4
    # the same keys as one shard: the same number of runs
    one = (ctypes.c_int64 * 1)(8192)
    assert lib.fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(s), 1, 1, one) == \
        lib.fedrag_partial_attn_workspace_bytes(ctypes.byref(s), 1, 8192) == need
    f = lib.fedrag_partial_attn_shards
    base = lambda: [ctypes.byref(s), 1, n, Ls, Kp, Vp, P(A), ctypes.c_float(0.088), P(6 * A), P(7 * A), P(8 * A), need,
                    None]
    for i in (3, 4, 5, 6, 8, 9):
        a = base(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    a = base(); a[2] = 0
    assert f(*a) == fb.ERR_SHAPE
    a = base(); a[2] = 17
    assert f(*a) == fb.ERR_SHAPE
    a = base(); a[11] = need - 1
    assert f(*a) == fb.ERR_WORKSPACE
    a = base(); a[10] = None
    assert f(*a) == fb.ERR_WORKSPACE
    a = base(); a[3] = (ctypes.c_int64 * n)(4096, -1)
    assert f(*a) == fb.ERR_SHAPE
    a = base(); a[4] = (ctypes.c_void_p * n)(2 * A, None)     # a non-empty shard without keys
    assert f(*a) == fb.ERR_NULL
    a = base(); a[5] = (ctypes.c_void_p * n)(4 * A, 5 * A + 4)
    assert f(*a) == fb.ERR_ALIAS
    for bad_scale in (float("nan"), 0.0):
        a = base(); a[7] = ctypes.c_float(bad_scale)
        assert f(*a) == fb.ERR_SHAPE
    # prefill shape with enough query tiles for the chip: one run and one partial per shard
    assert lib.fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(s), 4096, n, Ls) == n * 32 * 4096 * (128 + 1) * 4
    # bad arguments report 0 bytes
    assert lib.fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(s), 1, 17, Ls) == 0
    assert lib.fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(s), 1, n, None) == 0


def test_unscramble_merge_validation(lib):
    s = shape(B=1, Hq=4, Hkv=2)
    f = lib.fedrag_unscramble_merge
    base = lambda: [ctypes.byref(s), 8, P(A), P(2 * A), P(3 * A), None, P(4 * A), P(5 * A), P(6 * A), P(7 * A), None]
    for i in (2, 3, 4, 6, 7, 8, 9):
        a = base(); a[i] = None
        assert f(*a) == fb.ERR_NULL
    a = base(); a[1] = -1
    assert f(*a) == fb.ERR_SHAPE
    a = base(); a[8] = P(A)            # output on top of the scrambled input
    assert f(*a) == fb.ERR_ALIAS
    a = base(); a[8] = P(4 * A)        # output on top of the local partial
    assert f(*a) == fb.ERR_ALIAS
    a = base(); a[9] = P(5 * A)        # log-sum-exp output on top of the local one
    assert f(*a) == fb.ERR_ALIAS
    a = base(); a[9] = P(7 * A + 2)    # misaligned
    assert f(*a) == fb.ERR_ALIAS


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message that says so (no GPU needed)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr


def test_header_is_plain_c_and_links(tmp_path):
    """include/fedrag.h compiles as C99 with a C compiler, and a C program linked against the library runs its
    host-side paths (no GPU needed)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    from paper_2605_25716_amd import build as fbuild
    lib_dir = os.path.dirname(fbuild.LIB_PATH)
    exe = str(tmp_path / "abi_check")
    cmd = [gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(root, "include"),
           os.path.join(root, "tests", "c", "abi_check.c"), "-o", exe, "-L", lib_dir, "-lfedrag",
           "-Wl,-rpath," + lib_dir, "-Wl,-rpath,/opt/rocm/lib"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, f"exit {r.returncode}: {r.stdout} {r.stderr}"
    assert "abi ok" in r.stdout


def test_host_paths_under_address_and_undefined_behaviour_sanitizers():
    """The host side of every entry point (argument checks, key-run planner over 20000 random shapes, workspace
    queries) with the library's host code built under ASan + UBSan; the C driver makes no call that could reach a
    kernel launch, so this runs without a GPU.  A sanitizer report ends the program with a non-zero status."""
    from paper_2605_25716_amd import build as fbuild
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = fbuild.build_host_check(os.path.join(root, "tests", "c", "host_paths.c"))
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, f"host_paths under sanitizers failed:\n{res.stdout[-3000:]}\n{res.stderr[-3000:]}"
    assert "host paths ok" in res.stdout


def test_missing_library_fails_loudly(tmp_path):
    """There is no fallback path: with no built library the binding raises instead of computing something else."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r)\n"
        "from paper_2605_25716_amd import build as b\n"
        "b.LIB_PATH = %r\n"
        "from paper_2605_25716_amd import binding as fb\n"
        "try:\n"
        "    fb.load()\n"
        "except FileNotFoundError as e:\n"
        "    print('raised:', e); sys.exit(0)\n"
        "sys.exit(3)\n" % (root, str(tmp_path / "libfedrag_absent.so")))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "no fallback" in r.stdout


def test_product_and_oracle_do_not_reach_into_each_other():
    """The HIP path and the oracle share no code: the package never imports, loads or names anything under oracle/
    (the input generators only mention it in comments), and the oracle never names the package or its library."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2605_25716_amd")
    bad = []
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if not f.endswith((".py", ".hip", ".h")):
                continue
            text = open(os.path.join(dirpath, f), encoding="utf-8").read()
            if re.search(r"^\s*(import|from)\s+oracle\b", text, re.M) or "libfedrag_oracle" in text or "oracle/" in text:
                bad.append(os.path.join(dirpath, f))
    for f in os.listdir(os.path.join(root, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(root, "oracle", f), encoding="utf-8").read()
            if "paper_2605_25716_amd" in text or "libfedrag.so" in text or "fedrag.h" in text:
                bad.append(os.path.join("oracle", f))
    assert not bad, bad


def test_calls_without_rows_accept_null_tensors(lib):
    """A call whose output has no rows returns FEDRAG_OK at once; its tensor pointers may be NULL."""
    s = shape(B=2, Hq=8, Hkv=2)
    z = ctypes.c_float(0.088)
    assert lib.fedrag_scramble_q(ctypes.byref(s), 0, None, None, None, None, None) == fb.OK
    assert lib.fedrag_scramble_kv(ctypes.byref(s), 0, None, None, None, None, None, 1, None, None, None) == fb.OK
    assert lib.fedrag_partial_attn(ctypes.byref(s), 0, 100, None, None, None, z, None, None, None, 0, None) == fb.OK
    assert lib.fedrag_local_attn(ctypes.byref(s), 0, 100, None, None, None, z, None, None, None, 0, None) == fb.OK
    assert lib.fedrag_lse_merge(ctypes.byref(s), 0, 3, None, None, None, None, None) == fb.OK
    assert lib.fedrag_unscramble(ctypes.byref(s), 0, None, None, None, None, None) == fb.OK
    assert lib.fedrag_unscramble_merge(ctypes.byref(s), 0, None, None, None, None, None, None, None, None, None) == fb.OK
    # with rows the same pointers are refused
    assert lib.fedrag_scramble_q(ctypes.byref(s), 1, None, None, None, None, None) == fb.ERR_NULL
    assert lib.fedrag_unscramble(ctypes.byref(s), 1, None, None, None, None, None) == fb.ERR_NULL


def test_probe_library_exports_and_refuses_bad_arguments():
    """The rate probes bench.py reports as `achievable` live in a library of their own; without a device only the
    host-side argument checks can run (a refused call launches nothing)."""
    if not os.path.exists(fbuild.PROBES_LIB):
        fbuild.build_probes(force=True)
    p = ctypes.CDLL(fbuild.PROBES_LIB)
    for name in ("fedrag_probe_copy", "fedrag_probe_read", "fedrag_probe_mfma_bf16", "fedrag_probe_mfma_bf16_random",
                 "fedrag_probe_mfma_bf16_flop"):
        assert hasattr(p, name), name
    vp = ctypes.c_void_p
    p.fedrag_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    p.fedrag_probe_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    p.fedrag_probe_mfma_bf16.argtypes = [vp, ctypes.c_int, vp]
    p.fedrag_probe_mfma_bf16_random.argtypes = [vp, ctypes.c_int, vp]
    p.fedrag_probe_mfma_bf16_flop.argtypes = [ctypes.c_int]
    p.fedrag_probe_mfma_bf16_flop.restype = ctypes.c_double
    assert p.fedrag_probe_copy(None, None, 1024, None) == 1
    assert p.fedrag_probe_copy(vp(0x1000), vp(0x2000), 1000, None) == 1      # not a multiple of 16
    assert p.fedrag_probe_copy(vp(0x1008), vp(0x2000), 1024, None) == 1      # misaligned
    assert p.fedrag_probe_read(None, 1024, vp(0x1000), None) == 1
    assert p.fedrag_probe_mfma_bf16(None, 16, None) == 1
    assert p.fedrag_probe_mfma_bf16_random(vp(0x1000), 0, None) == 1
    # 256 workgroups x 8 waves x iters x 8 MFMAs of 2 * 32 * 32 * 16 flop
    assert p.fedrag_probe_mfma_bf16_flop(3) == 256 * 8 * 3 * 8 * 2.0 * 32 * 32 * 16


def test_bench_means_leave_out_stalls():
    """bench.py's per-call mean: a sample beyond three medians (a stall of the host or the box between the two event
    records) is left out and counted; the median is taken over everything."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)

    class Ev:
        def __init__(self, t):
            self.t = t

        def elapsed_time(self, other):
            return other.t - self.t

    timer = bench.CallTimer(torch=None)
    ms = [0.086] * 19 + [25.0]            # 19 calls of 86 us and one that spans a 25 ms stall
    timer.pairs["partial_attn"] = [(Ev(0.0), Ev(x)) for x in ms]
    timer.pairs["clean"] = [(Ev(0.0), Ev(0.190 + 0.001 * (i % 3))) for i in range(20)]
    s = timer.summary()
    assert s["partial_attn"]["stalls_left_out"] == 1 and abs(s["partial_attn"]["avg_us"] - 86.0) < 1e-6
    assert abs(s["partial_attn"]["med_us"] - 86.0) < 1e-6 and abs(s["partial_attn"]["max_us"] - 25000.0) < 1e-6
    assert s["clean"]["stalls_left_out"] == 0 and 190.0 <= s["clean"]["avg_us"] <= 192.0
