"""ctypes binding of the C-ABI library (include/fedrag.h), one Python function per entry point.

Argument marshalling only: tensors are torch CUDA tensors used as device memory, the stream is torch's
current HIP stream.  Every step of the path runs in the library's kernels; there is no fallback: if the
library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch  # noqa: F401  (imported before the library so that both share one HIP runtime)

from . import build as _build

OK, ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_ALIAS, ERR_DEVICE = range(7)
F32, BF16, F16 = 0, 1, 2
_DTYPES = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}

STATIC_SCRATCH_BYTES = 16 << 20  # FEDRAG_STATIC_SCRATCH_BYTES

EXPORTS = ("fedrag_scramble_kv", "fedrag_scramble_q", "fedrag_partial_attn", "fedrag_partial_attn_static",
           "fedrag_partial_attn_workspace_bytes", "fedrag_partial_attn_shards",
           "fedrag_partial_attn_shards_workspace_bytes", "fedrag_lse_merge", "fedrag_unscramble", "fedrag_unscramble_merge",
           "fedrag_scramble_kv_structured", "fedrag_scramble_q_structured", "fedrag_unscramble_structured",
           "fedrag_local_attn", "fedrag_unpermute_lse", "fedrag_partial_attn_varlen", "fedrag_quantize_rows",
           "fedrag_dequantize_rows", "fedrag_scramble_kv_quantized", "fedrag_scramble_kv_structured_quantized",
           "fedrag_partial_attn_quantized", "fedrag_partial_attn_varlen_quantized", "fedrag_invert_perm",
           "fedrag_validate_perm", "fedrag_status_string",
           "fedrag_version")


class Shape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("d_head", ctypes.c_int32), ("dtype", ctypes.c_int32)]


class StructuredKey(ctypes.Structure):
    """fedrag_structured_key: host struct of four device pointers, [Hkv, d] each."""
    _fields_ = [("scale_in", ctypes.c_void_p), ("perm_in", ctypes.c_void_p), ("perm_out", ctypes.c_void_p),
                ("scale_out", ctypes.c_void_p)]


class FedragError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib_path() -> str:
    return _build.LIB_PATH


def load() -> ctypes.CDLL:
    """Load libfedrag.so (built in-tree by paper_2605_25716_amd.build).  Raises if it is missing."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(
                f"{path} not found: build it first (python -m paper_2605_25716_amd.build); "
                "this package has no fallback path")
        lib = ctypes.CDLL(path)
        vp, i64, i32, f32p = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        sp = ctypes.POINTER(Shape)
        lib.fedrag_scramble_kv.argtypes = [sp, i64, vp, vp, vp, vp, vp, i32, vp, vp, vp]
        lib.fedrag_scramble_q.argtypes = [sp, i64, vp, vp, vp, vp, vp]
        lib.fedrag_partial_attn.argtypes = [sp, i64, i64, vp, vp, vp, ctypes.c_float, f32p, f32p, vp,
                                            ctypes.c_size_t, vp]
        lib.fedrag_local_attn.argtypes = lib.fedrag_partial_attn.argtypes
        lib.fedrag_partial_attn_static.argtypes = [sp, i64, i64, vp, vp, vp, ctypes.c_float, f32p, f32p, vp]
        lib.fedrag_partial_attn_shards.argtypes = [sp, i64, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64),
                                                   ctypes.POINTER(ctypes.c_void_p), ctypes.POINTER(ctypes.c_void_p),
                                                   vp, ctypes.c_float, f32p, f32p, vp, ctypes.c_size_t, vp]
        lib.fedrag_partial_attn_shards_workspace_bytes.argtypes = [sp, i64, ctypes.c_int32,
                                                                   ctypes.POINTER(ctypes.c_int64)]
        lib.fedrag_partial_attn_shards_workspace_bytes.restype = ctypes.c_size_t
        lib.fedrag_unscramble_merge.argtypes = [sp, i64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.fedrag_partial_attn_varlen.argtypes = [sp, i64, i64, vp, vp, vp, vp, vp, ctypes.c_float, f32p, f32p, vp,
                                                   ctypes.c_size_t, vp]
        lib.fedrag_unpermute_lse.argtypes = [sp, i64, f32p, vp, f32p, vp]
        lib.fedrag_partial_attn_workspace_bytes.argtypes = [sp, i64, i64]
        lib.fedrag_partial_attn_workspace_bytes.restype = ctypes.c_size_t
        lib.fedrag_lse_merge.argtypes = [sp, i64, i32, f32p, f32p, f32p, f32p, vp]
        lib.fedrag_unscramble.argtypes = [sp, i64, f32p, f32p, vp, f32p, vp]
        kp = ctypes.POINTER(StructuredKey)
        lib.fedrag_scramble_kv_structured.argtypes = [sp, i64, vp, vp, kp, kp, vp, i32, vp, vp, vp]
        lib.fedrag_scramble_q_structured.argtypes = [sp, i64, vp, kp, vp, vp, vp]
        lib.fedrag_unscramble_structured.argtypes = [sp, i64, f32p, kp, vp, f32p, vp]
        lib.fedrag_quantize_rows.argtypes = [i64, i32, ctypes.c_int, i32, vp, vp, vp, vp]
        lib.fedrag_dequantize_rows.argtypes = [i64, i32, ctypes.c_int, i32, vp, vp, vp, vp]
        lib.fedrag_scramble_kv_quantized.argtypes = [sp, i64, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp]
        lib.fedrag_scramble_kv_structured_quantized.argtypes = [sp, i64, vp, vp, kp, kp, vp, i32, i32, vp, vp, vp, vp, vp]
        lib.fedrag_partial_attn_quantized.argtypes = [sp, i64, i64, vp, vp, vp, vp, vp, i32, ctypes.c_float, f32p, f32p,
                                                      vp, ctypes.c_size_t, vp]
        lib.fedrag_partial_attn_varlen_quantized.argtypes = [sp, i64, i64, vp, vp, vp, vp, vp, i32, vp, vp,
                                                             ctypes.c_float, f32p, f32p, vp, ctypes.c_size_t, vp]
        lib.fedrag_invert_perm.argtypes = [vp, i64, vp, vp]
        lib.fedrag_validate_perm.argtypes = [vp, i32, i64, vp, vp, vp]
        lib.fedrag_status_string.argtypes = [ctypes.c_int]
        lib.fedrag_status_string.restype = ctypes.c_char_p
        lib.fedrag_version.restype = ctypes.c_int
        for name in ("fedrag_scramble_kv", "fedrag_scramble_q", "fedrag_partial_attn", "fedrag_partial_attn_static",
                     "fedrag_partial_attn_shards", "fedrag_unscramble_merge", "fedrag_lse_merge",
                     "fedrag_unscramble", "fedrag_invert_perm", "fedrag_validate_perm", "fedrag_scramble_kv_structured",
                     "fedrag_scramble_q_structured", "fedrag_unscramble_structured", "fedrag_local_attn",
                     "fedrag_unpermute_lse", "fedrag_partial_attn_varlen", "fedrag_quantize_rows",
                     "fedrag_dequantize_rows", "fedrag_scramble_kv_quantized",
                     "fedrag_scramble_kv_structured_quantized", "fedrag_partial_attn_quantized",
                     "fedrag_partial_attn_varlen_quantized"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().fedrag_status_string(int(status)).decode()


def version() -> int:
    return int(load().fedrag_version())


def _check(status: int, where: str) -> None:
    if status != OK:
        raise FedragError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("the library works on device memory: pass CUDA tensors")
    if not t.is_contiguous():
        raise ValueError("tensors must be dense row-major (contiguous)")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_shape(batch: int, n_q_heads: int, n_kv_heads: int, d_head: int, dtype) -> Shape:
    code = _DTYPES[dtype] if isinstance(dtype, torch.dtype) else int(dtype)
    return Shape(batch, n_q_heads, n_kv_heads, d_head, code)


def _shape_of(q_like: torch.Tensor, n_kv_heads: int, dtype=None) -> Shape:
    B, Hq, _, d = q_like.shape
    return make_shape(B, Hq, n_kv_heads, d, q_like.dtype if dtype is None else dtype)


# ----------------------------------------------------------------------------------------------- entry points
def fedrag_scramble_kv(K, V, phi_k, phi_v, perm_kv=None, n_q_heads: Optional[int] = None,
                       K_out=None, V_out=None):
    """K' = P_KV K Phi_KQ^{-T}, V' = P_KV V Phi_V for one shard.  K, V [B,Hkv,L,d]; perm_kv [n_perm,L] or [L]."""
    B, Hkv, L, d = K.shape
    shape = make_shape(B, n_q_heads or Hkv, Hkv, d, K.dtype)
    K_out = torch.empty_like(K) if K_out is None else K_out
    V_out = torch.empty_like(V) if V_out is None else V_out
    n_perm = 0
    if perm_kv is not None:
        n_perm = 1 if perm_kv.dim() == 1 else perm_kv.shape[0]
    st = load().fedrag_scramble_kv(ctypes.byref(shape), L, _ptr(K), _ptr(V), _ptr(phi_k), _ptr(phi_v),
                                   _ptr(perm_kv), n_perm, _ptr(K_out), _ptr(V_out), _stream())
    _check(st, "fedrag_scramble_kv")
    return K_out, V_out


def fedrag_scramble_q(Q, phi_q, perm_q=None, Q_out=None):
    """Q' = P_Q Q Phi_KQ.  Q [B,Hq,Lq,d]; phi_q [Hkv,d,d]."""
    B, Hq, Lq, d = Q.shape
    shape = make_shape(B, Hq, phi_q.shape[0], d, Q.dtype)
    Q_out = torch.empty_like(Q) if Q_out is None else Q_out
    st = load().fedrag_scramble_q(ctypes.byref(shape), Lq, _ptr(Q), _ptr(phi_q), _ptr(perm_q), _ptr(Q_out), _stream())
    _check(st, "fedrag_scramble_q")
    return Q_out


def fedrag_partial_attn_workspace_bytes(batch, n_q_heads, n_kv_heads, d_head, dtype, L_q, L_kv) -> int:
    shape = make_shape(batch, n_q_heads, n_kv_heads, d_head, dtype)
    return int(load().fedrag_partial_attn_workspace_bytes(ctypes.byref(shape), L_q, L_kv))


def fedrag_partial_attn(Qs, Ks, Vs, softmax_scale: Optional[float] = None, O_part=None, lse=None, workspace=None):
    """One shard's (O_i, lse_i).  Qs [B,Hq,Lq,d], Ks/Vs [B,Hkv,L,d] -> fp32 [B,Hq,Lq,d], fp32 [B,Hq,Lq]."""
    B, Hq, Lq, d = Qs.shape
    Hkv, L = Ks.shape[1], Ks.shape[2]
    shape = make_shape(B, Hq, Hkv, d, Qs.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    O_part = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=Qs.device) if O_part is None else O_part
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=Qs.device) if lse is None else lse
    need = int(load().fedrag_partial_attn_workspace_bytes(ctypes.byref(shape), Lq, L))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Qs.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fedrag_partial_attn(ctypes.byref(shape), Lq, L, _ptr(Qs), _ptr(Ks) if L > 0 else None,
                                    _ptr(Vs) if L > 0 else None, ctypes.c_float(softmax_scale), _ptr(O_part),
                                    _ptr(lse), _ptr(workspace), ws_bytes, _stream())
    _check(st, "fedrag_partial_attn")
    return O_part, lse


def fedrag_partial_attn_static(Qs, Ks, Vs, O_part, lse, softmax_scale: Optional[float] = None):
    """fedrag_partial_attn without a workspace argument (the library's static scratch array); the caller passes the
    outputs, so that the call allocates nothing."""
    B, Hq, Lq, d = Qs.shape
    Hkv, L = Ks.shape[1], Ks.shape[2]
    shape = make_shape(B, Hq, Hkv, d, Qs.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    st = load().fedrag_partial_attn_static(ctypes.byref(shape), Lq, L, _ptr(Qs), _ptr(Ks) if L > 0 else None,
                                           _ptr(Vs) if L > 0 else None, ctypes.c_float(softmax_scale), _ptr(O_part),
                                           _ptr(lse), _stream())
    _check(st, "fedrag_partial_attn_static")
    return O_part, lse


def fedrag_partial_attn_shards_workspace_bytes(batch, n_q_heads, n_kv_heads, d_head, dtype, L_q, L_kv_list) -> int:
    shape = make_shape(batch, n_q_heads, n_kv_heads, d_head, dtype)
    n = len(L_kv_list)
    Ls = (ctypes.c_int64 * n)(*[int(x) for x in L_kv_list])
    return int(load().fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(shape), L_q, n, Ls))


def fedrag_partial_attn_shards(Qs, Ks_list, Vs_list, softmax_scale: Optional[float] = None, O=None, lse=None,
                               workspace=None):
    """Per-shard attention and its aggregation over the shards in one call.  Qs [B,Hq,Lq,d];
    Ks_list[i], Vs_list[i] [B,Hkv,L_i,d] -> fp32 [B,Hq,Lq,d], fp32 [B,Hq,Lq] over all shards' keys."""
    B, Hq, Lq, d = Qs.shape
    n = len(Ks_list)
    Hkv = Ks_list[0].shape[1]
    shape = make_shape(B, Hq, Hkv, d, Qs.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    O = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=Qs.device) if O is None else O
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=Qs.device) if lse is None else lse
    Ls = (ctypes.c_int64 * n)(*[int(k.shape[2]) for k in Ks_list])
    Kp = (ctypes.c_void_p * n)(*[_ptr(k) if k.shape[2] > 0 else None for k in Ks_list])
    Vp = (ctypes.c_void_p * n)(*[_ptr(v) if v.shape[2] > 0 else None for v in Vs_list])
    need = int(load().fedrag_partial_attn_shards_workspace_bytes(ctypes.byref(shape), Lq, n, Ls))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Qs.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fedrag_partial_attn_shards(ctypes.byref(shape), Lq, n, Ls, Kp, Vp, _ptr(Qs),
                                           ctypes.c_float(softmax_scale), _ptr(O), _ptr(lse), _ptr(workspace),
                                           ws_bytes, _stream())
    _check(st, "fedrag_partial_attn_shards")
    return O, lse


def fedrag_partial_attn_varlen(Qs, Ks, Vs, kv_lens, softmax_scale: Optional[float] = None, O_part=None, lse=None,
                               workspace=None, q_lens=None):
    """fedrag_partial_attn over a padded batch: sequence b attends to its first kv_lens[b] keys.  kv_lens int32 [B]."""
    B, Hq, Lq, d = Qs.shape
    Hkv, L = Ks.shape[1], Ks.shape[2]
    if kv_lens.dtype != torch.int32 or kv_lens.shape != (B,):
        raise ValueError("kv_lens: int32 [B]")
    shape = make_shape(B, Hq, Hkv, d, Qs.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    O_part = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=Qs.device) if O_part is None else O_part
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=Qs.device) if lse is None else lse
    need = int(load().fedrag_partial_attn_workspace_bytes(ctypes.byref(shape), Lq, L))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Qs.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fedrag_partial_attn_varlen(ctypes.byref(shape), Lq, L, _ptr(Qs), _ptr(Ks) if L > 0 else None,
                                           _ptr(Vs) if L > 0 else None, _ptr(kv_lens), _ptr(q_lens),
                                           ctypes.c_float(softmax_scale),
                                           _ptr(O_part), _ptr(lse), _ptr(workspace), ws_bytes, _stream())
    _check(st, "fedrag_partial_attn_varlen")
    return O_part, lse


def fedrag_partial_attn_quantized(Qs, K_codes, K_params, V_codes, V_params, bits: int,
                                  softmax_scale: Optional[float] = None, O_part=None, lse=None, workspace=None):
    """fedrag_partial_attn reading K', V' as transport-codec codes (any query count; 16-bit storage)."""
    B, Hq, Lq, d = Qs.shape
    Hkv, L = K_codes.shape[1], K_codes.shape[2]
    shape = make_shape(B, Hq, Hkv, d, Qs.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    O_part = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=Qs.device) if O_part is None else O_part
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=Qs.device) if lse is None else lse
    need = int(load().fedrag_partial_attn_workspace_bytes(ctypes.byref(shape), Lq, L))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Qs.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    nz = L > 0
    st = load().fedrag_partial_attn_quantized(ctypes.byref(shape), Lq, L, _ptr(Qs), _ptr(K_codes) if nz else None,
                                              _ptr(K_params) if nz else None, _ptr(V_codes) if nz else None,
                                              _ptr(V_params) if nz else None, bits, ctypes.c_float(softmax_scale),
                                              _ptr(O_part), _ptr(lse), _ptr(workspace), ws_bytes, _stream())
    _check(st, "fedrag_partial_attn_quantized")
    return O_part, lse


def fedrag_partial_attn_varlen_quantized(Qs, K_codes, K_params, V_codes, V_params, bits: int, kv_lens,
                                         softmax_scale: Optional[float] = None, O_part=None, lse=None, workspace=None,
                                         q_lens=None):
    """fedrag_partial_attn_varlen reading K', V' as transport-codec codes: sequence b attends to its first kv_lens[b]
    keys; q_lens (optional) gives the real query rows per sequence."""
    B, Hq, Lq, d = Qs.shape
    Hkv, L = K_codes.shape[1], K_codes.shape[2]
    if kv_lens.dtype != torch.int32 or kv_lens.shape != (B,):
        raise ValueError("kv_lens: int32 [B]")
    shape = make_shape(B, Hq, Hkv, d, Qs.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    O_part = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=Qs.device) if O_part is None else O_part
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=Qs.device) if lse is None else lse
    need = int(load().fedrag_partial_attn_workspace_bytes(ctypes.byref(shape), Lq, L))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Qs.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    nz = L > 0
    st = load().fedrag_partial_attn_varlen_quantized(
        ctypes.byref(shape), Lq, L, _ptr(Qs), _ptr(K_codes) if nz else None, _ptr(K_params) if nz else None,
        _ptr(V_codes) if nz else None, _ptr(V_params) if nz else None, bits, _ptr(kv_lens), _ptr(q_lens),
        ctypes.c_float(softmax_scale), _ptr(O_part), _ptr(lse), _ptr(workspace), ws_bytes, _stream())
    _check(st, "fedrag_partial_attn_varlen_quantized")
    return O_part, lse


def fedrag_local_attn(Q, K, V, softmax_scale: Optional[float] = None, O_part=None, lse=None, workspace=None):
    """The Inquirer's own part (Section 5.3): the Lq queries are the last Lq of the L local tokens, each sees itself
    and what comes before.  Q [B,Hq,Lq,d], K/V [B,Hkv,L,d] plaintext -> fp32 [B,Hq,Lq,d], fp32 [B,Hq,Lq]."""
    B, Hq, Lq, d = Q.shape
    Hkv, L = K.shape[1], K.shape[2]
    shape = make_shape(B, Hq, Hkv, d, Q.dtype)
    if softmax_scale is None:
        softmax_scale = float(d) ** -0.5
    O_part = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=Q.device) if O_part is None else O_part
    lse = torch.empty((B, Hq, Lq), dtype=torch.float32, device=Q.device) if lse is None else lse
    need = int(load().fedrag_partial_attn_workspace_bytes(ctypes.byref(shape), Lq, L)) if Lq == 1 else 0
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st = load().fedrag_local_attn(ctypes.byref(shape), Lq, L, _ptr(Q), _ptr(K) if L > 0 else None,
                                  _ptr(V) if L > 0 else None, ctypes.c_float(softmax_scale), _ptr(O_part), _ptr(lse),
                                  _ptr(workspace), ws_bytes, _stream())
    _check(st, "fedrag_local_attn")
    return O_part, lse


def fedrag_unscramble_merge(O_scr, lse_scr, phi_v_inv, perm_q, O_local, lse_local, O_out=None, lse_out=None,
                            n_kv_heads: Optional[int] = None):
    """Dec of the remote result and its aggregation with the Inquirer's own partial, in one call."""
    B, Hq, Lq, d = O_scr.shape
    shape = make_shape(B, Hq, n_kv_heads or phi_v_inv.shape[0], d, F32)
    O_out = torch.empty_like(O_scr) if O_out is None else O_out
    lse_out = torch.empty_like(lse_scr) if lse_out is None else lse_out
    st = load().fedrag_unscramble_merge(ctypes.byref(shape), Lq, _ptr(O_scr), _ptr(lse_scr), _ptr(phi_v_inv),
                                        _ptr(perm_q), _ptr(O_local), _ptr(lse_local), _ptr(O_out), _ptr(lse_out),
                                        _stream())
    _check(st, "fedrag_unscramble_merge")
    return O_out, lse_out


def fedrag_unpermute_lse(lse_scr, perm_q=None, lse_out=None):
    """lse_out[b,h,perm_q[i]] = lse_scr[b,h,i]: the log-sum-exps back in the query rows' own order."""
    B, Hq, Lq = lse_scr.shape
    shape = make_shape(B, Hq, Hq, 128, F32)
    lse_out = torch.empty_like(lse_scr) if lse_out is None else lse_out
    st = load().fedrag_unpermute_lse(ctypes.byref(shape), Lq, _ptr(lse_scr), _ptr(perm_q), _ptr(lse_out), _stream())
    _check(st, "fedrag_unpermute_lse")
    return lse_out


def fedrag_lse_merge(O_parts, lses, n_kv_heads: Optional[int] = None, O_out=None, lse_out=None):
    """Aggregation over shards.  O_parts fp32 [S,B,Hq,Lq,d], lses fp32 [S,B,Hq,Lq]."""
    S, B, Hq, Lq, d = O_parts.shape
    shape = make_shape(B, Hq, n_kv_heads or Hq, d, F32)
    O_out = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=O_parts.device) if O_out is None else O_out
    lse_out = torch.empty((B, Hq, Lq), dtype=torch.float32, device=O_parts.device) if lse_out is None else lse_out
    st = load().fedrag_lse_merge(ctypes.byref(shape), Lq, S, _ptr(O_parts), _ptr(lses), _ptr(O_out), _ptr(lse_out),
                                 _stream())
    _check(st, "fedrag_lse_merge")
    return O_out, lse_out


def fedrag_unscramble(O_scr, phi_v_inv, perm_q=None, O_out=None):
    """Dec: out[b,h,perm_q[i]] = O_scr[b,h,i] @ phi_v_inv[h // G].  O_scr fp32 [B,Hq,Lq,d]; phi_v_inv fp32 [Hkv,d,d]."""
    B, Hq, Lq, d = O_scr.shape
    shape = make_shape(B, Hq, phi_v_inv.shape[0], d, F32)
    O_out = torch.empty_like(O_scr) if O_out is None else O_out
    st = load().fedrag_unscramble(ctypes.byref(shape), Lq, _ptr(O_scr), _ptr(phi_v_inv), _ptr(perm_q), _ptr(O_out),
                                  _stream())
    _check(st, "fedrag_unscramble")
    return O_out


def _key(key) -> StructuredKey:
    """key = (scale_in fp32, perm_in int32, perm_out int32, scale_out fp32), CUDA tensors [Hkv, d]."""
    a, g1, g2, b = key
    if a.dtype != torch.float32 or b.dtype != torch.float32 or g1.dtype != torch.int32 or g2.dtype != torch.int32:
        raise ValueError("structured key: scales are fp32, permutations int32")
    if not (a.shape == g1.shape == g2.shape == b.shape and a.dim() == 2):
        raise ValueError("structured key: four [Hkv, d] arrays")
    return StructuredKey(_ptr(a), _ptr(g1), _ptr(g2), _ptr(b))


def fedrag_scramble_kv_structured(K, V, key_k, key_v, perm_kv=None, n_q_heads: Optional[int] = None,
                                  K_out=None, V_out=None):
    """fedrag_scramble_kv with Phi_KQ^{-T} and Phi_V given as S1 P1 H P2 S2 factors (Section 4.2)."""
    B, Hkv, L, d = K.shape
    if key_k[0].shape != (Hkv, d) or key_v[0].shape != (Hkv, d):
        raise ValueError("structured key does not match [Hkv, d]")
    shape = make_shape(B, n_q_heads or Hkv, Hkv, d, K.dtype)
    K_out = torch.empty_like(K) if K_out is None else K_out
    V_out = torch.empty_like(V) if V_out is None else V_out
    n_perm = 0
    if perm_kv is not None:
        n_perm = 1 if perm_kv.dim() == 1 else perm_kv.shape[0]
    kk, kv = _key(key_k), _key(key_v)
    st = load().fedrag_scramble_kv_structured(ctypes.byref(shape), L, _ptr(K), _ptr(V), ctypes.byref(kk),
                                              ctypes.byref(kv), _ptr(perm_kv), n_perm, _ptr(K_out), _ptr(V_out),
                                              _stream())
    _check(st, "fedrag_scramble_kv_structured")
    return K_out, V_out


def fedrag_scramble_q_structured(Q, key_q, perm_q=None, Q_out=None):
    B, Hq, Lq, d = Q.shape
    if key_q[0].dim() != 2 or key_q[0].shape[1] != d:
        raise ValueError("structured key does not match [Hkv, d]")
    shape = make_shape(B, Hq, key_q[0].shape[0], d, Q.dtype)
    Q_out = torch.empty_like(Q) if Q_out is None else Q_out
    kq = _key(key_q)
    st = load().fedrag_scramble_q_structured(ctypes.byref(shape), Lq, _ptr(Q), ctypes.byref(kq), _ptr(perm_q),
                                             _ptr(Q_out), _stream())
    _check(st, "fedrag_scramble_q_structured")
    return Q_out


def fedrag_unscramble_structured(O_scr, key_v_inv, perm_q=None, O_out=None):
    B, Hq, Lq, d = O_scr.shape
    if key_v_inv[0].dim() != 2 or key_v_inv[0].shape[1] != d:
        raise ValueError("structured key does not match [Hkv, d]")
    shape = make_shape(B, Hq, key_v_inv[0].shape[0], d, F32)
    O_out = torch.empty_like(O_scr) if O_out is None else O_out
    kv = _key(key_v_inv)
    st = load().fedrag_unscramble_structured(ctypes.byref(shape), Lq, _ptr(O_scr), ctypes.byref(kv), _ptr(perm_q),
                                             _ptr(O_out), _stream())
    _check(st, "fedrag_unscramble_structured")
    return O_out


def fedrag_quantize_rows(X, bits: int, codes=None, params=None):
    """Transport codec (Section 7.5), per row of the last dimension.  X [..., d] -> (codes uint8 [..., d*bits/8],
    params fp32 [..., 2] = (scale, lo))."""
    d = X.shape[-1]
    n = X.numel() // d
    codes = torch.empty(X.shape[:-1] + (d * bits // 8,), dtype=torch.uint8, device=X.device) if codes is None else codes
    params = torch.empty(X.shape[:-1] + (2,), dtype=torch.float32, device=X.device) if params is None else params
    st = load().fedrag_quantize_rows(n, d, _DTYPES[X.dtype], bits, _ptr(X), _ptr(codes), _ptr(params), _stream())
    _check(st, "fedrag_quantize_rows")
    return codes, params


def fedrag_dequantize_rows(codes, params, bits: int, dtype, X_out=None):
    """Inverse map: codes uint8 [..., d*bits/8], params fp32 [..., 2] -> X [..., d] of `dtype`."""
    d = codes.shape[-1] * 8 // bits
    n = codes.numel() // codes.shape[-1]
    X_out = torch.empty(codes.shape[:-1] + (d,), dtype=dtype, device=codes.device) if X_out is None else X_out
    st = load().fedrag_dequantize_rows(n, d, _DTYPES[dtype], bits, _ptr(codes), _ptr(params), _ptr(X_out), _stream())
    _check(st, "fedrag_dequantize_rows")
    return X_out


def fedrag_scramble_kv_quantized(K, V, phi_k, phi_v, perm_kv, bits: int, n_q_heads: Optional[int] = None,
                                 structured: bool = False, out=None):
    """Enc of a KV shard with the transport codec as epilogue.  phi_k / phi_v: dense matrices, or structured keys
    with structured=True.  Returns (K_codes, K_params, V_codes, V_params)."""
    B, Hkv, L, d = K.shape
    shape = make_shape(B, n_q_heads or Hkv, Hkv, d, K.dtype)
    mk_c = lambda: torch.empty((B, Hkv, L, d * bits // 8), dtype=torch.uint8, device=K.device)
    mk_p = lambda: torch.empty((B, Hkv, L, 2), dtype=torch.float32, device=K.device)
    Kc, Kp, Vc, Vp = (mk_c(), mk_p(), mk_c(), mk_p()) if out is None else out
    n_perm = 0
    if perm_kv is not None:
        n_perm = 1 if perm_kv.dim() == 1 else perm_kv.shape[0]
    if structured:
        kk, kv = _key(phi_k), _key(phi_v)
        st = load().fedrag_scramble_kv_structured_quantized(ctypes.byref(shape), L, _ptr(K), _ptr(V), ctypes.byref(kk),
                                                            ctypes.byref(kv), _ptr(perm_kv), n_perm, bits, _ptr(Kc),
                                                            _ptr(Kp), _ptr(Vc), _ptr(Vp), _stream())
    else:
        st = load().fedrag_scramble_kv_quantized(ctypes.byref(shape), L, _ptr(K), _ptr(V), _ptr(phi_k), _ptr(phi_v),
                                                 _ptr(perm_kv), n_perm, bits, _ptr(Kc), _ptr(Kp), _ptr(Vc), _ptr(Vp),
                                                 _stream())
    _check(st, "fedrag_scramble_kv_quantized")
    return Kc, Kp, Vc, Vp


def fedrag_invert_perm(perm, inv_out=None):
    inv_out = torch.empty_like(perm) if inv_out is None else inv_out
    st = load().fedrag_invert_perm(_ptr(perm), perm.numel(), _ptr(inv_out), _stream())
    _check(st, "fedrag_invert_perm")
    return inv_out


def fedrag_validate_perm(perm, flag_out=None, marks=None):
    """Debug aid: device int32 flag, 0 when every row of perm ([L] or [n_perm, L] int32) is a permutation of 0..L-1,
    else bit 0 = an index out of range, bit 1 = an index repeated.  Read it after synchronising."""
    n_perm = 1 if perm.dim() == 1 else perm.shape[0]
    L = perm.shape[-1]
    flag_out = torch.empty(1, dtype=torch.int32, device=perm.device) if flag_out is None else flag_out
    marks = torch.empty(max(1, n_perm * L), dtype=torch.int32, device=perm.device) if marks is None else marks
    st = load().fedrag_validate_perm(_ptr(perm), n_perm, L, _ptr(marks), _ptr(flag_out), _stream())
    _check(st, "fedrag_validate_perm")
    return flag_out
