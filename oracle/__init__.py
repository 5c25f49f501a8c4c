"""CPU oracle for Scrambled Distributed Attention (FedRAG, Section 4).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports it, and it never imports the product package.

The arithmetic lives in ``fedrag_oracle.c`` (plain C, fp64).  This module only
compiles that file with gcc, marshals numpy arrays into it, and strings the
calls together in the order of the protocol (Enc -> attention per shard ->
aggregation -> Dec).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fedrag_oracle.c")
_LIB = os.path.join(_HERE, "libfedrag_oracle.so")
_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, no fast-math) and return the path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build())
            lib.oracle_get_threads.restype = ctypes.c_int
            _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    """Any array-like (numpy, or a CPU torch tensor of any float dtype) as C-contiguous fp64."""
    if hasattr(a, "detach"):  # torch tensor; bf16 has no numpy dtype, so widen first
        a = a.detach().cpu().double().numpy()
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    if a is None:
        return None
    if hasattr(a, "detach"):
        a = a.detach().cpu().numpy()
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


_c_int = ctypes.c_int
_c_i64 = ctypes.c_int64
_c_dbl = ctypes.c_double


def set_threads(n: int) -> None:
    _load().oracle_set_threads(_c_int(int(n)))


def get_threads() -> int:
    return int(_load().oracle_get_threads())


def plain_attention(Q, K, V):
    """Eq. (1) over [B,Hq,Lq,d] x [B,Hkv,Lk,d]; returns (O, lse) in fp64."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, Hq, Lq, d = Q.shape
    _, Hkv, Lk, _ = K.shape
    assert K.shape == V.shape and K.shape[0] == B and K.shape[3] == d and Hq % Hkv == 0
    O = np.empty((B, Hq, Lq, d), np.float64)
    lse = np.empty((B, Hq, Lq), np.float64)
    _load().oracle_plain_attention(_p(Q), _p(K), _p(V), _c_int(B), _c_int(Hq), _c_int(Hkv),
                                   _c_i64(Lq), _c_i64(Lk), _c_int(d), _p(O), _p(lse))
    return O, lse


def local_attention_raw(Q, K, V):
    """Section 4.1 literally: (O_i, w_i) with w_i the raw sum of exponentials."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, Hq, Lq, d = Q.shape
    _, Hkv, Lk, _ = K.shape
    assert K.shape == V.shape and Hq % Hkv == 0
    O = np.empty((B, Hq, Lq, d), np.float64)
    w = np.empty((B, Hq, Lq), np.float64)
    _load().oracle_local_attention_raw(_p(Q), _p(K), _p(V), _c_int(B), _c_int(Hq), _c_int(Hkv),
                                       _c_i64(Lq), _c_i64(Lk), _c_int(d), _p(O), _p(w))
    return O, w


def aggregate_raw(O_parts, w):
    """Section 4.1 aggregation literally: sum_i w_i O_i / sum_i w_i.  O_parts [M,...,d], w [M,...]."""
    O_parts, w = _f64(O_parts), _f64(w)
    M, d = O_parts.shape[0], O_parts.shape[-1]
    rows = int(np.prod(w.shape[1:]))
    O = np.empty(O_parts.shape[1:], np.float64)
    wt = np.empty(w.shape[1:], np.float64)
    _load().oracle_aggregate_raw(_p(O_parts), _p(w), _c_int(M), _c_i64(rows), _c_int(d), _p(O), _p(wt))
    return O, wt


def scramble(X, Phi, perm=None):
    """Enc for one operand: out[b,h,j,:] = X[b,h,perm[j],:] @ Phi[h // G].

    X [B,H,L,d]; Phi [Hkv,d,d] with G = H // Hkv; perm None, [L] or [n_perm,L] int32 (gather).
    """
    X, Phi = _f64(X), _f64(Phi)
    B, H, L, d = X.shape
    Hkv = Phi.shape[0]
    assert Phi.shape == (Hkv, d, d) and H % Hkv == 0
    perm = _i32(perm)
    n_perm = 1
    if perm is not None:
        if perm.ndim == 1:
            perm = perm[None, :]
        n_perm = perm.shape[0]
        assert perm.shape[1] == L and n_perm in (1, B)
        perm = np.ascontiguousarray(perm)
    out = np.empty_like(X)
    _load().oracle_scramble(_p(X), _p(Phi), _p(perm), _c_int(n_perm), _c_int(B), _c_int(H),
                            _c_int(H // Hkv), _c_i64(L), _c_int(d), _p(out))
    return out


def partial_attn(Qs, Ks, Vs, scale=None):
    """One shard's (O_i, lse_i = ln w_i), Section 4.1.  scale defaults to 1/sqrt(d)."""
    Qs, Ks, Vs = _f64(Qs), _f64(Ks), _f64(Vs)
    B, Hq, Lq, d = Qs.shape
    _, Hkv, Lk, _ = Ks.shape
    assert Ks.shape == Vs.shape and Ks.shape[0] == B and Ks.shape[3] == d and Hq % Hkv == 0
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    O = np.empty((B, Hq, Lq, d), np.float64)
    lse = np.empty((B, Hq, Lq), np.float64)
    _load().oracle_partial_attn(_p(Qs), _p(Ks), _p(Vs), _c_int(B), _c_int(Hq), _c_int(Hkv),
                                _c_i64(Lq), _c_i64(Lk), _c_int(d), _c_dbl(float(scale)), _p(O), _p(lse))
    return O, lse


def partial_attn_varlen(Qs, Ks, Vs, kv_lens, scale=None):
    """partial_attn over a padded batch: sequence b attends to its first kv_lens[b] keys (Section 5.2 workload)."""
    Qs, Ks, Vs = _f64(Qs), _f64(Ks), _f64(Vs)
    B, Hq, Lq, d = Qs.shape
    _, Hkv, Lk, _ = Ks.shape
    kv_lens = np.ascontiguousarray(_i32(kv_lens))
    assert Ks.shape == Vs.shape and Ks.shape[0] == B and Ks.shape[3] == d and Hq % Hkv == 0
    assert kv_lens.shape == (B,) and kv_lens.min() >= 0 and kv_lens.max() <= Lk
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    O = np.empty((B, Hq, Lq, d), np.float64)
    lse = np.empty((B, Hq, Lq), np.float64)
    _load().oracle_partial_attn_varlen(_p(Qs), _p(Ks), _p(Vs), _p(kv_lens), _c_int(B), _c_int(Hq), _c_int(Hkv),
                                       _c_i64(Lq), _c_i64(Lk), _c_int(d), _c_dbl(float(scale)), _p(O), _p(lse))
    return O, lse


def local_causal_attn(Q, K, V, scale=None):
    """The Inquirer's own part (Section 5.3): the Lq queries are the last Lq of the Lk local tokens and each sees
    itself and everything before it.  Returns (O, lse = ln w) like partial_attn."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    B, Hq, Lq, d = Q.shape
    _, Hkv, Lk, _ = K.shape
    assert K.shape == V.shape and K.shape[0] == B and K.shape[3] == d and Hq % Hkv == 0 and Lk >= Lq
    if scale is None:
        scale = 1.0 / np.sqrt(float(d))
    O = np.empty((B, Hq, Lq, d), np.float64)
    lse = np.empty((B, Hq, Lq), np.float64)
    _load().oracle_local_causal_attn(_p(Q), _p(K), _p(V), _c_int(B), _c_int(Hq), _c_int(Hkv),
                                     _c_i64(Lq), _c_i64(Lk), _c_int(d), _c_dbl(float(scale)), _p(O), _p(lse))
    return O, lse


def lse_merge(O_parts, lses):
    """Aggregation in the log domain.  O_parts [S,...,d], lses [S,...] -> (O [...,d], lse [...])."""
    O_parts, lses = _f64(O_parts), _f64(lses)
    S, d = O_parts.shape[0], O_parts.shape[-1]
    assert lses.shape == O_parts.shape[:-1]
    rows = int(np.prod(lses.shape[1:]))
    O = np.empty(O_parts.shape[1:], np.float64)
    lse = np.empty(lses.shape[1:], np.float64)
    _load().oracle_lse_merge(_p(O_parts), _p(lses), _c_int(S), _c_i64(rows), _c_int(d), _p(O), _p(lse))
    return O, lse


def unscramble(O, PhiInv, perm=None):
    """Dec: out[b,h,perm[i],:] = O[b,h,i,:] @ PhiInv[h // G] (perm = the gather array used on Q)."""
    O, PhiInv = _f64(O), _f64(PhiInv)
    B, H, L, d = O.shape
    Hkv = PhiInv.shape[0]
    assert PhiInv.shape == (Hkv, d, d) and H % Hkv == 0
    perm = _i32(perm)
    if perm is not None:
        assert perm.shape == (L,)
    out = np.zeros_like(O)
    _load().oracle_unscramble(_p(O), _p(PhiInv), _p(perm), _c_int(B), _c_int(H), _c_int(H // Hkv),
                              _c_i64(L), _c_int(d), _p(out))
    return out


def structured(X, key, perm=None, scatter=False):
    """Section 4.2 structured transform Phi = S1 P1 H P2 S2 applied factor by factor (never formed as a matrix).

    X [B,H,L,d]; key = (a, g1, g2, b), each [Hkv,d]: scale, channel gather, normalised Sylvester Hadamard, channel
    gather, scale.  perm None, [L] or [n_perm,L] int32; rows are gathered (Enc) or, with scatter=True, scattered (Dec).
    """
    X = _f64(X)
    a, g1, g2, b = key
    a, b = _f64(a), _f64(b)
    g1, g2 = np.ascontiguousarray(_i32(g1)), np.ascontiguousarray(_i32(g2))
    B, H, L, d = X.shape
    Hkv = a.shape[0]
    assert a.shape == (Hkv, d) and b.shape == (Hkv, d) and g1.shape == (Hkv, d) and g2.shape == (Hkv, d)
    assert H % Hkv == 0 and d & (d - 1) == 0, "Sylvester's Hadamard matrix needs d a power of two"
    perm = _i32(perm)
    n_perm = 1
    if perm is not None:
        if perm.ndim == 1:
            perm = perm[None, :]
        n_perm = perm.shape[0]
        assert perm.shape[1] == L and n_perm in (1, B)
        perm = np.ascontiguousarray(perm)
    out = np.empty_like(X)
    _load().oracle_structured(_p(X), _p(a), _p(g1), _p(g2), _p(b), _p(perm), _c_int(n_perm), _c_int(int(scatter)),
                              _c_int(B), _c_int(H), _c_int(H // Hkv), _c_i64(L), _c_int(d), _p(out))
    return out


def quantize_rows(X, bits):
    """Section 7.5 transport codec, per row (token) of d channels: returns (codes uint8 [..., d*bits/8], params fp32
    [..., 2] = (scale, lo)).  X: any float array/tensor [..., d]; it is taken in fp32 (exact for 16-bit storage)."""
    if hasattr(X, "detach"):
        X = X.detach().cpu().float().numpy()
    X = np.ascontiguousarray(X, dtype=np.float32)
    d = X.shape[-1]
    assert bits in (8, 4) and d % 2 == 0
    n = X.size // d
    codes = np.empty(X.shape[:-1] + (d * bits // 8,), np.uint8)
    params = np.empty(X.shape[:-1] + (2,), np.float32)
    _load().oracle_quantize_rows(_p(X), _c_i64(n), _c_int(d), _c_int(bits), _p(codes), _p(params))
    return codes, params


def dequantize_rows(codes, params, bits):
    """Inverse map of quantize_rows: fp32 values code * scale + lo (one fused multiply-add each)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    params = np.ascontiguousarray(params, dtype=np.float32)
    d = codes.shape[-1] * 8 // bits
    n = codes.size // codes.shape[-1]
    X = np.empty(codes.shape[:-1] + (d,), np.float32)
    _load().oracle_dequantize_rows(_p(codes), _p(params), _c_i64(n), _c_int(d), _c_int(bits), _p(X))
    return X


def invert_perm(perm):
    perm = _i32(perm)
    inv = np.empty_like(perm)
    _load().oracle_invert_perm(_p(perm), _c_i64(perm.shape[0]), _p(inv))
    return inv


def protocol(Q, K_shards, V_shards, phi_q, phi_k, phi_v, phi_v_inv, perm_q=None, perm_kv=None,
             descramble_first=False):
    """The whole scrambled attention protocol in fp64, in the paper's order.

    K_shards / V_shards: lists of [B,Hkv,L_s,d]; perm_kv: list of gather arrays (or None) per shard.
    phi_k is Phi_KQ^{-T}, phi_v_inv is Phi_V^{-1}; both are passed in (keys are inputs, not drawn here).
    descramble_first=True follows the prefill paragraph of Section 5.3 (Dec every partial, then aggregate);
    False aggregates the scrambled partials and applies Dec once (equal by the linearity lemma).
    Returns (out, lse) with out in the plaintext domain.
    """
    Qs = scramble(Q, phi_q, perm_q)
    parts, lses = [], []
    for s, (K, V) in enumerate(zip(K_shards, V_shards)):
        pk = None if perm_kv is None else perm_kv[s]
        Ks = scramble(K, phi_k, pk)
        Vs = scramble(V, phi_v, pk)
        O_s, l_s = partial_attn(Qs, Ks, Vs)
        if descramble_first:
            O_s = unscramble(O_s, phi_v_inv, None)  # feature part of Dec; rows still in P_Q order
        parts.append(O_s)
        lses.append(l_s)
    O, lse = lse_merge(np.stack(parts), np.stack(lses))
    if descramble_first:
        B, H, L, d = O.shape
        eye = np.broadcast_to(np.eye(d), (np.asarray(phi_v_inv).shape[0], d, d))
        out = unscramble(O, eye, perm_q)  # token part of Dec
    else:
        out = unscramble(O, phi_v_inv, perm_q)
    # lse rows are in P_Q order too: put them back
    if perm_q is not None:
        pq = _i32(perm_q)
        lse_out = np.empty_like(lse)
        lse_out[:, :, pq] = lse
        lse = lse_out
    return out, lse
