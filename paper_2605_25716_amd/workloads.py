"""Seeded synthetic inputs and key material for Scrambled Distributed Attention.

This module holds NO arithmetic of the method itself: it draws activations,
draws the key set Theta = {Phi_KQ, Phi_V, P_Q, P_KV} (Section 4.2, "Scrambled
Attention Protocol") and derives the dual / inverse matrices a key holder
would hand to the library.  Both the HIP path and the CPU oracle are fed from
here; neither of them is imported here.

Workload shapes follow the Llama-3-8B / 70B-shaped configurations this build is
measured on (they stand in for the paper's fixed-length synthetic latency
workloads, Section 7.1): activations N(0,1) with 1 % of the (head, channel)
axis scaled by 20 as outlier channels, a Haar-random orthogonal scramble per
KV head and a uniform random token permutation per shard.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional

import numpy as np
import torch

BASE_SEED = 0xFED2A6
KEY_SEED_XOR = 0x5C4A


@dataclass(frozen=True)
class Config:
    name: str
    batch: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    L_q: int
    n_shards: int
    L_kv: int            # tokens per shard
    dtype: str           # "f32" | "bf16" | "f16"
    outliers: bool
    index: int           # position in the configuration list (seeds derive from it)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def scaled(self, **kw) -> "Config":
        return replace(self, **kw)


CONFIGS = {
    # tiny fp32 case: parity only
    "tiny_f32": Config("tiny_f32", 1, 2, 2, 64, 4, 1, 512, "f32", False, 0),
    # Llama-3-8B-shaped decode: the configuration the headline metric is quoted on
    "llama8b_decode": Config("llama8b_decode", 16, 32, 8, 128, 1, 4, 8192, "bf16", True, 1),
    # RAG prefill, non-causal over retrieved documents
    "rag_prefill": Config("rag_prefill", 1, 32, 8, 128, 2048, 1, 16384, "bf16", True, 2),
    # long-context decode
    "long_decode": Config("long_decode", 64, 32, 8, 128, 1, 8, 32768, "bf16", True, 3),
    # 70B-shaped mixed workload, split into its two parts (they share KV shapes: 8 x 8192, G = 8)
    "mixed70b_decode": Config("mixed70b_decode", 32, 64, 8, 128, 1, 8, 8192, "bf16", True, 4),
    "mixed70b_prefill": Config("mixed70b_prefill", 1, 64, 8, 128, 4096, 8, 8192, "bf16", True, 4),
}

_TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def torch_dtype(name: str) -> torch.dtype:
    return _TORCH_DTYPE[name]


# ----------------------------------------------------------------------------- activations
def outlier_channels(n_heads: int, d_head: int, seed: int, tensor_id: int) -> np.ndarray:
    """Indices, over the flattened (head, channel) axis, of the channels scaled by 20."""
    n_out = max(1, int(round(0.01 * n_heads * d_head)))
    rng = np.random.default_rng([seed, tensor_id, 0x0071])
    return np.sort(rng.choice(n_heads * d_head, size=n_out, replace=False))


def activations(batch: int, n_heads: int, L: int, d_head: int, *, seed: int, tensor_id: int,
                outliers: bool, outlier_id: Optional[int] = None,
                dtype: torch.dtype = torch.float32, device="cpu") -> torch.Tensor:
    """[batch, n_heads, L, d_head] i.i.d. N(0,1), optional x20 outlier channels, rounded (RNE) to dtype.

    tensor_id selects the random stream (a shard gets its own); outlier_id selects the outlier channel
    set, which is fixed per tensor kind (Q, K or V) across batch, tokens and shards.
    """
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed((seed * 1000003 + tensor_id) & 0x7FFFFFFFFFFFFFFF)
    out = torch.empty((batch, n_heads, L, d_head), dtype=dtype, device=dev)
    scale = None
    if outliers:
        s = np.ones(n_heads * d_head, dtype=np.float32)
        s[outlier_channels(n_heads, d_head, seed, tensor_id if outlier_id is None else outlier_id)] = 20.0
        scale = torch.from_numpy(s).view(1, n_heads, 1, d_head).to(dev)
    for b in range(batch):  # one sequence at a time keeps the fp32 staging buffer small
        x = torch.randn((1, n_heads, L, d_head), generator=gen, dtype=torch.float32, device=dev)
        if scale is not None:
            x *= scale
        out[b:b + 1] = x.to(dtype)
    return out


# ----------------------------------------------------------------------------- key material
def haar_orthogonal(rng: np.random.Generator, d: int) -> np.ndarray:
    """Haar-distributed orthogonal d x d matrix: Q factor of a Gaussian matrix with diag(R) > 0."""
    a = rng.standard_normal((d, d))
    q, r = np.linalg.qr(a)
    return q * np.sign(np.diag(r))[None, :]


def sylvester_hadamard(d: int) -> np.ndarray:
    assert d > 0 and (d & (d - 1)) == 0, "Hadamard order must be a power of two"
    h = np.ones((1, 1))
    while h.shape[0] < d:
        h = np.block([[h, h], [h, -h]])
    return h


def structured_phi(rng: np.random.Generator, d: int, lo: float = 0.125, hi: float = 8.0,
                   use_s2: bool = True) -> np.ndarray:
    """Phi = S1 P1 H P2 S2 (Section 4.2): normalised Hadamard between two random permutations and two
    random-sign diagonal scalings with magnitudes log-uniform in [lo, hi].  use_s2=False drops S2."""
    def diag():
        mag = np.exp(rng.uniform(np.log(lo), np.log(hi), size=d))
        return mag * rng.choice([-1.0, 1.0], size=d)
    s1 = diag()
    s2 = diag() if use_s2 else np.ones(d)
    p1 = rng.permutation(d)
    p2 = rng.permutation(d)
    h = sylvester_hadamard(d) / np.sqrt(d)
    eye = np.eye(d)
    return np.diag(s1) @ eye[p1] @ h @ eye[p2] @ np.diag(s2)


def _round_to(a: np.ndarray, dtype: torch.dtype) -> np.ndarray:
    """Round an fp64 array to a storage dtype (RNE) and return the stored values as fp64."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(dtype).double().numpy()


@dataclass
class Keys:
    """Key set as the library consumes it.  phi_q, phi_k, phi_v are in the storage dtype; phi_v_inv is fp32.

    phi_k is the inverse transpose of phi_q *as stored*, and phi_v_inv the inverse of phi_v *as stored*
    (computed in fp64, then rounded once), so the duality error is first order in a single rounding.
    """
    phi_q: torch.Tensor        # [Hkv, d, d]  Phi_KQ
    phi_k: torch.Tensor        # [Hkv, d, d]  Phi_KQ^{-T}
    phi_v: torch.Tensor        # [Hkv, d, d]  Phi_V
    phi_v_inv: torch.Tensor    # [Hkv, d, d]  Phi_V^{-1}, fp32
    perm_q: Optional[torch.Tensor]   # [L_q] int32 gather indices, None = identity
    perm_kv: List[torch.Tensor]      # per shard: [n_perm, L_kv] int32 gather indices
    phi_kq_exact: np.ndarray   # fp64, before rounding (for oracle-side invariants)
    phi_v_exact: np.ndarray


def make_keys(n_kv_heads: int, d_head: int, L_q: int, L_kv: int, n_shards: int, *, seed: int,
              dtype: torch.dtype, kind: str = "orthogonal", n_perm: int = 1, batch: int = 1,
              permute_q: Optional[bool] = None) -> Keys:
    rng = np.random.default_rng([seed ^ KEY_SEED_XOR, 0x6B65])
    draw = (lambda: haar_orthogonal(rng, d_head)) if kind == "orthogonal" else \
           (lambda: structured_phi(rng, d_head)) if kind == "structured" else \
           (lambda: np.eye(d_head)) if kind == "identity" else None
    if draw is None:
        raise ValueError(kind)
    phi_kq = np.stack([draw() for _ in range(n_kv_heads)])
    phi_v = np.stack([draw() for _ in range(n_kv_heads)])
    phi_q_st = _round_to(phi_kq, dtype)
    phi_k_st = _round_to(np.transpose(np.linalg.inv(phi_q_st), (0, 2, 1)), dtype)
    phi_v_st = _round_to(phi_v, dtype)
    phi_v_inv = np.linalg.inv(phi_v_st)
    if permute_q is None:
        permute_q = L_q > 1
    perm_q = torch.from_numpy(rng.permutation(L_q).astype(np.int32)) if permute_q else None
    assert n_perm in (1, batch)
    perm_kv = [torch.from_numpy(np.stack([rng.permutation(L_kv) for _ in range(n_perm)]).astype(np.int32))
               for _ in range(n_shards)]
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(dt)
    return Keys(t(phi_q_st, dtype), t(phi_k_st, dtype), t(phi_v_st, dtype), t(phi_v_inv, torch.float32),
                perm_q, perm_kv, phi_kq, phi_v)


@dataclass
class StructuredKeys:
    """Keys of the structured form Phi = S1 P1 H P2 S2 (Section 4.2), never multiplied out.

    Each of q, k, v, v_inv is a tuple (scale_in [Hkv,d] fp32, perm_in [Hkv,d] int32, perm_out [Hkv,d] int32,
    scale_out [Hkv,d] fp32) with the permutations as gathers: y = (((x * scale_in)[perm_in]) H)[perm_out] * scale_out.
    k is the inverse transpose of q (same permutations, reciprocal scales) and v_inv the inverse of v (inverse
    permutations swapped, reciprocal scales swapped).  scale_in of q, k, v holds values the storage dtype represents
    exactly: the 16-bit kernels fold it into their +-1 operand matrix.
    """
    q: tuple
    k: tuple
    v: tuple
    v_inv: tuple
    perm_q: Optional[torch.Tensor]
    perm_kv: List[torch.Tensor]


def make_structured_keys(n_kv_heads: int, d_head: int, L_q: int, L_kv: int, n_shards: int, *, seed: int,
                         dtype: torch.dtype, lo: float = 0.125, hi: float = 8.0, use_s2: bool = True,
                         pow2: bool = False, n_perm: int = 1, batch: int = 1,
                         permute_q: Optional[bool] = None) -> StructuredKeys:
    """Draw S1, P1, P2, S2 per KV head for Phi_KQ and Phi_V: magnitudes log-uniform in [lo, hi] (powers of two with
    pow2=True), random signs, uniform permutations; use_s2=False leaves S2 out (all ones)."""
    rng = np.random.default_rng([seed ^ KEY_SEED_XOR, 0x5350])

    def diag(on=True):
        if not on:
            return np.ones((n_kv_heads, d_head))
        e = rng.uniform(np.log2(lo), np.log2(hi), size=(n_kv_heads, d_head))
        mag = np.exp2(np.round(e)) if pow2 else np.exp2(e)
        return mag * rng.choice([-1.0, 1.0], size=(n_kv_heads, d_head))

    def perms():
        return np.stack([rng.permutation(d_head) for _ in range(n_kv_heads)]).astype(np.int32)

    def inv(g):
        out = np.empty_like(g)
        for h in range(g.shape[0]):
            out[h, g[h]] = np.arange(g.shape[1], dtype=g.dtype)
        return out

    f32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32))
    out = {}
    for name in ("kq", "v"):
        a = _round_to(diag(), dtype)          # stored exactly by the storage dtype
        g1, g2 = perms(), perms()
        b = diag(use_s2).astype(np.float32).astype(np.float64)
        out[name] = (a, g1, g2, b)
    a, g1, g2, b = out["kq"]
    key_q = (f32(a), i32(g1), i32(g2), f32(b))
    key_k = (f32(_round_to(1.0 / a, dtype)), i32(g1), i32(g2), f32(1.0 / b))
    a, g1, g2, b = out["v"]
    key_v = (f32(a), i32(g1), i32(g2), f32(b))
    key_v_inv = (f32(1.0 / b), i32(inv(g2)), i32(inv(g1)), f32(1.0 / a))
    if permute_q is None:
        permute_q = L_q > 1
    perm_q = torch.from_numpy(rng.permutation(L_q).astype(np.int32)) if permute_q else None
    assert n_perm in (1, batch)
    perm_kv = [torch.from_numpy(np.stack([rng.permutation(L_kv) for _ in range(n_perm)]).astype(np.int32))
               for _ in range(n_shards)]
    return StructuredKeys(key_q, key_k, key_v, key_v_inv, perm_q, perm_kv)


# ----------------------------------------------------------------------------- whole cases
TID_Q, TID_K, TID_V = 1, 100, 200  # random-stream ids; shard s uses TID_K + s, TID_V + s


@dataclass
class Case:
    cfg: Config
    Q: torch.Tensor                 # [B,Hq,Lq,d]
    K: List[torch.Tensor]           # per shard [B,Hkv,L,d]
    V: List[torch.Tensor]
    keys: Keys


def make_case(cfg: Config, *, device="cpu", kind: str = "orthogonal", n_perm: int = 1) -> Case:
    """All plaintext tensors and keys of one configuration, drawn from cfg.seed."""
    dt = torch_dtype(cfg.dtype)
    Q = activations(cfg.batch, cfg.n_q_heads, cfg.L_q, cfg.d_head, seed=cfg.seed, tensor_id=TID_Q,
                    outliers=cfg.outliers, dtype=dt, device=device)
    K = [activations(cfg.batch, cfg.n_kv_heads, cfg.L_kv, cfg.d_head, seed=cfg.seed, tensor_id=TID_K + s,
                     outliers=cfg.outliers, outlier_id=TID_K, dtype=dt, device=device)
         for s in range(cfg.n_shards)]
    V = [activations(cfg.batch, cfg.n_kv_heads, cfg.L_kv, cfg.d_head, seed=cfg.seed, tensor_id=TID_V + s,
                     outliers=cfg.outliers, outlier_id=TID_V, dtype=dt, device=device)
         for s in range(cfg.n_shards)]
    keys = make_keys(cfg.n_kv_heads, cfg.d_head, cfg.L_q, cfg.L_kv, cfg.n_shards, seed=cfg.seed, dtype=dt,
                     kind=kind, n_perm=n_perm, batch=cfg.batch)
    return Case(cfg, Q, K, V, keys)
