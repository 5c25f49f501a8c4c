"""GPU parity of attention over a padded batch of unequal sequences (the re-ranking workload of Section 5.2)."""
import numpy as np
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"

CASES = [
    # name, B, Hq, Hkv, d, Lq, Lkv, dtype, lens
    ("rerank_bf16", 10, 8, 8, 64, 300, 300, "bf16", [300, 257, 64, 1, 129, 0, 200, 299, 63, 128]),   # bidirectional pairs
    ("prefill_bf16_d128", 3, 8, 2, 128, 70, 500, "bf16", [500, 33, 260]),
    ("decode_bf16", 5, 8, 2, 128, 1, 3000, "bf16", [3000, 0, 1, 517, 2048]),                           # KV-split path
    ("decode_f16_rows16", 2, 8, 2, 128, 4, 900, "f16", [640, 31]),
    ("f32", 3, 4, 2, 64, 5, 100, "f32", [100, 0, 37]),
]


@pytest.mark.parametrize("poison", ["huge", "nan", "inf"])
@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_partial_attn_varlen(oracle, case, poison):
    name, B, Hq, Hkv, d, Lq, L, dt, lens = case
    dtype = W.torch_dtype(dt)
    seed = 500 + len(name)
    keys = W.make_keys(Hkv, d, Lq, L, 1, seed=seed, dtype=dtype)
    rnd = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype)
    Q = W.activations(B, Hq, Lq, d, seed=seed, tensor_id=W.TID_Q, outliers=(dt != "f32"), dtype=dtype)
    K = W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_K, outliers=(dt != "f32"), dtype=dtype)
    V = W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_V, outliers=(dt != "f32"), dtype=dtype)
    Qs, Ks, Vs = rnd(oracle.scramble(Q, keys.phi_q, None)), rnd(oracle.scramble(K, keys.phi_k, None)), \
        rnd(oracle.scramble(V, keys.phi_v, None))
    lens_t = torch.tensor(lens, dtype=torch.int32)
    # poison the padding: it must not reach the result, not even through a product with a zero probability
    pk, pv = {"huge": (3.0e4 if dt != "bf16" else 1.0e30, -3.0e4 if dt != "bf16" else -1.0e30),
              "nan": (float("nan"), float("nan")), "inf": (float("inf"), -float("inf"))}[poison]
    for b, n in enumerate(lens):
        Ks[b, :, n:] = pk
        Vs[b, :, n:] = pv
    O, lse = fb.fedrag_partial_attn_varlen(Qs.to(DEV), Ks.to(DEV), Vs.to(DEV), lens_t.to(DEV))
    torch.cuda.synchronize()
    for b, n in enumerate(lens):  # the oracle never touches the padding either; give it finite values all the same
        Ks[b, :, n:] = 0
        Vs[b, :, n:] = 0
    Or, lr = oracle.partial_attn_varlen(Qs, Ks, Vs, lens_t)
    PT.check_attn(O, lse, Or, lr, dtype, f"{name}/{poison}")


@pytest.mark.parametrize("dt,d", [("bf16", 64), ("f32", 64)])
def test_query_lengths_skip_padding_rows(oracle, dt, d):
    """Re-ranking pairs: every token of a pair attends to the pair; rows past a pair's length are not written."""
    dtype = W.torch_dtype(dt)
    B, H, Lmax = 4, 4, 600
    lens = [600, 257, 0, 300]
    seed = 321
    mk = lambda tid: W.activations(B, H, Lmax, d, seed=seed, tensor_id=tid, outliers=False, dtype=dtype)
    Q, K, V = mk(W.TID_Q), mk(W.TID_K), mk(W.TID_V)
    lens_t = torch.tensor(lens, dtype=torch.int32)
    O = torch.full((B, H, Lmax, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, H, Lmax), 7.0, dtype=torch.float32, device=DEV)
    fb.fedrag_partial_attn_varlen(Q.to(DEV), K.to(DEV), V.to(DEV), lens_t.to(DEV), O_part=O, lse=lse,
                                  q_lens=lens_t.to(DEV))
    torch.cuda.synchronize()
    Or, lr = oracle.partial_attn_varlen(Q, K, V, lens_t)
    for b, n in enumerate(lens):
        if n:
            PT.check_attn(O[b:b + 1, :, :n], lse[b:b + 1, :, :n], Or[b:b + 1, :, :n], lr[b:b + 1, :, :n], dtype, f"seq {b}")
        assert bool((O[b, :, n:] == 7.0).all()) and bool((lse[b, :, n:] == 7.0).all()), "padding rows were written"


@pytest.mark.parametrize("L", [100, 3000])
def test_query_lengths_decode_shape(oracle, L):
    """Per-sequence query counts on a decode-shaped call (G * L_q <= 16: the streaming kernel, with L = 3000 also its
    key runs and their aggregation): rows past a sequence's count keep what they held."""
    dtype = torch.bfloat16
    B, Hq, Hkv, d, Lq = 4, 8, 2, 128, 4
    q_lens, kv_lens = [4, 2, 0, 3], [L, L // 3, 17, 0]
    seed = 4242
    mk = lambda H, n, tid: W.activations(B, H, n, d, seed=seed, tensor_id=tid, outliers=False, dtype=dtype)
    Q, K, V = mk(Hq, Lq, W.TID_Q), mk(Hkv, L, W.TID_K), mk(Hkv, L, W.TID_V)
    ql, kl = torch.tensor(q_lens, dtype=torch.int32), torch.tensor(kv_lens, dtype=torch.int32)
    O = torch.full((B, Hq, Lq, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq, Lq), 7.0, dtype=torch.float32, device=DEV)
    fb.fedrag_partial_attn_varlen(Q.to(DEV), K.to(DEV), V.to(DEV), kl.to(DEV), O_part=O, lse=lse, q_lens=ql.to(DEV))
    torch.cuda.synchronize()
    Or, lr = oracle.partial_attn_varlen(Q, K, V, kl)
    for b, n in enumerate(q_lens):
        if n:
            PT.check_attn(O[b:b + 1, :, :n], lse[b:b + 1, :, :n], Or[b:b + 1, :, :n], lr[b:b + 1, :, :n], dtype, f"seq {b}")
        assert bool((O[b, :, n:] == 7.0).all()) and bool((lse[b, :, n:] == 7.0).all()), "padding rows were written"
