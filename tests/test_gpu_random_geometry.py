"""GPU parity of the attention calls over seeded random geometries (Section 4.1: per-shard computation and
aggregation; Section 5.2: padded batches).  The fixed cases elsewhere were chosen by hand around the kernels' tile
sizes; these draw batch, head counts, group size, head dimension, query count, shard count and shard lengths at
random, so that the host-side dispatch (streaming kernel or tiled kernel, runs inside a shard, one launch or a
launch per shard, workspace layout) is exercised on combinations nobody picked.  Every case is compared with the
oracle's per-shard attention followed by its aggregation."""
import numpy as np
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"

LQ_CHOICES = [1, 1, 1, 2, 3, 4, 7, 16, 17, 33, 64, 100, 129, 256, 257, 300, 513]


def draw(seed):
    rng = np.random.default_rng(0xFED2A6 + seed)
    dt = ["bf16", "bf16", "f16", "f32"][rng.integers(4)]
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    Lq = int(rng.choice(LQ_CHOICES))
    B = int(rng.choice([1, 1, 2, 3, 5]))
    wide = rng.random() < 0.15
    if wide:  # as many (sequence, KV head) units as the chip has compute units, or more
        B, Hkv, Lq = int(rng.choice([32, 40, 64, 70])), 8, int(rng.choice([1, 1, 2]))
        G = min(G, 16 // Lq)
    n = int(rng.choice([1, 1, 2, 3, 4, 8]))
    top = int(rng.choice([40, 200, 700, 2100]))
    Ls = [int(rng.integers(0, top + 1)) for _ in range(n)]
    if rng.random() < 0.2:
        Ls[int(rng.integers(n))] = 0
    # keep the oracle's work per case small: rows x keys
    while B * Hkv * G * Lq * max(1, sum(Ls)) > 6e7 and B > 1 and not wide:
        B -= 1
    while B * Hkv * G * Lq * max(1, sum(Ls)) > 6e7:
        Ls = [L // 2 for L in Ls]
    if dt == "f32":  # one wave per query row: keep the row count down
        Lq = min(Lq, 33)
    return dict(dt=dt, d=d, Hkv=Hkv, Hq=Hkv * G, Lq=Lq, B=B, Ls=Ls)


@pytest.mark.parametrize("seed", range(48))
def test_shards_call_on_a_random_geometry(oracle, seed):
    c = draw(seed)
    dtype = W.torch_dtype(c["dt"])
    # N(0, 1) operands, as Q', K', V' are after Enc has spread the outlier channels over a head (the tiled kernel
    # feeds P to the second product as one storage-type term: its output error grows with max |V'|; operands with
    # concentrated outliers enter the attention tests through Enc, as they do in the protocol)
    mk = lambda H, L, tid: W.activations(c["B"], H, L, c["d"], seed=1000 + seed, tensor_id=tid, outliers=False,
                                         dtype=dtype)
    Q = mk(c["Hq"], c["Lq"], W.TID_Q)
    Ks = [mk(c["Hkv"], L, W.TID_K + 16 * (i + 1)) for i, L in enumerate(c["Ls"])]
    Vs = [mk(c["Hkv"], L, W.TID_V + 16 * (i + 1)) for i, L in enumerate(c["Ls"])]
    print(f"seed {seed}: {c}", flush=True)
    Qd, Kd, Vd = Q.to(DEV), [k.to(DEV) for k in Ks], [v.to(DEV) for v in Vs]
    O, lse = fb.fedrag_partial_attn_shards(Qd, Kd, Vd)
    torch.cuda.synchronize()
    parts = [oracle.partial_attn(Q, k, v) for k, v in zip(Ks, Vs)]
    Or, lr = oracle.lse_merge(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]))
    PT.check_attn(O, lse, Or, lr, dtype, f"seed {seed} {c}")
    # a single shard through the plain call as well (its own plan: runs inside the shard)
    j = int(np.argmax(c["Ls"]))
    O1, l1 = fb.fedrag_partial_attn(Qd, Kd[j], Vd[j])
    torch.cuda.synchronize()
    PT.check_attn(O1, l1, parts[j][0], parts[j][1], dtype, f"seed {seed} shard {j} alone {c}")


@pytest.mark.parametrize("seed", range(16))
def test_padded_batch_on_a_random_geometry(oracle, seed):
    """fedrag_partial_attn_varlen with random key counts (and, every other seed, query counts) per sequence; the
    padding is poisoned with NaN."""
    rng = np.random.default_rng(0x5EED + seed)
    dt = ["bf16", "f16"][seed % 2]
    dtype = W.torch_dtype(dt)
    d = int(rng.choice([64, 128]))
    Hkv, G = int(rng.choice([1, 2, 4])), int(rng.choice([1, 2, 4]))
    B = int(rng.integers(1, 6))
    Lq = int(rng.choice([1, 2, 4, 9, 40, 130, 300]))
    L = int(rng.choice([33, 64, 200, 777, 1500]))
    kv = rng.integers(0, L + 1, size=B).astype(np.int32)
    ql = rng.integers(1, Lq + 1, size=B).astype(np.int32) if seed % 2 else None
    Q = W.activations(B, Hkv * G, Lq, d, seed=2000 + seed, tensor_id=W.TID_Q, outliers=False, dtype=dtype)
    K = W.activations(B, Hkv, L, d, seed=2000 + seed, tensor_id=W.TID_K, outliers=False, dtype=dtype)
    V = W.activations(B, Hkv, L, d, seed=2000 + seed, tensor_id=W.TID_V, outliers=False, dtype=dtype)
    print(f"seed {seed}: dt={dt} d={d} Hkv={Hkv} G={G} B={B} Lq={Lq} L={L} kv={kv.tolist()} ql={None if ql is None else ql.tolist()}", flush=True)
    Kp, Vp, Qp = K.clone(), V.clone(), Q.clone()
    for b in range(B):
        Kp[b, :, kv[b]:] = float("nan")
        Vp[b, :, kv[b]:] = float("nan")
        if ql is not None:
            Qp[b, :, ql[b]:] = float("nan")
    sentinel = -7.25
    O = torch.full((B, Hkv * G, Lq, d), sentinel, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hkv * G, Lq), sentinel, dtype=torch.float32, device=DEV)
    fb.fedrag_partial_attn_varlen(Qp.to(DEV), Kp.to(DEV), Vp.to(DEV), torch.from_numpy(kv).to(DEV),
                                  q_lens=None if ql is None else torch.from_numpy(ql).to(DEV), O_part=O, lse=lse)
    torch.cuda.synchronize()
    Or, lr = oracle.partial_attn_varlen(Q, K, V, kv)
    for b in range(B):
        nq = Lq if ql is None else int(ql[b])
        PT.check_attn(O[b:b + 1, :, :nq], lse[b:b + 1, :, :nq], Or[b:b + 1, :, :nq], lr[b:b + 1, :, :nq], dtype,
                      f"seed {seed} sequence {b}")
        if nq < Lq:  # padding query rows are left as they were
            assert bool((O[b, :, nq:] == sentinel).all()) and bool((lse[b, :, nq:] == sentinel).all())
