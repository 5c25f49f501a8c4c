"""GPU parity of fedrag_partial_attn_shards: the per-shard computation and its aggregation (Section 4.1) in one
call, against the oracle's per-shard attention followed by the oracle's aggregation, and against the oracle's
attention over the concatenated keys (what Section 4.1 proves the aggregation equals)."""
import ctypes

import numpy as np
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"

CASES = [
    # name, B, Hq, Hkv, d, Lq, shard lengths, dtype
    ("dec_bf16", 2, 8, 2, 128, 1, [1000, 0, 333, 5001], "bf16"),       # decode kernel, an empty shard, ragged tails
    ("dec_bf16_rows16_d64", 1, 8, 2, 64, 4, [300, 37], "bf16"),
    ("dec_f16_many", 1, 4, 1, 128, 1, [130] * 16, "f16"),              # the maximum number of shards
    ("pre_bf16", 1, 4, 2, 128, 70, [1500, 64, 0, 700], "bf16"),        # prefill kernel, runs inside the long shards
    ("pre_bf16_d64", 2, 2, 2, 64, 300, [1111, 129], "bf16"),
    ("pre_f16", 1, 2, 1, 128, 40, [100, 777], "f16"),
    # enough query tiles to cover the chip: one run per shard
    ("pre_bf16_walk", 4, 8, 2, 128, 1100, [200, 0, 333], "bf16"),
    ("f32", 2, 4, 2, 128, 3, [197, 0, 50], "f32"),
    # prefill shapes where all shards together plan one run per shard (so the call launches shard by shard) while a
    # shard alone would be cut into runs: the per-shard launches must not cut, the workspace holds the shards' partials
    ("pre_bf16_two_shards_one_run_each", 1, 32, 8, 64, 1024, [1024, 1024], "bf16"),
    ("pre_bf16_16_shards_one_run_each", 2, 32, 8, 64, 64, [512] * 16, "bf16"),
    ("pre_f16_4_shards_one_run_each", 1, 32, 8, 128, 512, [1024] * 4, "f16"),
]


def make(B, Hq, Hkv, d, Lq, Ls, dt, seed=77):
    dtype = W.torch_dtype(dt)
    mk = lambda H, L, tid: W.activations(B, H, L, d, seed=seed, tensor_id=tid, outliers=False, dtype=dtype)
    Q = mk(Hq, Lq, W.TID_Q)
    Ks = [mk(Hkv, L, W.TID_K + 16 * (i + 1)) for i, L in enumerate(Ls)]
    Vs = [mk(Hkv, L, W.TID_V + 16 * (i + 1)) for i, L in enumerate(Ls)]
    return dtype, Q, Ks, Vs


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_shards_equal_per_shard_then_merge_and_concatenation(oracle, case):
    name, B, Hq, Hkv, d, Lq, Ls, dt = case
    dtype, Q, Ks, Vs = make(B, Hq, Hkv, d, Lq, Ls, dt)
    O, lse = fb.fedrag_partial_attn_shards(Q.to(DEV), [k.to(DEV) for k in Ks], [v.to(DEV) for v in Vs])
    torch.cuda.synchronize()
    # oracle, stage by stage
    parts = [oracle.partial_attn(Q, k, v) for k, v in zip(Ks, Vs)]
    Or, lr = oracle.lse_merge(np.stack([p[0] for p in parts]), np.stack([p[1] for p in parts]))
    PT.check_attn(O, lse, Or, lr, dtype, name + " vs per-shard + merge")
    # oracle, eq. (1) over all keys at once
    Oc, lc = oracle.partial_attn(Q, torch.cat(Ks, dim=2), torch.cat(Vs, dim=2))
    PT.check_attn(O, lse, Oc, lc, dtype, name + " vs concatenated keys")


def test_planner_geometries_launch_shard_by_shard():
    """The three cases above exist for one geometry: more than one run for a shard on its own, one run per shard for
    all of them together.  The workspace sizes say which plan the library made."""
    for (B, Hq, Hkv, d, Lq, Ls) in [(1, 32, 8, 64, 1024, [1024, 1024]), (2, 32, 8, 64, 64, [512] * 16),
                                     (1, 32, 8, 128, 512, [1024] * 4)]:
        per_part = B * Hq * Lq * (d + 1) * 4
        alone = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, torch.bfloat16, Lq, Ls[0])
        together = fb.fedrag_partial_attn_shards_workspace_bytes(B, Hq, Hkv, d, torch.bfloat16, Lq, Ls)
        assert alone >= 2 * per_part, "a shard alone is no longer cut into runs: pick another geometry"
        assert together == len(Ls) * per_part, "all shards together no longer plan one run per shard"


def test_one_shard_is_partial_attn_bit_for_bit():
    for (B, Hq, Hkv, d, Lq, L, dt) in [(2, 8, 2, 128, 1, 5001, "bf16"), (1, 4, 2, 128, 70, 1500, "bf16")]:
        dtype, Q, Ks, Vs = make(B, Hq, Hkv, d, Lq, [L], dt)
        Qd, Kd, Vd = Q.to(DEV), Ks[0].to(DEV), Vs[0].to(DEV)
        O1, l1 = fb.fedrag_partial_attn(Qd, Kd, Vd)
        O2, l2 = fb.fedrag_partial_attn_shards(Qd, [Kd], [Vd])
        torch.cuda.synchronize()
        assert torch.equal(O1, O2) and torch.equal(l1, l2)


def test_all_shards_empty():
    dtype, Q, Ks, Vs = make(1, 4, 2, 128, 5, [0, 0], "bf16")
    O, lse = fb.fedrag_partial_attn_shards(Q.to(DEV), [k.to(DEV) for k in Ks], [v.to(DEV) for v in Vs])
    torch.cuda.synchronize()
    assert bool((O == 0).all()) and bool(torch.isneginf(lse).all())


def test_workspace_too_small_is_refused():
    dtype, Q, Ks, Vs = make(1, 8, 2, 128, 1, [4096, 4096], "bf16")
    ws = torch.empty(64, dtype=torch.uint8, device=DEV)
    with pytest.raises(fb.FedragError) as e:
        fb.fedrag_partial_attn_shards(Q.to(DEV), [k.to(DEV) for k in Ks], [v.to(DEV) for v in Vs], workspace=ws)
    assert e.value.status == fb.ERR_WORKSPACE


def test_two_compute_nodes_compose(oracle):
    """Section 5.4: when every node supplies tokens the Compute Node role is given to two nodes, each holding the
    shards of some Context Owners; the Inquirer aggregates their two results.  Two calls on disjoint shard sets
    followed by fedrag_lse_merge equal one call on all shards (to rounding) and the oracle's attention over all keys."""
    B, Hq, Hkv, d, Lq, Ls, dt = 2, 8, 2, 128, 1, [700, 1300, 512, 2049], "bf16"
    dtype, Q, Ks, Vs = make(B, Hq, Hkv, d, Lq, Ls, dt, seed=91)
    Qd = Q.to(DEV)
    Kd, Vd = [k.to(DEV) for k in Ks], [v.to(DEV) for v in Vs]
    Oa, la = fb.fedrag_partial_attn_shards(Qd, Kd[:2], Vd[:2])       # first Compute Node
    Ob, lb = fb.fedrag_partial_attn_shards(Qd, Kd[2:], Vd[2:])       # second Compute Node
    O2, l2 = fb.fedrag_lse_merge(torch.stack([Oa, Ob]), torch.stack([la, lb]), n_kv_heads=Hkv)
    O1, l1 = fb.fedrag_partial_attn_shards(Qd, Kd, Vd)
    torch.cuda.synchronize()
    assert float((O1 - O2).abs().max()) <= 1e-5 and float((l1 - l2).abs().max()) <= 1e-5
    Oc, lc = oracle.partial_attn(Q, torch.cat(Ks, dim=2), torch.cat(Vs, dim=2))
    PT.check_attn(O2, l2, Oc, lc, dtype, "two compute nodes")
