"""Degenerate sizes through every call on the GPU: no queries, no keys, one row.  Nothing may fault, outputs that
exist get the documented values (O = 0, lse = -inf for attention over no keys)."""
import numpy as np
import pytest
import torch

from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("dt", ["bf16", "f32"])
def test_zero_queries_and_zero_keys(dt):
    dtype = W.torch_dtype(dt)
    B, Hq, Hkv, d = 2, 4, 2, 128
    keys = W.make_keys(Hkv, d, 1, 8, 1, seed=5, dtype=dtype)
    z = lambda H, L: torch.zeros((B, H, L, d), dtype=dtype, device=DEV)
    phi = lambda n: getattr(keys, n).to(DEV)
    # no rows at all
    assert fb.fedrag_scramble_q(z(Hq, 0), phi("phi_q"), None).shape == (B, Hq, 0, d)
    Ks, Vs = fb.fedrag_scramble_kv(z(Hkv, 0), z(Hkv, 0), phi("phi_k"), phi("phi_v"), None, n_q_heads=Hq)
    assert Ks.shape == (B, Hkv, 0, d) and Vs.shape == (B, Hkv, 0, d)
    O, lse = fb.fedrag_partial_attn(z(Hq, 0), z(Hkv, 5), z(Hkv, 5))
    assert O.shape == (B, Hq, 0, d) and lse.shape == (B, Hq, 0)
    # queries but no keys: the empty partial
    for Lq in (1, 70):
        O, lse = fb.fedrag_partial_attn(z(Hq, Lq), z(Hkv, 0), z(Hkv, 0))
        O2, lse2 = fb.fedrag_partial_attn_shards(z(Hq, Lq), [z(Hkv, 0), z(Hkv, 0)], [z(Hkv, 0), z(Hkv, 0)])
        torch.cuda.synchronize()
        for o, l in ((O, lse), (O2, lse2)):
            assert bool((o == 0).all()) and bool(torch.isneginf(l).all())
    # the aggregation of empty partials stays empty, Dec of no rows is a no-op
    Op = torch.zeros((3, B, Hq, 2, d), device=DEV)
    lp = torch.full((3, B, Hq, 2), -np.inf, device=DEV)
    Om, lm = fb.fedrag_lse_merge(Op, lp, n_kv_heads=Hkv)
    torch.cuda.synchronize()
    assert bool((Om == 0).all()) and bool(torch.isneginf(lm).all())
    out = fb.fedrag_unscramble(torch.zeros((B, Hq, 0, d), device=DEV), phi("phi_v_inv"), None)
    assert out.shape == (B, Hq, 0, d)
    torch.cuda.synchronize()


def test_single_row_everything():
    """One sequence, one head, one query, one key: every kernel at its smallest non-empty size."""
    dtype = torch.bfloat16
    d = 64
    keys = W.make_keys(1, d, 1, 1, 1, seed=6, dtype=dtype)
    g = torch.Generator().manual_seed(3)
    Q = torch.randn((1, 1, 1, d), generator=g).to(dtype).to(DEV)
    K = torch.randn((1, 1, 1, d), generator=g).to(dtype).to(DEV)
    V = torch.randn((1, 1, 1, d), generator=g).to(dtype).to(DEV)
    Qs = fb.fedrag_scramble_q(Q, keys.phi_q.to(DEV), None)
    Ks, Vs = fb.fedrag_scramble_kv(K, V, keys.phi_k.to(DEV), keys.phi_v.to(DEV), None, n_q_heads=1)
    O, lse = fb.fedrag_partial_attn(Qs, Ks, Vs)
    out = fb.fedrag_unscramble(O, keys.phi_v_inv.to(DEV), None)
    torch.cuda.synchronize()
    # one key: the output is that key's value row, whatever the score
    assert float((O - Vs.float()).abs().max()) == 0.0
    assert float((out - V.float()).abs().max()) <= 2e-2
    assert np.isfinite(float(lse))


def test_zero_sequences():
    """batch = 0 is a legal shape: every call returns at once and writes nothing."""
    dtype = torch.bfloat16
    Hq, Hkv, d = 4, 2, 128
    keys = W.make_keys(Hkv, d, 3, 8, 1, seed=5, dtype=dtype)
    z = lambda H, L: torch.zeros((0, H, L, d), dtype=dtype, device=DEV)
    phi = lambda n: getattr(keys, n).to(DEV)
    assert fb.fedrag_scramble_q(z(Hq, 3), phi("phi_q"), None).shape == (0, Hq, 3, d)
    Ks, Vs = fb.fedrag_scramble_kv(z(Hkv, 8), z(Hkv, 8), phi("phi_k"), phi("phi_v"), None, n_q_heads=Hq)
    assert Ks.shape == (0, Hkv, 8, d)
    for Lq in (1, 300):  # decode kernel and prefill kernel
        O, lse = fb.fedrag_partial_attn(z(Hq, Lq), z(Hkv, 8), z(Hkv, 8))
        assert O.shape == (0, Hq, Lq, d) and lse.shape == (0, Hq, Lq)
        O, lse = fb.fedrag_partial_attn_shards(z(Hq, Lq), [z(Hkv, 8), z(Hkv, 5)], [z(Hkv, 8), z(Hkv, 5)])
        assert O.shape == (0, Hq, Lq, d)
        O, lse = fb.fedrag_local_attn(z(Hq, Lq), z(Hkv, 300), z(Hkv, 300))
        assert O.shape == (0, Hq, Lq, d)
    Om, lm = fb.fedrag_lse_merge(torch.zeros((2, 0, Hq, 3, d), device=DEV), torch.zeros((2, 0, Hq, 3), device=DEV),
                                 n_kv_heads=Hkv)
    assert Om.shape == (0, Hq, 3, d)
    out = fb.fedrag_unscramble(torch.zeros((0, Hq, 3, d), device=DEV), phi("phi_v_inv"), None)
    assert out.shape == (0, Hq, 3, d)
    torch.cuda.synchronize()


def test_validate_perm_flags():
    """The debug check of a token permutation: 0 for permutations, bit 0 for an index out of range, bit 1 for a repeat."""
    L = 5000
    g = torch.Generator().manual_seed(11)
    good = torch.stack([torch.randperm(L, generator=g) for _ in range(3)]).to(torch.int32)
    cases = {"good": (good, 0)}
    bad = good.clone(); bad[1, 17] = L
    cases["too_large"] = (bad, 1)
    bad = good.clone(); bad[2, 0] = -1
    cases["negative"] = (bad, 1)
    bad = good.clone(); bad[0, 5] = bad[0, 6]
    cases["repeat"] = (bad, 2)
    bad = good.clone(); bad[0, 5] = bad[0, 6]; bad[2, 9] = L + 3
    cases["both"] = (bad, 3)
    cases["one_row"] = (good[0].contiguous(), 0)
    # a row that is a permutation of another row's range only as a whole tensor: rows are checked one by one
    two = torch.stack([torch.arange(4), torch.tensor([0, 1, 2, 2])]).to(torch.int32)
    cases["second_row_repeats"] = (two, 2)
    for name, (perm, want) in cases.items():
        flag = fb.fedrag_validate_perm(perm.to(DEV))
        torch.cuda.synchronize()
        assert int(flag.item()) == want, name
    assert int(fb.fedrag_validate_perm(torch.zeros((1, 0), dtype=torch.int32, device=DEV)).item()) == 0
