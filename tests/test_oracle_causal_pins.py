"""Pins for the oracle's Inquirer-local attention (Section 5.3: a token attends to itself and the tokens before it)
and for the way Section 4.1 splits a decoder layer's attention into that local part plus the remote partials.
Runs without a GPU."""
import math

import numpy as np
import pytest
import torch


def rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


@pytest.mark.parametrize("Lq,Lk,d", [(1, 1, 2), (3, 3, 2), (2, 5, 3), (4, 4, 4)])
def test_brute_force_tiny(oracle, Lq, Lk, d):
    Q, K, V = rand(1, 1, 2, Lq, d), rand(2, 1, 1, Lk, d), rand(3, 1, 1, Lk, d)
    O, lse = oracle.local_causal_attn(Q, K, V)
    off = Lk - Lq
    for h in range(2):
        for i in range(Lq):
            e = [math.exp(sum(Q[0, h, i, c] * K[0, 0, t, c] for c in range(d)) / math.sqrt(d)) for t in range(i + off + 1)]
            tot = sum(e)
            for c in range(d):
                assert O[0, h, i, c] == pytest.approx(sum(e[t] * V[0, 0, t, c] for t in range(i + off + 1)) / tot, rel=1e-12)
            assert lse[0, h, i] == pytest.approx(math.log(tot), rel=1e-12, abs=1e-12)


def test_each_row_is_unmasked_attention_over_its_prefix(oracle):
    B, Hq, Hkv, Lq, Lk, d = 2, 4, 2, 7, 19, 8
    Q, K, V = rand(4, B, Hq, Lq, d), rand(5, B, Hkv, Lk, d), rand(6, B, Hkv, Lk, d)
    O, lse = oracle.local_causal_attn(Q, K, V)
    for i in range(Lq):
        n = i + (Lk - Lq) + 1
        Oi, li = oracle.partial_attn(Q[:, :, i:i + 1], K[:, :, :n], V[:, :, :n])
        np.testing.assert_allclose(O[:, :, i:i + 1], Oi, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lse[:, :, i:i + 1], li, rtol=1e-13, atol=1e-15)


def test_library_causal_attention_agrees(oracle):
    B, H, L, d = 2, 3, 33, 16
    Q, K, V = (torch.from_numpy(rand(s, B, H, L, d)) for s in (7, 8, 9))
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
    O, lse = oracle.local_causal_attn(Q, K, V)
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-10, atol=1e-12)
    s = (Q @ K.transpose(-1, -2)) / math.sqrt(d)
    s = s.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=1e-12)


def test_single_decoding_query_sees_everything(oracle):
    Q, K, V = rand(10, 1, 2, 1, 8), rand(11, 1, 1, 13, 8), rand(12, 1, 1, 13, 8)
    O, lse = oracle.local_causal_attn(Q, K, V)
    O2, lse2 = oracle.partial_attn(Q, K, V)
    np.testing.assert_array_equal(O, O2)
    np.testing.assert_array_equal(lse, lse2)


def test_segment_split_of_a_decoder_layer(oracle):
    """Section 5.3 prefill of segment T_3: remote partials over the earlier segments T_1, T_2 (no mask), the local
    part over T_3 itself, aggregated as in Section 4.1, equal attention with the usual mask over the whole sequence."""
    B, Hq, Hkv, d = 1, 4, 2, 8
    L1, L2, L3 = 11, 6, 9
    K = rand(20, B, Hkv, L1 + L2 + L3, d)
    V = rand(21, B, Hkv, L1 + L2 + L3, d)
    Qall = rand(22, B, Hq, L1 + L2 + L3, d)
    full, full_lse = oracle.local_causal_attn(Qall, K, V)       # the whole sequence at once
    Q3 = Qall[:, :, L1 + L2:]
    parts, lses = [], []
    for a, b in ((0, L1), (L1, L1 + L2)):
        o, l = oracle.partial_attn(Q3, K[:, :, a:b], V[:, :, a:b])
        parts.append(o); lses.append(l)
    o, l = oracle.local_causal_attn(Q3, K[:, :, L1 + L2:], V[:, :, L1 + L2:])
    parts.append(o); lses.append(l)
    O, lse = oracle.lse_merge(np.stack(parts), np.stack(lses))
    np.testing.assert_allclose(O, full[:, :, L1 + L2:], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, full_lse[:, :, L1 + L2:], rtol=1e-12)


def test_planted_off_by_one_is_caught(oracle):
    """Seeing one key too few or too many changes the first row: with Lq = Lk the first query sees exactly one key."""
    Q, K, V = rand(30, 1, 1, 4, 4), rand(31, 1, 1, 4, 4), rand(32, 1, 1, 4, 4)
    O, lse = oracle.local_causal_attn(Q, K, V)
    np.testing.assert_allclose(O[0, 0, 0], V[0, 0, 0], rtol=1e-14)
    assert lse[0, 0, 0] == pytest.approx(float(Q[0, 0, 0] @ K[0, 0, 0]) / 2.0, rel=1e-13)
    assert np.abs(O[0, 0, 1] - V[0, 0, 1]).max() > 1e-3        # the second row mixes two keys
