"""Pins for the oracle's attention over a padded batch of sequences of unequal length (the re-ranking workload of
Section 5.2: several query-document pairs, each a sequence of its own).  Runs without a GPU."""
import math

import numpy as np
import pytest
import torch


def rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_brute_force_tiny(oracle):
    B, H, Lq, Lk, d = 3, 2, 2, 4, 3
    Q, K, V = rand(1, B, H, Lq, d), rand(2, B, 1, Lk, d), rand(3, B, 1, Lk, d)
    lens = np.array([4, 1, 0], np.int32)
    O, lse = oracle.partial_attn_varlen(Q, K, V, lens)
    for b in range(B):
        for h in range(H):
            for i in range(Lq):
                n = int(lens[b])
                if n == 0:
                    assert np.all(O[b, h, i] == 0) and lse[b, h, i] == -np.inf
                    continue
                e = [math.exp(sum(Q[b, h, i, c] * K[b, 0, t, c] for c in range(d)) / math.sqrt(d)) for t in range(n)]
                for c in range(d):
                    assert O[b, h, i, c] == pytest.approx(sum(e[t] * V[b, 0, t, c] for t in range(n)) / sum(e), rel=1e-12)
                assert lse[b, h, i] == pytest.approx(math.log(sum(e)), rel=1e-12, abs=1e-12)


def test_library_attention_with_a_key_padding_mask_agrees(oracle):
    B, H, Lq, Lk, d = 4, 3, 9, 21, 16
    Q, K, V = (torch.from_numpy(rand(s, B, H, L, d)) for s, L in ((4, Lq), (5, Lk), (6, Lk)))
    lens = torch.tensor([21, 7, 1, 13], dtype=torch.int32)
    mask = (torch.arange(Lk)[None, :] < lens[:, None])[:, None, None, :]          # True = attend
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask)
    O, lse = oracle.partial_attn_varlen(Q, K, V, lens)
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-10, atol=1e-12)
    s = (Q @ K.transpose(-1, -2)) / math.sqrt(d)
    s = s.masked_fill(~mask, float("-inf"))
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=1e-12)


def test_padding_rows_do_not_matter_and_full_length_is_the_dense_call(oracle):
    B, H, Lq, Lk, d = 2, 2, 3, 10, 8
    Q, K, V = rand(7, B, H, Lq, d), rand(8, B, H, Lk, d), rand(9, B, H, Lk, d)
    lens = np.array([6, 10], np.int32)
    O, lse = oracle.partial_attn_varlen(Q, K, V, lens)
    K2, V2 = K.copy(), V.copy()
    K2[0, :, 6:] = 1e6; V2[0, :, 6:] = -1e6                       # garbage in the padding
    O2, lse2 = oracle.partial_attn_varlen(Q, K2, V2, lens)
    np.testing.assert_array_equal(O, O2); np.testing.assert_array_equal(lse, lse2)
    Of, lf = oracle.partial_attn(Q, K, V)
    np.testing.assert_array_equal(O[1], Of[1]); np.testing.assert_array_equal(lse[1], lf[1])
    assert np.abs(O[0] - Of[0]).max() > 1e-3                       # the shorter sequence differs from the dense call
