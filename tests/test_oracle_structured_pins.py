"""Pins for the oracle's structured transform (Section 4.2, "Our construction", Phi = S1 P1 H P2 S2).

The oracle applies the factors one after the other and never forms Phi.  Here it is held to what fixes it from
outside: the matrix product of the five factors written out with a library Hadamard matrix, hand-expanded cases at
d = 2 and d = 4, the orthogonality of H, Lemma 1 and Lemma 2 of Section 4.2, Dec undoing Enc, and the protocol with
structured keys reproducing eq. (1).  Runs without a GPU.
"""
import numpy as np
import pytest
import torch
from scipy.linalg import hadamard

from paper_2605_25716_amd import workloads as W


def np_key(key):
    a, g1, g2, b = key
    return a.double().numpy(), g1.numpy(), g2.numpy(), b.double().numpy()


def dense_from_factors(a, g1, g2, b):
    """S1 P1 H P2 S2 as a product of explicit matrices; (x P)[j] = x[g[j]] means P[g[j], j] = 1."""
    d = a.shape[0]
    P1 = np.zeros((d, d)); P1[g1, np.arange(d)] = 1.0
    P2 = np.zeros((d, d)); P2[g2, np.arange(d)] = 1.0
    return np.diag(a) @ P1 @ (hadamard(d) / np.sqrt(d)) @ P2 @ np.diag(b)


@pytest.mark.parametrize("d", [2, 4, 16, 64, 128])
def test_equals_product_of_the_five_factors(oracle, d):
    Hkv, H = 2, 4
    ks = W.make_structured_keys(Hkv, d, 5, 9, 1, seed=10 + d, dtype=torch.float32)
    X = np.random.default_rng(d).standard_normal((2, H, 9, d))
    for key in (ks.q, ks.k, ks.v, ks.v_inv):
        Y = oracle.structured(X, key)
        a, g1, g2, b = np_key(key)
        for h in range(H):
            Phi = dense_from_factors(a[h // 2], g1[h // 2], g2[h // 2], b[h // 2])
            np.testing.assert_allclose(Y[:, h], X[:, h] @ Phi, rtol=0, atol=1e-12 * np.abs(Y).max())
        # and the dense oracle path (pinned on its own) agrees when handed the multiplied-out matrix
        Phi_all = np.stack([dense_from_factors(a[g], g1[g], g2[g], b[g]) for g in range(Hkv)])
        np.testing.assert_allclose(Y, oracle.scramble(X, Phi_all), rtol=0, atol=1e-12 * np.abs(Y).max())


def test_hand_expanded_d2(oracle):
    # d = 2: H = [[1, 1], [1, -1]] / sqrt(2); key a = (2, -3), g1 = (1, 0), g2 = (0, 1), b = (5, 7)
    x = np.array([[[[0.5, -1.25]]]])
    key = (np.array([[2.0, -3.0]]), np.array([[1, 0]], np.int32), np.array([[0, 1]], np.int32), np.array([[5.0, 7.0]]))
    u = (0.5 * 2.0, -1.25 * -3.0)            # x S1
    v = (u[1], u[0])                         # gather by g1
    w = ((v[0] + v[1]) / np.sqrt(2), (v[0] - v[1]) / np.sqrt(2))
    y = (w[0] * 5.0, w[1] * 7.0)
    np.testing.assert_allclose(oracle.structured(x, key)[0, 0, 0], y, rtol=1e-15)


def test_hand_expanded_d4_signs(oracle):
    # identity scales and permutations: row m of the output is sum_i x_i (-1)^{popcount(i & m)} / 2
    x = np.array([[[[1.0, 10.0, 100.0, 1000.0]]]])
    one, idt = np.ones((1, 4)), np.arange(4, dtype=np.int32)[None]
    y = oracle.structured(x, (one, idt, idt, one))[0, 0, 0]
    np.testing.assert_allclose(y, np.array([1111.0, 1 - 10 + 100 - 1000, 1 + 10 - 100 - 1000, 1 - 10 - 100 + 1000]) / 2)


@pytest.mark.parametrize("d", [8, 128])
def test_hadamard_factor_is_an_orthogonal_involution(oracle, d):
    one, idt = np.ones((1, d)), np.arange(d, dtype=np.int32)[None]
    X = np.random.default_rng(1).standard_normal((1, 1, 6, d))
    Y = oracle.structured(X, (one, idt, idt, one))
    np.testing.assert_allclose(np.linalg.norm(Y, axis=-1), np.linalg.norm(X, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(oracle.structured(Y, (one, idt, idt, one)), X, atol=1e-13)


@pytest.mark.parametrize("use_s2", [True, False])
def test_lemma1_inner_products_survive(oracle, use_s2):
    d, Hkv = 64, 2
    ks = W.make_structured_keys(Hkv, d, 4, 11, 1, seed=77, dtype=torch.float32, use_s2=use_s2)
    r = np.random.default_rng(5)
    x, y = r.standard_normal((1, Hkv, 4, d)), r.standard_normal((1, Hkv, 11, d))
    xs, ys = oracle.structured(x, ks.q), oracle.structured(y, ks.k)
    np.testing.assert_allclose(xs @ ys.transpose(0, 1, 3, 2), x @ y.transpose(0, 1, 3, 2), atol=1e-5)
    if not use_s2:
        assert (ks.q[3] == 1).all() and (ks.k[3] == 1).all()


def test_lemma2_linearity_and_dec_undoes_enc(oracle):
    d, Hkv = 32, 1
    ks = W.make_structured_keys(Hkv, d, 6, 6, 1, seed=5, dtype=torch.float32)
    r = np.random.default_rng(9)
    V = r.standard_normal((1, 1, 6, d))
    A = r.standard_normal((6, 6))
    lhs = A @ oracle.structured(V, ks.v)[0, 0]
    rhs = oracle.structured((A @ V[0, 0])[None, None], ks.v)[0, 0]
    np.testing.assert_allclose(lhs, rhs, atol=1e-10)
    back = oracle.structured(oracle.structured(V, ks.v), ks.v_inv)
    np.testing.assert_allclose(back, V, atol=2e-5)   # 1/a, 1/b are carried in fp32


def test_row_gather_and_scatter_are_inverse(oracle):
    d = 16
    ks = W.make_structured_keys(1, d, 9, 9, 1, seed=6, dtype=torch.float32)
    X = np.random.default_rng(2).standard_normal((2, 1, 9, d))
    perm = ks.perm_q.numpy()
    Y = oracle.structured(X, ks.v, perm)                      # row j <- row perm[j]
    np.testing.assert_allclose(Y, oracle.structured(X, ks.v)[:, :, perm], atol=0)
    Z = oracle.structured(Y, ks.v_inv, perm, scatter=True)    # row perm[i] <- row i
    np.testing.assert_allclose(Z, X, atol=2e-5)


def test_protocol_with_structured_keys_is_plain_attention(oracle):
    B, Hq, Hkv, d, Lq, L, S = 2, 4, 2, 32, 5, 23, 3
    ks = W.make_structured_keys(Hkv, d, Lq, L, S, seed=12, dtype=torch.float32)
    r = np.random.default_rng(3)
    Q = r.standard_normal((B, Hq, Lq, d))
    Ks = [r.standard_normal((B, Hkv, L, d)) for _ in range(S)]
    Vs = [r.standard_normal((B, Hkv, L, d)) for _ in range(S)]
    Qs = oracle.structured(Q, ks.q, ks.perm_q)
    parts, lses = [], []
    for s in range(S):
        o, l = oracle.partial_attn(Qs, oracle.structured(Ks[s], ks.k, ks.perm_kv[s]),
                                   oracle.structured(Vs[s], ks.v, ks.perm_kv[s]))
        parts.append(o); lses.append(l)
    O, _ = oracle.lse_merge(np.stack(parts), np.stack(lses))
    out = oracle.structured(O, ks.v_inv, ks.perm_q, scatter=True)
    ref, _ = oracle.plain_attention(Q, np.concatenate(Ks, 2), np.concatenate(Vs, 2))
    assert np.abs(out - ref).max() <= 1e-5 * np.abs(ref).max()


def test_planted_mistakes_are_caught(oracle):
    """A wrong factor order, a scatter in place of a gather or a missing normalisation would not survive the pins."""
    d = 8
    ks = W.make_structured_keys(1, d, 3, 3, 1, seed=8, dtype=torch.float32)
    a, g1, g2, b = np_key(ks.q)
    X = np.random.default_rng(4).standard_normal((1, 1, 3, d))
    Y = oracle.structured(X, ks.q)[0, 0]
    H = hadamard(d) / np.sqrt(d)
    P1 = np.zeros((d, d)); P1[g1[0], np.arange(d)] = 1.0
    P2 = np.zeros((d, d)); P2[g2[0], np.arange(d)] = 1.0
    wrong = [np.diag(a[0]) @ P1.T @ H @ P2 @ np.diag(b[0]),          # scatter instead of gather
             P1 @ np.diag(a[0]) @ H @ P2 @ np.diag(b[0]),            # scale after the permutation
             np.diag(a[0]) @ P1 @ hadamard(d) @ P2 @ np.diag(b[0]),  # normalisation left out
             np.diag(a[0]) @ P1 @ H @ np.diag(b[0]) @ P2]            # S2 before P2
    for Phi in wrong:
        assert np.abs(X[0, 0] @ Phi - Y).max() > 1e-3
