"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself and never against the HIP path.  Runs without a GPU.

Citations are to the paper's sections/equations:
  eq. (1)            scaled dot-product attention
  Section 4.1        node-local output O_i, normalisation factor w_i, global aggregation
  Section 4.2        Lemma 1 (inner products), Lemma 2 (linearity), structured Phi, token
                     permutation, Enc / Attention / Dec of the scrambled attention protocol
"""
import math
import os

import numpy as np
import pytest
import torch

from paper_2605_25716_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def rand_case(seed, B=2, Hq=4, Hkv=2, Lq=3, Lk=37, d=8, scale=1.0):
    r = rng(seed)
    Q = r.standard_normal((B, Hq, Lq, d)) * scale
    K = r.standard_normal((B, Hkv, Lk, d)) * scale
    V = r.standard_normal((B, Hkv, Lk, d))
    return Q, K, V


# --------------------------------------------------------------------------- brute force, eq. (1)
def brute_attention(Q, K, V):
    """Pure-Python eq. (1), exponentials expanded term by term (no max subtraction)."""
    B, Hq, Lq, d = Q.shape
    Hkv, Lk = K.shape[1], K.shape[2]
    G = Hq // Hkv
    O = np.zeros((B, Hq, Lq, d))
    lse = np.zeros((B, Hq, Lq))
    for b in range(B):
        for h in range(Hq):
            g = h // G
            for i in range(Lq):
                e = []
                for t in range(Lk):
                    dot = sum(float(Q[b, h, i, c]) * float(K[b, g, t, c]) for c in range(d))
                    e.append(math.exp(dot / math.sqrt(d)))
                tot = sum(e)
                for c in range(d):
                    O[b, h, i, c] = sum(e[t] * float(V[b, g, t, c]) for t in range(Lk)) / tot
                lse[b, h, i] = math.log(tot)
    return O, lse


@pytest.mark.parametrize("d,Lk", [(2, 1), (2, 4), (3, 3), (4, 4)])
def test_plain_attention_brute_force_tiny(oracle, d, Lk):
    Q, K, V = rand_case(11 + d + Lk, B=1, Hq=2, Hkv=1, Lq=2, Lk=Lk, d=d)
    O, lse = oracle.plain_attention(Q, K, V)
    Ob, lb = brute_attention(Q, K, V)
    np.testing.assert_allclose(O, Ob, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, lb, rtol=1e-13, atol=1e-14)


def test_partial_attn_brute_force_tiny(oracle):
    Q, K, V = rand_case(5, B=2, Hq=4, Hkv=2, Lq=2, Lk=4, d=3)
    O, lse = oracle.partial_attn(Q, K, V)
    Ob, lb = brute_attention(Q, K, V)
    np.testing.assert_allclose(O, Ob, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, lb, rtol=1e-13, atol=1e-14)


# --------------------------------------------------------------------------- library special case
@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2)])
def test_plain_attention_vs_torch_sdpa_fp64(oracle, Hq, Hkv):
    Q, K, V = rand_case(21, B=2, Hq=Hq, Hkv=Hkv, Lq=5, Lk=65, d=16)
    O, lse = oracle.plain_attention(Q, K, V)
    G = Hq // Hkv
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    tk, tv = tk.repeat_interleave(G, dim=1), tv.repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)
    ref_lse = torch.logsumexp(tq @ tk.transpose(-1, -2) / math.sqrt(16), dim=-1)
    np.testing.assert_allclose(O, ref.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, ref_lse.numpy(), rtol=1e-12, atol=1e-13)
    # the per-shard function is the same definition applied to one node's keys
    O2, lse2 = oracle.partial_attn(Q, K, V)
    np.testing.assert_allclose(O2, ref.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse2, ref_lse.numpy(), rtol=1e-12, atol=1e-13)


def test_partial_attn_custom_scale(oracle):
    Q, K, V = rand_case(22, B=1, Hq=2, Hkv=2, Lq=3, Lk=20, d=8)
    O, lse = oracle.partial_attn(Q, K, V, scale=0.37)
    tq, tk, tv = (torch.from_numpy(x) for x in (Q, K, V))
    s = tq @ tk.transpose(-1, -2) * 0.37
    np.testing.assert_allclose(O, (torch.softmax(s, -1) @ tv).numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, torch.logsumexp(s, -1).numpy(), rtol=1e-12)


# --------------------------------------------------------------------------- golden closed form
def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = np.array([float(x) for x in v])
    return out


def golden_inputs():
    q = np.array([[[[math.sqrt(2.0), 0.0]]]])
    K1 = np.array([[[[math.log(2.0), 5.0], [0.0, -3.0], [math.log(3.0), 1.0]]]])
    V1 = np.array([[[[3.0, 6.0], [6.0, -12.0], [2.0, 4.0]]]])
    K2 = np.array([[[[math.log(4.0), 0.0]]]])
    V2 = np.array([[[[9.0, -4.0]]]])
    return q, K1, V1, K2, V2


def test_golden_two_shard_closed_form(oracle):
    g = read_golden("two_shard_closed_form.txt")
    q, K1, V1, K2, V2 = golden_inputs()
    # Section 4.1 literal functions
    O1, w1 = oracle.local_attention_raw(q, K1, V1)
    O2, w2 = oracle.local_attention_raw(q, K2, V2)
    np.testing.assert_allclose(w1.ravel(), g["w_1"], rtol=1e-14)
    np.testing.assert_allclose(O1.ravel(), g["O_1"], rtol=1e-14)
    np.testing.assert_allclose(w2.ravel(), g["w_2"], rtol=1e-14)
    np.testing.assert_allclose(O2.ravel(), g["O_2"], rtol=1e-14)
    Ot, wt = oracle.aggregate_raw(np.stack([O1, O2]), np.stack([w1, w2]))
    np.testing.assert_allclose(wt.ravel(), g["w_total"], rtol=1e-14)
    np.testing.assert_allclose(Ot.ravel(), g["O_total"], rtol=1e-14)
    # log-domain functions used for parity
    P1, l1 = oracle.partial_attn(q, K1, V1)
    P2, l2 = oracle.partial_attn(q, K2, V2)
    np.testing.assert_allclose(np.exp(l1).ravel(), g["w_1"], rtol=1e-14)
    np.testing.assert_allclose(P1.ravel(), g["O_1"], rtol=1e-14)
    np.testing.assert_allclose(np.exp(l2).ravel(), g["w_2"], rtol=1e-14)
    np.testing.assert_allclose(P2.ravel(), g["O_2"], rtol=1e-14)
    Om, lm = oracle.lse_merge(np.stack([P1, P2]), np.stack([l1, l2]))
    np.testing.assert_allclose(np.exp(lm).ravel(), g["w_total"], rtol=1e-14)
    np.testing.assert_allclose(Om.ravel(), g["O_total"], rtol=1e-14, atol=1e-15)
    # and eq. (1) over the concatenation
    Of, lf = oracle.plain_attention(q, np.concatenate([K1, K2], 2), np.concatenate([V1, V2], 2))
    np.testing.assert_allclose(Of.ravel(), g["O_total"], rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(np.exp(lf).ravel(), g["w_total"], rtol=1e-14)


# --------------------------------------------------------------------------- Section 4.1 equivalences
def test_log_domain_equals_raw_definition(oracle):
    Q, K, V = rand_case(31, B=2, Hq=4, Hkv=2, Lq=4, Lk=50, d=8)
    Or, w = oracle.local_attention_raw(Q, K, V)
    O, lse = oracle.partial_attn(Q, K, V)
    np.testing.assert_allclose(O, Or, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, np.log(w), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("splits", [[50], [1, 49], [7, 20, 23], [10, 10, 10, 10, 10]])
def test_merge_of_shards_equals_full_attention(oracle, splits):
    Q, K, V = rand_case(41, B=2, Hq=4, Hkv=2, Lq=3, Lk=sum(splits), d=8)
    Of, lf = oracle.plain_attention(Q, K, V)
    parts, lses, raws, ws = [], [], [], []
    a = 0
    for n in splits:
        o, l = oracle.partial_attn(Q, K[:, :, a:a + n], V[:, :, a:a + n])
        orr, w = oracle.local_attention_raw(Q, K[:, :, a:a + n], V[:, :, a:a + n])
        parts.append(o); lses.append(l); raws.append(orr); ws.append(w)
        a += n
    O, lse = oracle.lse_merge(np.stack(parts), np.stack(lses))
    np.testing.assert_allclose(O, Of, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, lf, rtol=1e-12, atol=1e-13)
    # the paper's raw aggregation formula gives the same
    Or, wt = oracle.aggregate_raw(np.stack(raws), np.stack(ws))
    np.testing.assert_allclose(Or, Of, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(np.log(wt), lf, rtol=1e-12, atol=1e-13)


def test_merge_handles_empty_shards_and_is_never_nan(oracle):
    Q, K, V = rand_case(42, B=1, Hq=2, Hkv=1, Lq=2, Lk=9, d=4)
    o1, l1 = oracle.partial_attn(Q, K, V)
    o0, l0 = oracle.partial_attn(Q, K[:, :, :0], V[:, :, :0])
    assert np.all(o0 == 0) and np.all(np.isneginf(l0))
    O, lse = oracle.lse_merge(np.stack([o0, o1, o0]), np.stack([l0, l1, l0]))
    np.testing.assert_allclose(O, o1, rtol=1e-15)
    np.testing.assert_allclose(lse, l1, rtol=1e-15)
    O, lse = oracle.lse_merge(np.stack([o0, o0]), np.stack([l0, l0]))
    assert np.all(O == 0) and np.all(np.isneginf(lse))


def test_large_logits_do_not_overflow(oracle):
    # logits ~ +-2000: the raw sum of exponentials is not representable, the log form is
    Q, K, V = rand_case(43, B=1, Hq=2, Hkv=1, Lq=2, Lk=16, d=4, scale=40.0)
    O, lse = oracle.partial_attn(Q, K, V)
    assert np.all(np.isfinite(O)) and np.all(np.isfinite(lse))
    s = np.einsum("bhid,bgtd->bhit", Q, K) / 2.0
    np.testing.assert_allclose(lse, torch.logsumexp(torch.from_numpy(s), -1).numpy(), rtol=1e-13)
    # shifting every logit of a row by a constant c adds c to lse and leaves O alone:
    # append a constant channel to q and k
    c = 3.25
    Q2 = np.concatenate([Q, np.full(Q.shape[:-1] + (1,), 1.0)], -1)
    K2 = np.concatenate([K, np.full(K.shape[:-1] + (1,), c)], -1)
    V2 = np.concatenate([V, np.zeros(V.shape[:-1] + (1,))], -1)
    O2, lse2 = oracle.partial_attn(Q2, K2, V2, scale=0.5)
    np.testing.assert_allclose(O2[..., :-1], O, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(lse2, lse + c * 0.5, rtol=1e-12)


# --------------------------------------------------------------------------- closed forms
def test_closed_forms(oracle):
    r = rng(51)
    B, H, L, d = 1, 2, 33, 8
    K = r.standard_normal((B, H, L, d)); V = r.standard_normal((B, H, L, d))
    # zero query: uniform attention
    O, lse = oracle.partial_attn(np.zeros((B, H, 2, d)), K, V)
    np.testing.assert_allclose(O, np.broadcast_to(V.mean(2, keepdims=True), O.shape), rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(lse, math.log(L), rtol=1e-14)
    # all keys equal: uniform attention, lse = s0 + ln L
    Q = r.standard_normal((B, H, 2, d))
    Kc = np.broadcast_to(K[:, :, :1], K.shape).copy()
    O, lse = oracle.partial_attn(Q, Kc, V)
    s0 = np.einsum("bhid,bhd->bhi", Q, Kc[:, :, 0]) / math.sqrt(d)
    np.testing.assert_allclose(O, np.broadcast_to(V.mean(2, keepdims=True), O.shape), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(lse, s0 + math.log(L), rtol=1e-13)
    # a single key: O = v0, lse = s0
    O, lse = oracle.partial_attn(Q, K[:, :, :1], V[:, :, :1])
    np.testing.assert_allclose(O, np.broadcast_to(V[:, :, :1], O.shape), rtol=1e-15)
    np.testing.assert_allclose(lse, np.einsum("bhid,bhd->bhi", Q, K[:, :, 0]) / math.sqrt(d), rtol=1e-14)
    # one dominant key (logit +60 over the rest)
    Kd = np.zeros((B, H, L, d)); Kd[:, :, 5, 0] = 60.0 * math.sqrt(d)
    Qd = np.zeros((B, H, 1, d)); Qd[..., 0] = 1.0
    O, lse = oracle.partial_attn(Qd, Kd, V)
    np.testing.assert_allclose(O[:, :, 0], V[:, :, 5], atol=1e-20 + 40 * math.exp(-60) * np.abs(V).max())
    np.testing.assert_allclose(lse, 60.0, atol=1e-12)
    # duplicating a shard: O unchanged, lse + ln 2
    o, l = oracle.partial_attn(Q, K, V)
    O2, l2 = oracle.lse_merge(np.stack([o, o]), np.stack([l, l]))
    np.testing.assert_allclose(O2, o, rtol=1e-14)
    np.testing.assert_allclose(l2, l + math.log(2.0), rtol=1e-14)


# --------------------------------------------------------------------------- Section 4.2 lemmas
def general_phi(r, H, d):
    """A well-conditioned but neither orthogonal nor symmetric invertible matrix per head."""
    return np.stack([W.haar_orthogonal(r, d) @ np.diag(r.uniform(0.5, 2.0, d)) @ W.haar_orthogonal(r, d)
                     for _ in range(H)])


def test_lemma1_inner_product_preservation(oracle):
    r = rng(61)
    H, d, L = 2, 16, 9
    phi = general_phi(r, H, d)
    phi_inv_t = np.transpose(np.linalg.inv(phi), (0, 2, 1))
    x1 = r.standard_normal((1, H, L, d)); x2 = r.standard_normal((1, H, L, d))
    a = oracle.scramble(x1, phi); b = oracle.scramble(x2, phi_inv_t)
    np.testing.assert_allclose(np.einsum("bhid,bhjd->bhij", a, b), np.einsum("bhid,bhjd->bhij", x1, x2),
                               rtol=1e-10, atol=1e-11)
    # planted mistake: using Phi^{-1} instead of Phi^{-T} (a transposed operand) must break the lemma
    b_bad = oracle.scramble(x2, np.linalg.inv(phi))
    assert np.abs(np.einsum("bhid,bhjd->bhij", a, b_bad) - np.einsum("bhid,bhjd->bhij", x1, x2)).max() > 1e-2


def test_lemma2_linearity(oracle):
    r = rng(62)
    H, d, L = 2, 16, 7
    phi = general_phi(r, H, d)
    x = r.standard_normal((1, H, L, d)); w = r.standard_normal(L)
    lhs = np.einsum("l,bhld->bhd", w, oracle.scramble(x, phi))
    rhs = oracle.scramble(np.einsum("l,bhld->bhd", w, x)[:, :, None, :], phi)[:, :, 0]
    np.testing.assert_allclose(lhs, rhs, rtol=1e-11, atol=1e-12)


def test_scramble_matches_matmul_and_gather(oracle):
    r = rng(63)
    B, H, Hkv, L, d = 2, 4, 2, 11, 8
    X = r.standard_normal((B, H, L, d)); phi = general_phi(r, Hkv, d)
    perm = np.stack([r.permutation(L) for _ in range(B)]).astype(np.int32)
    for p, idx in ((None, [np.arange(L)] * B), (perm[0], [perm[0]] * B), (perm, list(perm))):
        Y = oracle.scramble(X, phi, p)
        for b in range(B):
            for h in range(H):
                ref = torch.from_numpy(X[b, h][idx[b]]) @ torch.from_numpy(phi[h // 2])
                np.testing.assert_allclose(Y[b, h], ref.numpy(), rtol=1e-13, atol=1e-14)


def test_identity_phi_is_a_pure_row_move(oracle):
    r = rng(64)
    B, H, L, d = 1, 2, 13, 8
    X = r.standard_normal((B, H, L, d)); perm = r.permutation(L).astype(np.int32)
    eye = np.broadcast_to(np.eye(d), (H, d, d))
    Y = oracle.scramble(X, eye, perm)
    assert np.array_equal(Y, X[:, :, perm])                 # bit-exact gather
    Z = oracle.unscramble(Y, eye, perm)
    assert np.array_equal(Z, X)                             # scatter undoes the gather bit-exactly
    inv = oracle.invert_perm(perm)
    assert np.array_equal(inv[perm], np.arange(L)) and np.array_equal(perm[inv], np.arange(L))
    assert np.array_equal(oracle.scramble(Y, eye, inv), X)


def test_unscramble_matches_matmul_and_scatter(oracle):
    r = rng(65)
    B, H, Hkv, L, d = 2, 4, 2, 6, 8
    X = r.standard_normal((B, H, L, d)); phi = general_phi(r, Hkv, d); perm = r.permutation(L).astype(np.int32)
    Y = oracle.unscramble(X, phi, perm)
    for b in range(B):
        for h in range(H):
            ref = np.zeros((L, d)); ref[perm] = (torch.from_numpy(X[b, h]) @ torch.from_numpy(phi[h // 2])).numpy()
            np.testing.assert_allclose(Y[b, h], ref, rtol=1e-13, atol=1e-14)


# --------------------------------------------------------------------------- protocol invariants
def protocol_inputs(seed, kind, B=2, Hq=4, Hkv=2, Lq=5, shards=(17, 9, 30), d=16, n_perm=1):
    r = rng(seed)
    Q = r.standard_normal((B, Hq, Lq, d))
    K = [r.standard_normal((B, Hkv, n, d)) for n in shards]
    V = [r.standard_normal((B, Hkv, n, d)) for n in shards]
    if kind == "general":
        phi_kq = general_phi(r, Hkv, d); phi_v = general_phi(r, Hkv, d)
    elif kind == "structured":
        phi_kq = np.stack([W.structured_phi(r, d) for _ in range(Hkv)])
        phi_v = np.stack([W.structured_phi(r, d) for _ in range(Hkv)])
    else:
        phi_kq = np.stack([W.haar_orthogonal(r, d) for _ in range(Hkv)])
        phi_v = np.stack([W.haar_orthogonal(r, d) for _ in range(Hkv)])
    phi_k = np.transpose(np.linalg.inv(phi_kq), (0, 2, 1))
    phi_v_inv = np.linalg.inv(phi_v)
    perm_q = r.permutation(Lq).astype(np.int32)
    perm_kv = [np.stack([r.permutation(n) for _ in range(n_perm)]).astype(np.int32) for n in shards]
    return Q, K, V, phi_kq, phi_k, phi_v, phi_v_inv, perm_q, perm_kv


@pytest.mark.parametrize("kind", ["orthogonal", "general", "structured"])
@pytest.mark.parametrize("n_perm", [1, 2])
def test_protocol_equals_plain_attention(oracle, kind, n_perm):
    Q, K, V, pq, pk, pv, pvi, perm_q, perm_kv = protocol_inputs(71, kind, n_perm=n_perm)
    out, lse = oracle.protocol(Q, K, V, pq, pk, pv, pvi, perm_q, perm_kv)
    Of, lf = oracle.plain_attention(Q, np.concatenate(K, 2), np.concatenate(V, 2))
    tol = 1e-10 if kind != "structured" else 1e-8   # S1,S2 in [1/8,8] condition the matrices up to 64^2
    np.testing.assert_allclose(out, Of, rtol=tol, atol=tol)
    np.testing.assert_allclose(lse, lf, rtol=tol, atol=tol)
    # both orders of Dec and aggregation agree (linearity lemma)
    out2, lse2 = oracle.protocol(Q, K, V, pq, pk, pv, pvi, perm_q, perm_kv, descramble_first=True)
    np.testing.assert_allclose(out2, out, rtol=tol, atol=tol)
    np.testing.assert_allclose(lse2, lse, rtol=1e-12)


def test_scrambled_attention_is_PQ_attention_PhiV(oracle):
    """Step 2 of the protocol: Attention(Q',K',V') = P_Q Attention(Q,K,V) Phi_V."""
    Q, K, V, pq, pk, pv, pvi, perm_q, perm_kv = protocol_inputs(72, "general", shards=(23,))
    Qs = oracle.scramble(Q, pq, perm_q)
    Ks = oracle.scramble(K[0], pk, perm_kv[0]); Vs = oracle.scramble(V[0], pv, perm_kv[0])
    Os, _ = oracle.plain_attention(Qs, Ks, Vs)
    Of, _ = oracle.plain_attention(Q, K[0], V[0])
    G = Q.shape[1] // K[0].shape[1]
    expect = np.einsum("bhid,hde->bhie", Of[:, :, perm_q], np.repeat(pv, G, axis=0))
    np.testing.assert_allclose(Os, expect, rtol=1e-10, atol=1e-11)


def test_output_invariant_under_token_permutations(oracle):
    Q, K, V, pq, pk, pv, pvi, perm_q, perm_kv = protocol_inputs(73, "orthogonal")
    base, lbase = oracle.protocol(Q, K, V, pq, pk, pv, pvi, None, None)
    r = rng(74)
    for _ in range(3):
        pkv = [r.permutation(k.shape[2]).astype(np.int32)[None] for k in K]
        pq_ = r.permutation(Q.shape[2]).astype(np.int32)
        out, lse = oracle.protocol(Q, K, V, pq, pk, pv, pvi, pq_, pkv)
        np.testing.assert_allclose(out, base, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse, lbase, rtol=1e-11, atol=1e-12)
    # planted mistake: permuting K and V inconsistently must change the result
    Ks = oracle.scramble(K[0], pk, perm_kv[0]); Vs_bad = oracle.scramble(V[0], pv, None)
    Qs = oracle.scramble(Q, pq, None)
    bad, _ = oracle.partial_attn(Qs, Ks, Vs_bad)
    good, _ = oracle.partial_attn(Qs, Ks, oracle.scramble(V[0], pv, perm_kv[0]))
    assert np.abs(bad - good).max() > 1e-3


def test_identity_keys_reduce_protocol_to_plain_path_bitwise(oracle):
    Q, K, V, *_ = protocol_inputs(75, "orthogonal", shards=(19,))
    Hkv, d = K[0].shape[1], K[0].shape[3]
    eye = np.broadcast_to(np.eye(d), (Hkv, d, d)).copy()
    out, lse = oracle.protocol(Q, K, V, eye, eye, eye, eye, None, None)
    O, l = oracle.partial_attn(Q, K[0], V[0])
    assert np.array_equal(out, O) and np.array_equal(lse, l)


# --------------------------------------------------------------------------- key generation
def test_generated_keys(oracle):
    keys = W.make_keys(4, 64, 16, 100, 3, seed=7, dtype=torch.float32, n_perm=1)
    for m in (keys.phi_kq_exact, keys.phi_v_exact):
        for h in range(4):
            np.testing.assert_allclose(m[h] @ m[h].T, np.eye(64), atol=1e-12)
    assert sorted(keys.perm_q.tolist()) == list(range(16))
    for p in keys.perm_kv:
        assert p.shape == (1, 100) and p.dtype == torch.int32 and sorted(p[0].tolist()) == list(range(100))
    # duality as stored: phi_q @ phi_k^T ~ I to storage precision, phi_v @ phi_v_inv ~ I
    pq, pk = keys.phi_q.double().numpy(), keys.phi_k.double().numpy()
    np.testing.assert_allclose(pq @ np.transpose(pk, (0, 2, 1)), np.broadcast_to(np.eye(64), (4, 64, 64)), atol=1e-5)
    kb = W.make_keys(2, 128, 1, 64, 1, seed=8, dtype=torch.bfloat16)
    assert kb.perm_q is None and kb.phi_q.dtype == torch.bfloat16 and kb.phi_v_inv.dtype == torch.float32
    pv, pvi = kb.phi_v.double().numpy(), kb.phi_v_inv.double().numpy()
    np.testing.assert_allclose(pv @ pvi, np.broadcast_to(np.eye(128), (2, 128, 128)), atol=1e-5)


def test_structured_phi_construction():
    r = rng(81)
    d = 64
    h = W.sylvester_hadamard(d)
    assert set(np.unique(h)) == {-1.0, 1.0}
    np.testing.assert_array_equal(h @ h.T, d * np.eye(d))
    phi = W.structured_phi(r, d)
    # every entry has magnitude |s1_i| |s2_j| / sqrt(d): rank-one magnitude pattern, in [1/64, 64]/sqrt(d)
    mag = np.abs(phi) * math.sqrt(d)
    assert mag.min() >= 1 / 64 - 1e-12 and mag.max() <= 64 + 1e-12
    np.testing.assert_allclose(mag, np.outer(mag[:, 0], mag[0, :]) / mag[0, 0], rtol=1e-12)
    assert np.linalg.cond(phi) <= 64 * 64 * (1 + 1e-9)


def test_activation_generator_outliers():
    x = W.activations(2, 4, 64, 32, seed=5, tensor_id=9, outliers=True)
    idx = W.outlier_channels(4, 32, 5, 9)
    assert len(idx) == 1
    std = x.double().permute(1, 3, 0, 2).reshape(4 * 32, -1).std(dim=1).numpy()
    assert 12 < std[idx[0]] < 28
    others = np.delete(std, idx)
    assert 0.7 < others.min() and others.max() < 1.3
    y = W.activations(2, 4, 64, 32, seed=5, tensor_id=9, outliers=True)
    assert torch.equal(x, y)
