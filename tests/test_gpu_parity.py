"""GPU parity: every C-ABI call against the CPU oracle, element by element, on identical seeded inputs.

Stage-wise rule: each call is checked on inputs that come from the input generator or from the ORACLE's
previous stage (rounded to the storage type), never from the HIP path, so both sides consume identical bits.
Sizes span several tiles and ragged tails of every kernel (16-row scramble tiles, 32/128-key decode steps,
64-key / 128-query prefill tiles, 64-key fp32 steps).
"""
import math

import numpy as np
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def to_dev(t):
    return None if t is None else t.to(DEV)


def small_case(name, B, Hq, Hkv, d, Lq, S, L, dtype, outliers=True, index=7, n_perm=1, kind="orthogonal"):
    cfg = W.Config(name, B, Hq, Hkv, d, Lq, S, L, dtype, outliers, index)
    return W.make_case(cfg, kind=kind, n_perm=n_perm)


def rounded(a64, dtype):
    return torch.from_numpy(np.ascontiguousarray(a64)).to(dtype)


# ------------------------------------------------------------------------------------------------ scramble
SCR_CASES = [
    # name, B, Hq, Hkv, d, Lq, L, dtype, n_perm
    ("bf16_d128", 2, 8, 2, 128, 5, 203, "bf16", 1),
    ("bf16_d128_perm_per_seq", 2, 4, 2, 128, 70, 1000, "bf16", 2),
    ("bf16_d64", 1, 4, 4, 64, 33, 129, "bf16", 1),
    ("f16_d128", 1, 4, 2, 128, 17, 95, "f16", 1),
    ("f32_d64", 1, 2, 2, 64, 4, 512, "f32", 1),
    ("f32_d128", 2, 4, 2, 128, 9, 77, "f32", 2),
]


@pytest.mark.parametrize("case", SCR_CASES, ids=[c[0] for c in SCR_CASES])
def test_scramble_kv_and_q(oracle, case):
    name, B, Hq, Hkv, d, Lq, L, dt, n_perm = case
    c = small_case(name, B, Hq, Hkv, d, Lq, 1, L, dt, n_perm=n_perm)
    dtype = W.torch_dtype(dt)
    k = c.keys
    Kd, Vd = fb.fedrag_scramble_kv(to_dev(c.K[0]), to_dev(c.V[0]), to_dev(k.phi_k), to_dev(k.phi_v),
                                   to_dev(k.perm_kv[0]))
    Qd = fb.fedrag_scramble_q(to_dev(c.Q), to_dev(k.phi_q), to_dev(k.perm_q))
    torch.cuda.synchronize()
    PT.check_scramble(Kd, oracle.scramble(c.K[0], k.phi_k, k.perm_kv[0]), c.K[0], k.phi_k, k.perm_kv[0], 1, dtype, "K'")
    PT.check_scramble(Vd, oracle.scramble(c.V[0], k.phi_v, k.perm_kv[0]), c.V[0], k.phi_v, k.perm_kv[0], 1, dtype, "V'")
    PT.check_scramble(Qd, oracle.scramble(c.Q, k.phi_q, k.perm_q), c.Q, k.phi_q, k.perm_q, Hq // Hkv, dtype, "Q'")


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_identity_phi_is_bit_exact_row_move(oracle, dt):
    """With Phi = I the scramble is a pure gather and Dec a pure scatter: results are bit-identical."""
    c = small_case("ident", 2, 4, 2, 128, 50, 1, 301, dt, kind="identity", n_perm=2)
    k = c.keys
    Kd, Vd = fb.fedrag_scramble_kv(to_dev(c.K[0]), to_dev(c.V[0]), to_dev(k.phi_k), to_dev(k.phi_v),
                                   to_dev(k.perm_kv[0]))
    Qd = fb.fedrag_scramble_q(to_dev(c.Q), to_dev(k.phi_q), to_dev(k.perm_q))
    p = k.perm_kv[0].long()
    for b in range(2):
        assert torch.equal(Kd[b].cpu(), c.K[0][b][:, p[b]])
        assert torch.equal(Vd[b].cpu(), c.V[0][b][:, p[b]])
    assert torch.equal(Qd.cpu(), c.Q[:, :, k.perm_q.long()])
    # no permutation at all: plain copy
    Kd2, _ = fb.fedrag_scramble_kv(to_dev(c.K[0]), to_dev(c.V[0]), to_dev(k.phi_k), to_dev(k.phi_v), None)
    assert torch.equal(Kd2.cpu(), c.K[0])
    # Dec with identity matrix: scatter positions
    X = torch.randn(2, 4, 50, 128, generator=torch.Generator().manual_seed(3))
    out = fb.fedrag_unscramble(to_dev(X), to_dev(k.phi_v_inv), to_dev(k.perm_q))
    ref = torch.empty_like(X); ref[:, :, k.perm_q.long()] = X
    assert torch.equal(out.cpu(), ref)


def test_invert_perm_bit_exact(oracle):
    for L in (1, 2, 255, 256, 257, 10000):
        p = torch.from_numpy(np.random.default_rng(L).permutation(L).astype(np.int32))
        inv = fb.fedrag_invert_perm(to_dev(p)).cpu()
        assert np.array_equal(inv.numpy(), oracle.invert_perm(p))
        assert torch.equal(inv[p.long()], torch.arange(L, dtype=torch.int32))


# ------------------------------------------------------------------------------------------------ partial attention
ATTN_CASES = [
    # name, B, Hq, Hkv, d, Lq, L, dtype          kernel exercised
    ("tiny_f32", 1, 2, 2, 64, 4, 512, "f32"),         # the tiny fp32 configuration itself
    ("f32_d128_ragged", 2, 4, 2, 128, 3, 197, "f32"),
    ("dec_bf16_g4", 2, 8, 2, 128, 1, 1000, "bf16"),    # decode, one partial 128-key step, splits = 1
    ("dec_bf16_g4_split", 2, 8, 2, 128, 1, 5001, "bf16"),  # decode, several KV splits + ragged tail
    ("dec_bf16_L1", 1, 4, 1, 128, 1, 1, "bf16"),
    ("dec_bf16_L37", 1, 4, 1, 128, 1, 37, "bf16"),
    ("dec_bf16_g8", 1, 16, 2, 128, 1, 700, "bf16"),
    ("dec_bf16_rows16", 1, 8, 2, 128, 4, 300, "bf16"),  # G * Lq = 16 rows per KV head
    ("dec_bf16_d64", 2, 4, 2, 64, 2, 450, "bf16"),
    ("dec_f16", 1, 8, 2, 128, 1, 333, "f16"),
    ("pre_bf16", 1, 4, 2, 128, 200, 333, "bf16"),      # prefill: 2 query tiles (one ragged), 6 key tiles
    ("pre_bf16_small", 2, 2, 1, 128, 17, 64, "bf16"),
    ("pre_bf16_d64", 1, 2, 2, 64, 130, 130, "bf16"),
    ("pre_f16", 1, 2, 1, 128, 40, 100, "f16"),
    # few query tiles, many keys: the keys are cut into runs over more workgroups and the partials merged
    ("pre_bf16_kv_runs", 1, 4, 2, 128, 70, 1500, "bf16"),       # 24 tiles -> 6 runs of 4, last tile ragged
    ("pre_bf16_d64_kv_runs", 2, 2, 2, 64, 300, 1111, "bf16"),   # 18 tiles -> runs of 4,4,4,4,2; 2 query tiles
    ("pre_f16_kv_runs", 1, 2, 1, 128, 40, 777, "f16"),
]


def scrambled_inputs(oracle, c):
    """Q', K', V' produced by the ORACLE from generator inputs, rounded to the storage type."""
    dtype = W.torch_dtype(c.cfg.dtype)
    k = c.keys
    Qs = rounded(oracle.scramble(c.Q, k.phi_q, k.perm_q), dtype)
    Ks = [rounded(oracle.scramble(K, k.phi_k, p), dtype) for K, p in zip(c.K, k.perm_kv)]
    Vs = [rounded(oracle.scramble(V, k.phi_v, p), dtype) for V, p in zip(c.V, k.perm_kv)]
    return Qs, Ks, Vs


@pytest.mark.parametrize("case", ATTN_CASES, ids=[c[0] for c in ATTN_CASES])
def test_partial_attn(oracle, case):
    name, B, Hq, Hkv, d, Lq, L, dt = case
    c = small_case(name, B, Hq, Hkv, d, Lq, 1, L, dt, outliers=(dt != "f32"))
    dtype = W.torch_dtype(dt)
    Qs, Ks, Vs = scrambled_inputs(oracle, c)
    O, lse = fb.fedrag_partial_attn(to_dev(Qs), to_dev(Ks[0]), to_dev(Vs[0]))
    torch.cuda.synchronize()
    Or, lr = oracle.partial_attn(Qs, Ks[0], Vs[0])
    eo, el = PT.check_attn(O, lse, Or, lr, dtype, name)
    print(f"{name}: O err {eo:.3e} lse err {el:.3e}")


def test_partial_attn_plain_inputs_with_concentrated_outliers(oracle):
    """Unscrambled activations (outlier channels not spread by Phi) make logits of order 10^2."""
    c = small_case("plain_outliers", 2, 8, 2, 128, 1, 1, 2000, "bf16")
    O, lse = fb.fedrag_partial_attn(to_dev(c.Q), to_dev(c.K[0]), to_dev(c.V[0]))
    Or, lr = oracle.partial_attn(c.Q, c.K[0], c.V[0])
    assert np.abs(lr).max() > 20
    # V is not scrambled here either (outlier channels reach |v| ~ 80); the decode kernel feeds the second product
    # two storage-type terms per probability, so the flat bound holds
    PT.check_attn(O, lse, Or, lr, torch.bfloat16, "plain inputs with concentrated outliers", report=True)


def test_partial_attn_empty_shard_and_custom_scale(oracle):
    c = small_case("empty", 1, 4, 2, 128, 1, 1, 64, "bf16")
    Qs, Ks, Vs = scrambled_inputs(oracle, c)
    O, lse = fb.fedrag_partial_attn(to_dev(Qs), to_dev(Ks[0][:, :, :0]), to_dev(Vs[0][:, :, :0]))
    assert torch.all(O == 0) and torch.all(torch.isneginf(lse))
    O, lse = fb.fedrag_partial_attn(to_dev(Qs), to_dev(Ks[0]), to_dev(Vs[0]), softmax_scale=0.03)
    Or, lr = oracle.partial_attn(Qs, Ks[0], Vs[0], scale=0.03)
    PT.check_attn(O, lse, Or, lr, torch.bfloat16, "custom scale")


# ------------------------------------------------------------------------------------------------ merge / unscramble
@pytest.mark.parametrize("d,S,rows_shape", [(128, 4, (2, 8, 3)), (64, 8, (1, 4, 130)), (128, 1, (1, 2, 5))])
def test_lse_merge(oracle, d, S, rows_shape):
    g = torch.Generator().manual_seed(11)
    B, H, Lq = rows_shape
    O = torch.randn((S, B, H, Lq, d), generator=g) * 3
    l = torch.randn((S, B, H, Lq), generator=g) * 30
    if S > 2:
        l[1] = float("-inf")              # an empty shard
        l[:, 0, 0, 0] = float("-inf")     # a row empty everywhere
        O[1] = 123.0                      # must be ignored
    Om, lm = fb.fedrag_lse_merge(to_dev(O), to_dev(l))
    Or, lr = oracle.lse_merge(O, l)
    assert PT.rel_normwise(Om, Or) <= PT.TOL_F32_REL
    assert PT.rel_normwise(lm, lr) <= PT.TOL_F32_REL
    assert not torch.isnan(Om).any() and not torch.isnan(lm).any()


@pytest.mark.parametrize("d,Hq,Hkv,Lq", [(128, 8, 2, 1), (128, 4, 2, 77), (64, 4, 4, 40), (128, 4, 2, 300),
                                           (64, 4, 4, 130)])
def test_unscramble(oracle, d, Hq, Hkv, Lq):
    keys = W.make_keys(Hkv, d, Lq, 8, 1, seed=5 + Lq, dtype=torch.bfloat16)
    g = torch.Generator().manual_seed(12)
    X = torch.randn((2, Hq, Lq, d), generator=g) * 2
    out = fb.fedrag_unscramble(to_dev(X), to_dev(keys.phi_v_inv), to_dev(keys.perm_q))
    ref = oracle.unscramble(X, keys.phi_v_inv, keys.perm_q)
    assert PT.rel_normwise(out, ref) <= PT.TOL_F32_REL
    # element-wise against the fp32 accumulation bound
    mag = np.einsum("bhlk,hkj->bhlj", np.abs(PT.f64(X)), np.repeat(np.abs(PT.f64(keys.phi_v_inv)), Hq // Hkv, axis=0))
    if keys.perm_q is not None:
        m2 = np.empty_like(mag); m2[:, :, keys.perm_q.long().numpy()] = mag; mag = m2
    assert np.all(np.abs(PT.f64(out) - ref) <= 2e-5 * mag + 1e-30)


# ------------------------------------------------------------------------------------------------ whole chain
CHAIN_CASES = [
    ("chain_tiny_f32", 1, 2, 2, 64, 4, 1, 512, "f32", False),
    ("chain_decode_bf16", 2, 8, 2, 128, 1, 3, 700, "bf16", True),
    ("chain_prefill_bf16", 1, 4, 2, 128, 150, 2, 260, "bf16", True),
]


@pytest.mark.parametrize("case", CHAIN_CASES, ids=[c[0] for c in CHAIN_CASES])
def test_whole_chain_stagewise_and_end_to_end(oracle, case):
    """All five calls in protocol order.  Stage-wise: each GPU call consumes the oracle's previous stage and is
    held to the tolerance.  End to end: the GPU chain's own result against plain attention, eq. (1)."""
    name, B, Hq, Hkv, d, Lq, S, L, dt, outliers = case
    c = small_case(name, B, Hq, Hkv, d, Lq, S, L, dt, outliers=outliers)
    dtype = W.torch_dtype(dt)
    k = c.keys
    # --- stage-wise
    Qs, Ks, Vs = scrambled_inputs(oracle, c)
    parts, lses, gparts, glses = [], [], [], []
    for s in range(S):
        o, l = oracle.partial_attn(Qs, Ks[s], Vs[s])
        go, gl = fb.fedrag_partial_attn(to_dev(Qs), to_dev(Ks[s]), to_dev(Vs[s]))
        PT.check_attn(go, gl, o, l, dtype, f"{name} shard {s}")
        parts.append(o); lses.append(l)
    P32 = torch.from_numpy(np.stack(parts)).float(); L32 = torch.from_numpy(np.stack(lses)).float()
    Om, lm = oracle.lse_merge(P32, L32)
    gOm, glm = fb.fedrag_lse_merge(to_dev(P32), to_dev(L32))
    assert PT.rel_normwise(gOm, Om) <= PT.TOL_F32_REL and PT.rel_normwise(glm, lm) <= PT.TOL_F32_REL
    Om32 = torch.from_numpy(Om).float()
    fin = oracle.unscramble(Om32, k.phi_v_inv, k.perm_q)
    gfin = fb.fedrag_unscramble(to_dev(Om32), to_dev(k.phi_v_inv), to_dev(k.perm_q))
    assert PT.rel_normwise(gfin, fin) <= PT.TOL_F32_REL
    # --- end to end on the GPU alone
    gQs = fb.fedrag_scramble_q(to_dev(c.Q), to_dev(k.phi_q), to_dev(k.perm_q))
    go_all, gl_all = [], []
    for s in range(S):
        gK, gV = fb.fedrag_scramble_kv(to_dev(c.K[s]), to_dev(c.V[s]), to_dev(k.phi_k), to_dev(k.phi_v),
                                       to_dev(k.perm_kv[s]))
        go, gl = fb.fedrag_partial_attn(gQs, gK, gV)
        go_all.append(go); gl_all.append(gl)
    gO, gL = fb.fedrag_lse_merge(torch.stack(go_all), torch.stack(gl_all))
    gout = fb.fedrag_unscramble(gO, to_dev(k.phi_v_inv), to_dev(k.perm_q))
    plain, plain_lse = oracle.plain_attention(c.Q, torch.cat(c.K, 2), torch.cat(c.V, 2))
    rel = PT.rel_normwise(gout, plain)
    print(f"{name}: end-to-end rel err vs plain attention {rel:.3e}")
    if dtype == torch.float32:
        assert rel <= 1e-4      # fp32 keys: two rounded matrices in the loop, still ~1e-6
    else:
        assert rel <= 0.15      # reported, not held to 2e-2: storage rounding of Q', K', V' moves the logits
    # lse rows come back in P_Q order
    gl_plain = torch.empty_like(gL)
    if k.perm_q is not None:
        gl_plain[:, :, k.perm_q.long().to(DEV)] = gL
    else:
        gl_plain = gL
    if dtype == torch.float32:
        assert PT.rel_normwise(gl_plain, plain_lse) <= 1e-4


# Score patterns along the keys that make the running maximum move late, inside the pipelined (steady-state) key
# tiles of the prefill kernel, where the accumulators are only rescaled when some row's maximum moved: rising and
# falling scores, isolated spikes in either half of a 64-key tile, plateaus, a random walk.  beta[j] is added to every
# query's score of key j (in natural-log units).
def _pattern(name, L, rng):
    j = np.arange(L, dtype=np.float64)
    if name == "rising":          # every tile's maximum far above the one before: a rescale in every tile
        return 0.9 * j
    if name == "falling":         # the first tile holds the maximum: never a rescale
        return -0.5 * j
    if name == "spikes_first_half":   # a few keys 45 above the rest, in the first 32 keys of their 64-key tile
        b = np.zeros(L)
        b[[64 * 5 + 3, 64 * 11 + 31, 64 * 17 + 16]] = [45.0, 80.0, 120.0]
        return b
    if name == "spikes_second_half":
        b = np.zeros(L)
        b[[64 * 4 + 32, 64 * 9 + 63, 64 * 20 + 40]] = [45.0, 80.0, 120.0]
        return b
    if name == "steps":           # plateaus that rise by 9 now and then
        return 9.0 * np.floor(j / 150.0)
    if name == "random_walk":
        return np.cumsum(rng.normal(0.0, 1.5, size=L))
    raise ValueError(name)


@pytest.mark.parametrize("causal", [False, True], ids=["remote", "local_causal"])
@pytest.mark.parametrize("pattern", ["rising", "falling", "spikes_first_half", "spikes_second_half", "steps",
                                     "random_walk"])
@pytest.mark.parametrize("dt,d", [("bf16", 128), ("f16", 64)])
def test_prefill_running_maximum_that_moves_late(oracle, dt, d, pattern, causal):
    dtype = W.torch_dtype(dt)
    B, Hq, Hkv, Lq, L = 1, 2, 1, 300, 1600
    rng = np.random.default_rng(len(pattern) + d)
    g = torch.Generator().manual_seed(7 + d)
    Q = torch.randn((B, Hq, Lq, d), generator=g) * 0.5
    K = torch.randn((B, Hkv, L, d), generator=g) * 0.5
    V = torch.randn((B, Hkv, L, d), generator=g) * 2.0
    # channel 0 carries the pattern: q[0] = 4, k_j[0] = beta_j * sqrt(d) / 4, so that q[0] k_j[0] / sqrt(d) = beta_j
    beta = _pattern(pattern, L, rng)
    if dt == "f16":
        beta = np.clip(beta, -600.0, 600.0)   # keep k[0] inside the fp16 range
    Q[..., 0] = 4.0
    K[..., 0] = torch.from_numpy(beta * np.sqrt(d) / 4.0).float()
    Q, K, V = Q.to(dtype), K.to(dtype), V.to(dtype)
    if causal:
        O, lse = fb.fedrag_local_attn(Q.to(DEV), K.to(DEV), V.to(DEV))
        Or, lr = oracle.local_causal_attn(Q, K, V)
    else:
        O, lse = fb.fedrag_partial_attn(Q.to(DEV), K.to(DEV), V.to(DEV))
        Or, lr = oracle.partial_attn(Q, K, V)
    torch.cuda.synchronize()
    assert torch.isfinite(O).all() and torch.isfinite(lse).all()
    PT.check_attn(O, lse, Or, lr, dtype, f"{pattern}/{dt}/{'causal' if causal else 'plain'}", report=True)
