"""GPU parity of the transport codec (Section 7.5) - bit-exact codes, parameters and dequantised values - and its
effect on the attention result: the variant of the structured scramble without S2 under 8-bit transport."""
import numpy as np
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def data(seed, shape, dtype):
    r = np.random.default_rng(seed)
    x = r.standard_normal(shape) * np.exp(r.uniform(-4, 4, size=shape[:-1] + (1,))) + r.uniform(-3, 3, size=shape[:-1] + (1,))
    x[..., 0, :] = 0.75                    # a constant row
    return torch.from_numpy(x).to(dtype)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dt,d,shape", [("bf16", 128, (2, 3, 1001)), ("bf16", 64, (1, 2, 77)), ("f16", 128, (5, 333)),
                                        ("f32", 64, (3, 130)), ("f32", 128, (1,))])
def test_codec_bit_exact(oracle, bits, dt, d, shape):
    dtype = W.torch_dtype(dt)
    X = data(bits + d + len(shape), shape + (d,), dtype)
    codes, params = fb.fedrag_quantize_rows(X.to(DEV), bits)
    Xh = fb.fedrag_dequantize_rows(codes, params, bits, dtype)
    torch.cuda.synchronize()
    c_ref, p_ref = oracle.quantize_rows(X, bits)
    assert np.array_equal(codes.cpu().numpy(), c_ref), "codes differ"
    assert np.array_equal(params.cpu().numpy().view(np.uint32), p_ref.view(np.uint32)), "scale / lo differ"
    x_ref = torch.from_numpy(oracle.dequantize_rows(c_ref, p_ref, bits)).to(dtype)      # one RNE narrowing
    assert torch.equal(Xh.cpu(), x_ref), "dequantised values differ"


def test_codec_at_shard_size_sampled(oracle):
    cfg = W.CONFIGS["llama8b_decode"]
    dt = W.torch_dtype(cfg.dtype)
    K = W.activations(cfg.batch, cfg.n_kv_heads, cfg.L_kv, cfg.d_head, seed=cfg.seed, tensor_id=W.TID_K, outliers=True,
                      dtype=dt, device=DEV)
    for bits in (8, 4):
        codes, params = fb.fedrag_quantize_rows(K, bits)
        Kh = fb.fedrag_dequantize_rows(codes, params, bits, dt)
        torch.cuda.synchronize()
        rng = np.random.default_rng(bits)
        for _ in range(3):
            b, g = int(rng.integers(cfg.batch)), int(rng.integers(cfg.n_kv_heads))
            c_ref, p_ref = oracle.quantize_rows(K[b, g].cpu(), bits)
            assert np.array_equal(codes[b, g].cpu().numpy(), c_ref)
            assert np.array_equal(params[b, g].cpu().numpy().view(np.uint32), p_ref.view(np.uint32))
            assert torch.equal(Kh[b, g].cpu(), torch.from_numpy(oracle.dequantize_rows(c_ref, p_ref, bits)).to(dt))
        # property over the whole tensor: within half a step, plus the storage rounding (2^-9 relative, bf16) of the
        # reconstruction, whose magnitude is at most |x| + step / 2
        step = params[..., :1]
        err = (Kh.float() - K.float()).abs()
        assert bool((err <= 0.5 * step * (1 + 2.0 ** -7) + 2.0 ** -8 * K.float().abs() + 1e-30).all())


def test_eight_bit_transport_with_and_without_s2(oracle):
    """Section 7.5: with both scalings the scrambled states have a wide per-token range and 8-bit transport hurts;
    leaving S2 out repairs it.  Synthetic N(0,1) activations, structured keys, K' and V' sent through the codec."""
    B, Hq, Hkv, d, Lq, L = 1, 8, 2, 128, 64, 1024
    dt = torch.bfloat16
    seed = 606
    Q = W.activations(B, Hq, Lq, d, seed=seed, tensor_id=W.TID_Q, outliers=False, dtype=dt)
    K = W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_K, outliers=False, dtype=dt)
    V = W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_V, outliers=False, dtype=dt)
    ref, _ = oracle.plain_attention(Q, K, V)
    errs = {}
    for use_s2 in (True, False):
        ks = W.make_structured_keys(Hkv, d, Lq, L, 1, seed=seed, dtype=dt, use_s2=use_s2)
        dk = lambda key: tuple(t.to(DEV) for t in key)
        pq = ks.perm_q.to(DEV)
        Qs = fb.fedrag_scramble_q_structured(Q.to(DEV), dk(ks.q), pq)
        Ks, Vs = fb.fedrag_scramble_kv_structured(K.to(DEV), V.to(DEV), dk(ks.k), dk(ks.v), ks.perm_kv[0].to(DEV))
        for bits in (16, 8):
            if bits == 16:
                Kt, Vt = Ks, Vs
            else:
                Kt = fb.fedrag_dequantize_rows(*fb.fedrag_quantize_rows(Ks, 8), 8, dt)
                Vt = fb.fedrag_dequantize_rows(*fb.fedrag_quantize_rows(Vs, 8), 8, dt)
            O, _ = fb.fedrag_partial_attn(Qs, Kt, Vt)
            out = fb.fedrag_unscramble_structured(O, dk(ks.v_inv), pq)
            errs[(use_s2, bits)] = float(np.linalg.norm(PT.f64(out) - ref) / np.linalg.norm(ref))
    print("relative attention-output error (Frobenius): " +
          ", ".join(f"S2={'on' if k[0] else 'off'} {k[1]}-bit {100 * v:.2f} %" for k, v in errs.items()))
    assert errs[(False, 8)] < errs[(True, 8)]
    assert errs[(False, 8)] < 0.10 and errs[(True, 8)] > 0.25


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("dt,d,structured", [("bf16", 128, False), ("bf16", 128, True), ("f16", 64, False),
                                              ("bf16", 64, True)])
def test_scramble_with_codec_epilogue(oracle, bits, dt, d, structured):
    """The fused call equals the two calls one after the other bit for bit, and both agree with the oracle's
    composition up to the scramble's own one-ulp differences."""
    dtype = W.torch_dtype(dt)
    B, Hkv, L = 2, 2, 333
    seed = 70 + bits + d
    K = W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_K, outliers=True, dtype=dtype)
    V = W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_V, outliers=True, dtype=dtype)
    if structured:
        ks = W.make_structured_keys(Hkv, d, 1, L, 1, seed=seed, dtype=dtype, n_perm=B, batch=B)
        kk, kv = tuple(t.to(DEV) for t in ks.k), tuple(t.to(DEV) for t in ks.v)
        perm = ks.perm_kv[0]
        Ks, Vs = fb.fedrag_scramble_kv_structured(K.to(DEV), V.to(DEV), kk, kv, perm.to(DEV))
        Kref = oracle.structured(K, ks.k, perm)
    else:
        keys = W.make_keys(Hkv, d, 1, L, 1, seed=seed, dtype=dtype, n_perm=B, batch=B)
        kk, kv = keys.phi_k.to(DEV), keys.phi_v.to(DEV)
        perm = keys.perm_kv[0]
        Ks, Vs = fb.fedrag_scramble_kv(K.to(DEV), V.to(DEV), kk, kv, perm.to(DEV))
        Kref = oracle.scramble(K, keys.phi_k, perm)
    Kc, Kp, Vc, Vp = fb.fedrag_scramble_kv_quantized(K.to(DEV), V.to(DEV), kk, kv, perm.to(DEV), bits,
                                                     structured=structured)
    Kc2, Kp2 = fb.fedrag_quantize_rows(Ks, bits)
    Vc2, Vp2 = fb.fedrag_quantize_rows(Vs, bits)
    torch.cuda.synchronize()
    assert torch.equal(Kc, Kc2) and torch.equal(Vc, Vc2)
    assert torch.equal(Kp.view(torch.int32), Kp2.view(torch.int32)) and torch.equal(Vp.view(torch.int32), Vp2.view(torch.int32))
    # against the oracle's composition: rows whose stored K' equals round(oracle) bit for bit must give equal codes
    Kr = torch.from_numpy(Kref).to(dtype)
    same_rows = (Ks.cpu() == Kr).all(dim=-1)
    assert same_rows.float().mean() > 0.2
    c_ref, p_ref = oracle.quantize_rows(Kr, bits)
    assert np.array_equal(Kc.cpu().numpy()[same_rows.numpy()], c_ref[same_rows.numpy()])
    assert np.array_equal(Kp.cpu().numpy()[same_rows.numpy()], p_ref[same_rows.numpy()])
    # every row: dequantised values within one step (+ an ulp of K') of the oracle's composition
    Kh = fb.fedrag_dequantize_rows(Kc, Kp, bits, dtype).cpu().double().numpy()
    ref_h = oracle.dequantize_rows(c_ref, p_ref, bits).astype(np.float64)
    step = p_ref[..., :1].astype(np.float64)
    assert (np.abs(Kh - ref_h) <= 1.01 * step + 3 * PT.storage_ulp(ref_h, dtype)).all()


ATTN_Q_CASES = [
    # name, B, Hq, Hkv, Lq, L, dtype
    ("g4_L3000", 3, 8, 2, 1, 3000, "bf16"),        # several KV splits, ragged tail
    ("g8_L517", 2, 16, 2, 1, 517, "bf16"),
    ("rows16_L95", 1, 8, 2, 4, 95, "f16"),         # G * Lq = 16, fp16 (the two-rounding reconstruction matters)
    ("one_key", 1, 4, 1, 1, 1, "bf16"),
]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("case", ATTN_Q_CASES, ids=[c[0] for c in ATTN_Q_CASES])
def test_partial_attn_on_codes(oracle, case, bits):
    name, B, Hq, Hkv, Lq, L, dt = case
    d = 128
    dtype = W.torch_dtype(dt)
    seed = 800 + len(name) + bits
    keys = W.make_keys(Hkv, d, Lq, L, 1, seed=seed, dtype=dtype)
    rnd = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype)
    mk = lambda H, n, tid: W.activations(B, H, n, d, seed=seed, tensor_id=tid, outliers=True, dtype=dtype)
    Qs = rnd(oracle.scramble(mk(Hq, Lq, W.TID_Q), keys.phi_q, None))
    Ks = rnd(oracle.scramble(mk(Hkv, L, W.TID_K), keys.phi_k, keys.perm_kv[0]))
    Vs = rnd(oracle.scramble(mk(Hkv, L, W.TID_V), keys.phi_v, keys.perm_kv[0]))
    # codes and parameters from the ORACLE, so that both sides start from identical bits
    kc, kp = oracle.quantize_rows(Ks, bits)
    vc, vp = oracle.quantize_rows(Vs, bits)
    t = lambda a: torch.from_numpy(a).to(DEV)
    O, lse = fb.fedrag_partial_attn_quantized(Qs.to(DEV), t(kc), t(kp), t(vc), t(vp), bits)
    # the oracle's composition: reconstruct (fp32), narrow once to the storage type, attend
    Kh = torch.from_numpy(oracle.dequantize_rows(kc, kp, bits)).to(dtype)
    Vh = torch.from_numpy(oracle.dequantize_rows(vc, vp, bits)).to(dtype)
    Or, lr = oracle.partial_attn(Qs, Kh, Vh)
    PT.check_attn(O, lse, Or, lr, dtype, name)
    # and the library's own two calls one after the other consume the same reconstructed elements; the fused call
    # contracts the channels of the first product in another order (fp32 sums of exact products), nothing else
    Kd = fb.fedrag_dequantize_rows(t(kc), t(kp), bits, dtype)
    Vd = fb.fedrag_dequantize_rows(t(vc), t(vp), bits, dtype)
    O2, lse2 = fb.fedrag_partial_attn(Qs.to(DEV), Kd, Vd)
    torch.cuda.synchronize()
    do, dl = float((O - O2).abs().max()), float((lse - lse2).abs().max())
    print(f"{name} {bits} bits: fused vs two calls: O {do:.2e} lse {dl:.2e}")
    assert do <= 1e-3 and dl <= 1e-4


PREFILL_Q_CASES = [
    # name, B, Hq, Hkv, d, Lq, L, dtype                         the tiled kernel rebuilding key tiles from codes
    ("rerank_d64", 2, 4, 4, 64, 300, 300, "bf16"),             # 2 query tiles, 5 key tiles, ragged
    ("prefill_d128", 1, 8, 2, 128, 70, 500, "bf16"),           # d = 128, two chunks per thread and tile
    ("prefill_d128_f16", 1, 4, 2, 128, 200, 333, "f16"),
    ("kv_runs_d64", 1, 2, 1, 64, 40, 1500, "bf16"),            # few query tiles: keys cut into runs, partials merged
    ("decode_shape_d64", 2, 8, 2, 64, 1, 700, "bf16"),         # decode shape with d = 64: also the tiled kernel
]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("case", PREFILL_Q_CASES, ids=[c[0] for c in PREFILL_Q_CASES])
def test_partial_attn_on_codes_at_prefill_shapes(oracle, case, bits):
    name, B, Hq, Hkv, d, Lq, L, dt = case
    dtype = W.torch_dtype(dt)
    seed = 900 + len(name) + bits
    keys = W.make_keys(Hkv, d, Lq, L, 1, seed=seed, dtype=dtype)
    rnd = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype)
    mk = lambda H, n, tid: W.activations(B, H, n, d, seed=seed, tensor_id=tid, outliers=True, dtype=dtype)
    Qs = rnd(oracle.scramble(mk(Hq, Lq, W.TID_Q), keys.phi_q, keys.perm_q))
    Ks = rnd(oracle.scramble(mk(Hkv, L, W.TID_K), keys.phi_k, keys.perm_kv[0]))
    Vs = rnd(oracle.scramble(mk(Hkv, L, W.TID_V), keys.phi_v, keys.perm_kv[0]))
    kc, kp = oracle.quantize_rows(Ks, bits)
    vc, vp = oracle.quantize_rows(Vs, bits)
    t = lambda a: torch.from_numpy(a).to(DEV)
    O, lse = fb.fedrag_partial_attn_quantized(Qs.to(DEV), t(kc), t(kp), t(vc), t(vp), bits)
    Kh = torch.from_numpy(oracle.dequantize_rows(kc, kp, bits)).to(dtype)
    Vh = torch.from_numpy(oracle.dequantize_rows(vc, vp, bits)).to(dtype)
    Or, lr = oracle.partial_attn(Qs, Kh, Vh)
    PT.check_attn(O, lse, Or, lr, dtype, f"{name}/{bits}", report=True)
    # the same tiles rebuilt by the dequantise call and attended to by the 16-bit call: identical values in on-chip
    # memory, identical arithmetic after that
    Kd = fb.fedrag_dequantize_rows(t(kc), t(kp), bits, dtype)
    Vd = fb.fedrag_dequantize_rows(t(vc), t(vp), bits, dtype)
    O2, lse2 = fb.fedrag_partial_attn(Qs.to(DEV), Kd, Vd)
    torch.cuda.synchronize()
    if name != "decode_shape_d64":   # (that one compares two different kernels)
        assert torch.equal(O, O2) and torch.equal(lse, lse2), "fused call differs from dequantise + attend"


@pytest.mark.parametrize("bits", [8, 4])
def test_reranker_batch_on_codes(oracle, bits):
    """The re-ranker's padded batch (Section 5.2) with K', V' as codes (Section 7.5): per-sequence key and query
    counts, padding poisoned in the codes AND in the parameters, padding query rows not written."""
    dtype = torch.bfloat16
    B, H, d, Lmax = 5, 4, 64, 400
    lens = [400, 129, 0, 64, 333]
    seed = 950 + bits
    keys = W.make_keys(H, d, Lmax, Lmax, 1, seed=seed, dtype=dtype, permute_q=False)
    rnd = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dtype)
    mk = lambda tid: W.activations(B, H, Lmax, d, seed=seed, tensor_id=tid, outliers=True, dtype=dtype)
    Qs = rnd(oracle.scramble(mk(W.TID_Q), keys.phi_q, None))
    Ks = rnd(oracle.scramble(mk(W.TID_K), keys.phi_k, None))
    Vs = rnd(oracle.scramble(mk(W.TID_V), keys.phi_v, None))
    kc, kp = oracle.quantize_rows(Ks, bits)
    vc, vp = oracle.quantize_rows(Vs, bits)
    Kh = torch.from_numpy(oracle.dequantize_rows(kc, kp, bits)).to(dtype)
    Vh = torch.from_numpy(oracle.dequantize_rows(vc, vp, bits)).to(dtype)
    lens_t = torch.tensor(lens, dtype=torch.int32)
    Or, lr = oracle.partial_attn_varlen(Qs, Kh, Vh, lens_t)
    kc, kp, vc, vp = kc.copy(), kp.copy(), vc.copy(), vp.copy()
    for b, n in enumerate(lens):   # poison: codes all ones, parameters NaN / Inf
        kc[b, :, n:] = 255
        vc[b, :, n:] = 255
        kp[b, :, n:] = np.nan
        vp[b, :, n:] = np.inf
    t = lambda a: torch.from_numpy(a).to(DEV)
    O = torch.full((B, H, Lmax, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, H, Lmax), 7.0, dtype=torch.float32, device=DEV)
    fb.fedrag_partial_attn_varlen_quantized(Qs.to(DEV), t(kc), t(kp), t(vc), t(vp), bits, lens_t.to(DEV), O_part=O,
                                            lse=lse, q_lens=lens_t.to(DEV))
    torch.cuda.synchronize()
    for b, n in enumerate(lens):
        if n:
            PT.check_attn(O[b:b + 1, :, :n], lse[b:b + 1, :, :n], Or[b:b + 1, :, :n], lr[b:b + 1, :, :n], dtype,
                          f"pair {b} at {bits} bits", report=True)
        assert bool((O[b, :, n:] == 7.0).all()) and bool((lse[b, :, n:] == 7.0).all()), "padding rows were written"


def test_partial_attn_on_codes_rejects_fp32_storage():
    Q = torch.zeros((1, 8, 64, 128), dtype=torch.float32, device=DEV)
    c = torch.zeros((1, 2, 64, 128), dtype=torch.uint8, device=DEV)
    p = torch.zeros((1, 2, 64, 2), dtype=torch.float32, device=DEV)
    with pytest.raises(fb.FedragError) as e:
        fb.fedrag_partial_attn_quantized(Q, c, p, c, p, 8)
    assert e.value.status == fb.ERR_UNSUPPORTED
