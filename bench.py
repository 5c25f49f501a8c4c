#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of all five calls over the Llama-3-8B-shaped decode workload (batch 16, 32 query / 8 KV
heads, d 128, 4 shards of 8192 tokens, bf16): scramble_q, then per shard scramble_kv and partial_attn, then
lse_merge and unscramble.  `value` is the step's algorithmic HBM bytes divided by the step time.  The same
JSON line carries the roofline of the kernel that dominates the step, per-call figures, the RAG-prefill
TFLOP/s (2048 queries x 16384 keys) and the CPU oracle timed on a bounded sample of the same workload.

    python bench.py --gpus 1 --steps 20 --warmup 3
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a 1 GiB copy kernel of
# known size; see profiles/bench_llama8b_decode_hbm_traffic.txt for the commands and the readings).
MEASURED_TRAFFIC_BYTES = {
    "scramble_kv": int((516.46 + 512.02) * 2**20),
    "partial_attn": int((512.48 + 0.51) * 2**20),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-prefill", action="store_true", help="skip the RAG-prefill leg")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--legs", default="all",
                    help="comma-separated extra legs to run after the decode step: shards, codec, structured, rerank, "
                         "local_attn, request, mixed70b, prefill, long_decode (default: all; 'none' for the step alone)")
    ap.add_argument("--cpu-shards", type=int, default=4, help="KV shards (all sequences) the oracle is timed on")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run one 1 GiB device-to-device copy kernel before the timed region: a kernel of known "
                         "traffic to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings with")
    return ap.parse_args()


class CallTimer:
    """HIP events on the stream the kernels are launched on (torch's current stream)."""

    def __init__(self, torch):
        self.torch = torch
        self.pairs = {}

    def run(self, name, fn):
        a = self.torch.cuda.Event(enable_timing=True)
        b = self.torch.cuda.Event(enable_timing=True)
        a.record()
        out = fn()
        b.record()
        self.pairs.setdefault(name, []).append((a, b))
        return out

    def summary(self):
        out = {}
        for name, pairs in self.pairs.items():
            ms = [a.elapsed_time(b) for a, b in pairs]
            out[name] = {"calls": len(ms), "avg_us": 1e3 * sum(ms) / len(ms), "total_ms": sum(ms)}
        return out


def decode_workload(torch, W, fb, dev):
    cfg = W.CONFIGS["llama8b_decode"]
    dt = W.torch_dtype(cfg.dtype)
    keys = W.make_keys(cfg.n_kv_heads, cfg.d_head, cfg.L_q, cfg.L_kv, cfg.n_shards, seed=cfg.seed, dtype=dt)
    g = {
        "cfg": cfg,
        "Q": W.activations(cfg.batch, cfg.n_q_heads, cfg.L_q, cfg.d_head, seed=cfg.seed, tensor_id=W.TID_Q,
                           outliers=True, dtype=dt, device=dev),
        "K": [W.activations(cfg.batch, cfg.n_kv_heads, cfg.L_kv, cfg.d_head, seed=cfg.seed, tensor_id=W.TID_K + s,
                            outliers=True, outlier_id=W.TID_K, dtype=dt, device=dev) for s in range(cfg.n_shards)],
        "V": [W.activations(cfg.batch, cfg.n_kv_heads, cfg.L_kv, cfg.d_head, seed=cfg.seed, tensor_id=W.TID_V + s,
                            outliers=True, outlier_id=W.TID_V, dtype=dt, device=dev) for s in range(cfg.n_shards)],
        "keys": keys,
    }
    k = keys
    g["phi_q"], g["phi_k"], g["phi_v"], g["phi_v_inv"] = (t.to(dev) for t in (k.phi_q, k.phi_k, k.phi_v, k.phi_v_inv))
    g["perm_kv"] = [p.to(dev) for p in k.perm_kv]
    B, Hq, Hkv, d, Lq, L, S = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head, cfg.L_q, cfg.L_kv, cfg.n_shards
    g["Qs"] = torch.empty_like(g["Q"])
    g["Ks"] = [torch.empty_like(x) for x in g["K"]]
    g["Vs"] = [torch.empty_like(x) for x in g["V"]]
    g["O_parts"] = torch.empty((S, B, Hq, Lq, d), dtype=torch.float32, device=dev)
    g["lses"] = torch.empty((S, B, Hq, Lq), dtype=torch.float32, device=dev)
    g["O"] = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=dev)
    g["lse"] = torch.empty((B, Hq, Lq), dtype=torch.float32, device=dev)
    g["out"] = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=dev)
    ws = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dt, Lq, L)
    g["ws"] = torch.empty(max(ws, 16), dtype=torch.uint8, device=dev)
    es = 2
    kv_bytes = B * Hkv * L * d * es * 2          # K' + V' of one shard
    g["bytes"] = {
        "scramble_q": 2 * B * Hq * Lq * d * es,
        "scramble_kv": 2 * kv_bytes + 4 * L,     # read K,V + write K',V' + the permutation
        "partial_attn": kv_bytes + B * Hq * Lq * (d * es + d * 4 + 4),
        "lse_merge": (S + 1) * B * Hq * Lq * (d + 1) * 4,
        "unscramble": 2 * B * Hq * Lq * d * 4,
    }
    g["step_bytes"] = (g["bytes"]["scramble_q"] + S * (g["bytes"]["scramble_kv"] + g["bytes"]["partial_attn"]) +
                       g["bytes"]["lse_merge"] + g["bytes"]["unscramble"])
    return g


def decode_step(fb, g, timer=None):
    run = (lambda n, f: timer.run(n, f)) if timer else (lambda n, f: f())
    cfg = g["cfg"]
    run("scramble_q", lambda: fb.fedrag_scramble_q(g["Q"], g["phi_q"], None, Q_out=g["Qs"]))
    for s in range(cfg.n_shards):
        run("scramble_kv", lambda: fb.fedrag_scramble_kv(g["K"][s], g["V"][s], g["phi_k"], g["phi_v"], g["perm_kv"][s],
                                                         n_q_heads=cfg.n_q_heads, K_out=g["Ks"][s], V_out=g["Vs"][s]))
        run("partial_attn", lambda: fb.fedrag_partial_attn(g["Qs"], g["Ks"][s], g["Vs"][s], None,
                                                           O_part=g["O_parts"][s], lse=g["lses"][s], workspace=g["ws"]))
    run("lse_merge", lambda: fb.fedrag_lse_merge(g["O_parts"], g["lses"], n_kv_heads=cfg.n_kv_heads,
                                                 O_out=g["O"], lse_out=g["lse"]))
    run("unscramble", lambda: fb.fedrag_unscramble(g["O"], g["phi_v_inv"], None, O_out=g["out"]))


def graph_leg(torch, fb, g, steps):
    """Record one decode step into a HIP graph, check one replay against the eager outputs bit for bit, then time
    `steps` replays between synchronisations.  Returns ms per step, or None if the replay does not reproduce."""
    torch.cuda.synchronize()
    ref = (g["out"].clone(), g["lse"].clone())
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            decode_step(fb, g)
    torch.cuda.current_stream().wait_stream(side)
    g["out"].fill_(0.0)
    g["lse"].fill_(0.0)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    if not (torch.equal(g["out"], ref[0]) and torch.equal(g["lse"], ref[1])):
        return None
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return 1e3 * (time.perf_counter() - t0) / steps


def shards_leg(torch, fb, g, steps, warmup):
    """Rows a3 + a4 of the decode step as one call over the 4 shards (after the step has left K', V' in place)."""
    cfg = g["cfg"]
    need = fb.fedrag_partial_attn_shards_workspace_bytes(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head,
                                                         g["Qs"].dtype, cfg.L_q, [cfg.L_kv] * cfg.n_shards)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=g["Qs"].device)
    O, lse = torch.empty_like(g["O"]), torch.empty_like(g["lse"])
    call = lambda: fb.fedrag_partial_attn_shards(g["Qs"], g["Ks"], g["Vs"], None, O=O, lse=lse, workspace=ws)
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(steps):
        timer.run("a", call)
    torch.cuda.synchronize()
    us = timer.summary()["a"]["avg_us"]
    nb = cfg.n_shards * g["bytes"]["partial_attn"]
    # the aggregation adds the partials in another order than per shard + across shards: equal to rounding
    err = float((O - g["O"]).abs().max())
    return {"call": "partial_attn_shards (4 shards + aggregation)", "avg_us": round(us, 2), "bytes": nb,
            "GB/s": round(nb / us / 1e3, 1), "frac_hbm": round(nb / us / 1e3 / HBM_PEAK_GBS, 4),
            "max_abs_diff_vs_step": err}


def structured_leg(torch, W, fb, g, dev, steps, warmup):
    """Enc of one KV shard with the keys in structured form (S1 P1 H P2 S2 by its factors): same bytes as scramble_kv."""
    cfg = g["cfg"]
    dt = W.torch_dtype(cfg.dtype)
    ks = W.make_structured_keys(cfg.n_kv_heads, cfg.d_head, cfg.L_q, cfg.L_kv, 1, seed=cfg.seed, dtype=dt)
    kk, kv = tuple(t.to(dev) for t in ks.k), tuple(t.to(dev) for t in ks.v)
    perm = ks.perm_kv[0].to(dev)
    call = lambda: fb.fedrag_scramble_kv_structured(g["K"][0], g["V"][0], kk, kv, perm, n_q_heads=cfg.n_q_heads,
                                                    K_out=g["Ks"][0], V_out=g["Vs"][0])
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(steps):
        timer.run("scramble_kv_structured", call)
    torch.cuda.synchronize()
    t = timer.summary()["scramble_kv_structured"]
    gbs = g["bytes"]["scramble_kv"] / (t["avg_us"] * 1e-6) / 1e9
    return {"call": "scramble_kv_structured", "avg_us": round(t["avg_us"], 2), "bytes": g["bytes"]["scramble_kv"],
            "GB/s": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}


def local_attn_leg(torch, W, fb, dev, steps, warmup):
    """The Inquirer's own part of a segment's attention: 4096 plaintext tokens attending to themselves and their
    predecessors, Llama-3-8B head shape.  Counted flops: 4 d Hq Lq (Lq + 1) / 2 (visible pairs only)."""
    B, Hq, Hkv, d, L = 1, 32, 8, 128, 4096
    dt = torch.bfloat16
    mk = lambda H, tid: W.activations(B, H, L, d, seed=W.BASE_SEED + 6, tensor_id=tid, outliers=True, outlier_id=tid,
                                      dtype=dt, device=dev)
    Q, K, V = mk(Hq, W.TID_Q), mk(Hkv, W.TID_K), mk(Hkv, W.TID_V)
    O = torch.empty((B, Hq, L, d), dtype=torch.float32, device=dev)
    lse = torch.empty((B, Hq, L), dtype=torch.float32, device=dev)
    for _ in range(warmup):
        fb.fedrag_local_attn(Q, K, V, None, O_part=O, lse=lse)
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(steps):
        timer.run("local_attn", lambda: fb.fedrag_local_attn(Q, K, V, None, O_part=O, lse=lse))
    torch.cuda.synchronize()
    t = timer.summary()["local_attn"]
    flop = 4.0 * d * Hq * B * (L * (L + 1) / 2)
    tflops = flop / (t["avg_us"] * 1e-6) / 1e12
    return {"workload": "local_attn: B1 Hq32 Hkv8 d128, 4096-token segment, bf16", "flop": flop,
            "avg_us": round(t["avg_us"], 2), "value": round(tflops, 1), "unit": "TFLOP/s",
            "frac_mfma": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4)}


def rerank_leg(torch, W, fb, dev, steps, warmup):
    """Re-ranking shape (Section 7.1: 10 candidate documents): 10 query-document pairs of unequal length, 16 heads of
    64 channels, bidirectional attention of every token of a pair over the pair, padded to 1024 tokens."""
    B, H, d, Lmax = 10, 16, 64, 1024
    lens = [1024, 896, 777, 640, 512, 512, 400, 333, 256, 130]
    dt = torch.bfloat16
    mk = lambda tid: W.activations(B, H, Lmax, d, seed=W.BASE_SEED + 7, tensor_id=tid, outliers=True, outlier_id=tid,
                                   dtype=dt, device=dev)
    keys = W.make_keys(H, d, Lmax, Lmax, 1, seed=W.BASE_SEED + 7, dtype=dt, permute_q=False)
    Qs = fb.fedrag_scramble_q(mk(W.TID_Q), keys.phi_q.to(dev), None)
    Ks, Vs = fb.fedrag_scramble_kv(mk(W.TID_K), mk(W.TID_V), keys.phi_k.to(dev), keys.phi_v.to(dev), None)
    kv = torch.tensor(lens, dtype=torch.int32, device=dev)
    O = torch.empty((B, H, Lmax, d), dtype=torch.float32, device=dev)
    lse = torch.empty((B, H, Lmax), dtype=torch.float32, device=dev)
    call = lambda: fb.fedrag_partial_attn_varlen(Qs, Ks, Vs, kv, None, O_part=O, lse=lse, q_lens=kv)
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(steps):
        timer.run("rerank", call)
    torch.cuda.synchronize()
    t = timer.summary()["rerank"]
    flop = sum(4.0 * n * n * d * H for n in lens)   # real pairs only: n queries x n keys
    return {"workload": "rerank: 10 pairs of 130..1024 tokens padded to 1024, 16 heads x 64, bf16, bidirectional",
            "flop_valid_pairs": flop, "avg_us": round(t["avg_us"], 2),
            "value": round(flop / (t["avg_us"] * 1e-6) / 1e12, 1), "unit": "TFLOP/s"}


def mixed_leg(torch, W, fb, dev, steps, warmup):
    """70B-shaped mixed batch (64 query heads over 8 KV heads, 8 shards x 8192 tokens): 32 decoding sequences and one
    4096-token prefill chunk.  partial_attn over the 8 shards + lse_merge for each part, alone and with the two parts
    issued on two streams at once (scramble_kv is timed on its own in the main step)."""
    cd, cp = W.CONFIGS["mixed70b_decode"], W.CONFIGS["mixed70b_prefill"]
    dt = W.torch_dtype(cd.dtype)
    S, d = cd.n_shards, cd.d_head
    gen = torch.Generator(device=dev)
    gen.manual_seed(cd.seed)
    rnd = lambda *shape: torch.randn(shape, generator=gen, device=dev).to(dt)

    def part(cfg):
        Q = rnd(cfg.batch, cfg.n_q_heads, cfg.L_q, d)
        KV = [(rnd(cfg.batch, cfg.n_kv_heads, cfg.L_kv, d), rnd(cfg.batch, cfg.n_kv_heads, cfg.L_kv, d))
              for _ in range(S)]
        O = torch.empty((S, cfg.batch, cfg.n_q_heads, cfg.L_q, d), dtype=torch.float32, device=dev)
        lse = torch.empty((S, cfg.batch, cfg.n_q_heads, cfg.L_q), dtype=torch.float32, device=dev)
        Om, lm = torch.empty_like(O[0]), torch.empty_like(lse[0])
        need = fb.fedrag_partial_attn_workspace_bytes(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, d, dt, cfg.L_q, cfg.L_kv)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

        def run():
            for s_ in range(S):
                fb.fedrag_partial_attn(Q, KV[s_][0], KV[s_][1], None, O_part=O[s_], lse=lse[s_], workspace=ws)
            fb.fedrag_lse_merge(O, lse, O_out=Om, lse_out=lm)
        need1 = fb.fedrag_partial_attn_shards_workspace_bytes(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, d, dt, cfg.L_q,
                                                              [cfg.L_kv] * S)
        ws1 = torch.empty(max(need1, 16), dtype=torch.uint8, device=dev)

        def run_one_call():
            fb.fedrag_partial_attn_shards(Q, [kv[0] for kv in KV], [kv[1] for kv in KV], None, O=Om, lse=lm,
                                          workspace=ws1)
        return run, run_one_call

    (run_d, run_d1), (run_p, run_p1) = part(cd), part(cp)
    s_d, s_p = torch.cuda.Stream(), torch.cuda.Stream()   # default priority, both

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return 1e3 * (time.perf_counter() - t0) / steps

    def both():
        with torch.cuda.stream(s_p):
            run_p()
        with torch.cuda.stream(s_d):
            run_d()

    ms_d, ms_p, ms_b = timed(run_d), timed(run_p), timed(both)
    ms_d1, ms_p1 = timed(run_d1), timed(run_p1)
    byts = 4.0 * d * cd.batch * cd.n_kv_heads * cd.L_kv * S              # K' + V', 16-bit, read once per KV head
    flop = 4.0 * cp.L_q * cp.L_kv * S * d * cp.n_q_heads * cp.batch
    return {"workload": "mixed70b: Hq64 Hkv8 d128, 8 shards x 8192 tokens, bf16; 32 decode sequences + one 4096-token "
                        "prefill chunk; partial_attn x 8 + lse_merge per part",
            "decode": {"ms": round(ms_d, 4), "GB/s": round(byts / ms_d / 1e6, 1),
                       "frac_hbm": round(byts / ms_d / 1e6 / HBM_PEAK_GBS, 4)},
            "prefill": {"ms": round(ms_p, 4), "TFLOP/s": round(flop / ms_p / 1e9, 1),
                        "frac_mfma": round(flop / ms_p / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)},
            "decode_one_call": {"ms": round(ms_d1, 4), "GB/s": round(byts / ms_d1 / 1e6, 1),
                                "frac_hbm": round(byts / ms_d1 / 1e6 / HBM_PEAK_GBS, 4)},
            "prefill_one_call": {"ms": round(ms_p1, 4), "TFLOP/s": round(flop / ms_p1 / 1e9, 1),
                                 "frac_mfma": round(flop / ms_p1 / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)},
            "both_on_two_streams_ms": round(ms_b, 4), "sum_ms": round(ms_d + ms_p, 4),
            "max_ms": round(max(ms_d, ms_p), 4)}


def request_leg(torch, W, fb, dev, steps, warmup, n_layers=32):
    """The attention path of one request at the largest length configuration of Section 7.1 (context 4096 + 4096 on
    two Context Owners, 128-token query segment), Llama-3-8B-shaped (32 layers, 32/8 heads of 128), batch 1:
    per layer scramble_q -> attention on the two shards and their aggregation -> the Inquirer's own causal attention
    -> Dec and the aggregation of the two.  Once for the 128-token segment (prefill) and once for one decoded token
    (the segment's 128 + 64 generated tokens local), each as one HIP graph of all layers; with the fused calls
    (partial_attn_shards, unscramble_merge: 4 calls per layer) and call by call (8 calls per layer)."""
    B, Hq, Hkv, d, S, Lc, Lseg, Lgen = 1, 32, 8, 128, 2, 4096, 128, 64
    dt = torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.BASE_SEED + 9)
    rnd = lambda *shape: torch.randn(shape, generator=gen, device=dev).to(dt)
    keys = W.make_keys(Hkv, d, Lseg, Lc, S, seed=W.BASE_SEED + 9, dtype=dt)
    phi_q, phi_vi = keys.phi_q.to(dev), keys.phi_v_inv.to(dev)
    # per layer: the scrambled caches the Compute Node holds (distinct memory per layer, 1 GiB in all)
    Ks = [[rnd(B, Hkv, Lc, d) for _ in range(S)] for _ in range(n_layers)]
    Vs = [[rnd(B, Hkv, Lc, d) for _ in range(S)] for _ in range(n_layers)]

    def chain(Lq, L_local, fused):
        Q = rnd(B, Hq, Lq, d)
        Kl = [rnd(B, Hkv, L_local, d) for _ in range(n_layers)]   # the Inquirer's own plaintext K, V per layer
        Vl = [rnd(B, Hkv, L_local, d) for _ in range(n_layers)]
        perm_q = keys.perm_q.to(dev) if Lq == Lseg else None
        f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
        Qs = torch.empty_like(Q)
        Op, lp = f32(S, B, Hq, Lq, d), f32(S, B, Hq, Lq)
        Om, lm, Ou, lu = f32(B, Hq, Lq, d), f32(B, Hq, Lq), f32(B, Hq, Lq, d), f32(B, Hq, Lq)
        pair_O, pair_l = f32(2, B, Hq, Lq, d), f32(2, B, Hq, Lq)
        out, out_l = f32(B, Hq, Lq, d), f32(B, Hq, Lq)
        need = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dt, Lq, Lc)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        need_l = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dt, Lq, L_local)
        ws_l = torch.empty(max(need_l, 16), dtype=torch.uint8, device=dev)

        need_s = fb.fedrag_partial_attn_shards_workspace_bytes(B, Hq, Hkv, d, dt, Lq, [Lc] * S)
        ws_s = torch.empty(max(need_s, 16), dtype=torch.uint8, device=dev)

        def layer_fused(i):
            fb.fedrag_scramble_q(Q, phi_q, perm_q, Q_out=Qs)
            fb.fedrag_partial_attn_shards(Qs, Ks[i], Vs[i], None, O=Om, lse=lm, workspace=ws_s)
            fb.fedrag_local_attn(Q, Kl[i], Vl[i], None, O_part=pair_O[1], lse=pair_l[1], workspace=ws_l)
            fb.fedrag_unscramble_merge(Om, lm, phi_vi, perm_q, pair_O[1], pair_l[1], O_out=out, lse_out=out_l,
                                       n_kv_heads=Hkv)

        def layer(i):
            if fused:
                return layer_fused(i)
            fb.fedrag_scramble_q(Q, phi_q, perm_q, Q_out=Qs)
            for s_ in range(S):
                fb.fedrag_partial_attn(Qs, Ks[i][s_], Vs[i][s_], None, O_part=Op[s_], lse=lp[s_], workspace=ws)
            fb.fedrag_lse_merge(Op, lp, n_kv_heads=Hkv, O_out=Om, lse_out=lm)
            fb.fedrag_unscramble(Om, phi_vi, perm_q, O_out=pair_O[0])
            fb.fedrag_unpermute_lse(lm, perm_q, lse_out=pair_l[0])
            fb.fedrag_local_attn(Q, Kl[i], Vl[i], None, O_part=pair_O[1], lse=pair_l[1], workspace=ws_l)
            fb.fedrag_lse_merge(pair_O, pair_l, n_kv_heads=Hkv, O_out=out, lse_out=out_l)

        def all_layers():
            for i in range(n_layers):
                layer(i)
        return all_layers, out

    res = {"workload": "request: B1 Hq32 Hkv8 d128 bf16, 32 layers, context 4096 + 4096 on 2 shards, 128-token query "
                       "segment; 4 C-ABI calls per layer (call_by_call: 8)"}
    for name, Lq, L_local, fused in (("segment_prefill", Lseg, Lseg, True), ("decode_token", 1, Lseg + Lgen, True),
                                     ("segment_prefill_call_by_call", Lseg, Lseg, False),
                                     ("decode_token_call_by_call", 1, Lseg + Lgen, False)):
        run, out = chain(Lq, L_local, fused)
        for _ in range(max(1, warmup)):
            run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        eager_ms = 1e3 * (time.perf_counter() - t0) / steps
        ref = out.clone()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                run()
        torch.cuda.current_stream().wait_stream(side)
        out.fill_(0.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        same = bool(torch.equal(out, ref))
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - t0) / steps
        res[name] = {"eager_ms": round(eager_ms, 4), "graph_ms": round(graph_ms, 4),
                     "graph_us_per_layer": round(1e3 * graph_ms / n_layers, 2), "replay_equals_eager": same}
    res["decode_token"]["tokens_per_s_attention_path"] = round(1e3 / res["decode_token"]["graph_ms"], 1)
    return res


def long_decode_leg(torch, W, fb, dev, steps, warmup):
    """Long-context decode (B64, 32/8 heads, d128, 8 shards x 32768 tokens, bf16): rows a3 + a4 with all 64 GiB of
    K', V' resident, as one call over the 8 shards and shard by shard."""
    cfg = W.CONFIGS["long_decode"]
    dt = W.torch_dtype(cfg.dtype)
    B, Hq, Hkv, d, S, L = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head, cfg.n_shards, cfg.L_kv
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)

    def rnd(*shape):   # drawn in slabs so that the fp32 intermediate stays small
        out = torch.empty(shape, dtype=dt, device=dev)
        for b in range(shape[0]):
            out[b] = torch.randn(shape[1:], generator=gen, device=dev).to(dt)
        return out
    Q = rnd(B, Hq, 1, d)
    Ks = [rnd(B, Hkv, L, d) for _ in range(S)]
    Vs = [rnd(B, Hkv, L, d) for _ in range(S)]
    O, lse = torch.empty((B, Hq, 1, d), dtype=torch.float32, device=dev), torch.empty((B, Hq, 1), dtype=torch.float32, device=dev)
    Op = torch.empty((S, B, Hq, 1, d), dtype=torch.float32, device=dev)
    lp = torch.empty((S, B, Hq, 1), dtype=torch.float32, device=dev)
    need = fb.fedrag_partial_attn_shards_workspace_bytes(B, Hq, Hkv, d, dt, 1, [L] * S)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    need1 = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dt, 1, L)
    ws1 = torch.empty(max(need1, 16), dtype=torch.uint8, device=dev)

    def one_call():
        fb.fedrag_partial_attn_shards(Q, Ks, Vs, None, O=O, lse=lse, workspace=ws)

    def per_shard():
        for s_ in range(S):
            fb.fedrag_partial_attn(Q, Ks[s_], Vs[s_], None, O_part=Op[s_], lse=lp[s_], workspace=ws1)
        fb.fedrag_lse_merge(Op, lp, n_kv_heads=Hkv, O_out=O, lse_out=lse)

    out = {"workload": "long_decode: B64 Hq32 Hkv8 d128 Lq1, 8 shards x 32768 tokens, bf16 (64 GiB of K', V')"}
    # Enc of one shard at this size (8 GiB read, 8 GiB written), into a spare pair of buffers
    keys = W.make_keys(Hkv, d, 1, L, 1, seed=cfg.seed, dtype=dt)
    phi_k, phi_v, perm = keys.phi_k.to(dev), keys.phi_v.to(dev), keys.perm_kv[0].to(dev)
    Ko, Vo = torch.empty_like(Ks[0]), torch.empty_like(Vs[0])
    enc = lambda: fb.fedrag_scramble_kv(Ks[0], Vs[0], phi_k, phi_v, perm, n_q_heads=Hq, K_out=Ko, V_out=Vo)
    enc()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        enc()
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / 3
    enc_bytes = 8.0 * d * B * Hkv * L
    out["scramble_kv_one_shard"] = {"ms": round(ms, 3), "GB/s": round(enc_bytes / ms / 1e6, 1),
                                    "frac_hbm": round(enc_bytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
    del Ko, Vo
    byts = 4.0 * d * B * Hkv * L * S
    for name, fn in (("one_call", one_call), ("shard_by_shard", per_shard)):
        for _ in range(max(1, warmup // 2)):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        ms = 1e3 * (time.perf_counter() - t0) / steps
        out[name] = {"ms": round(ms, 3), "GB/s": round(byts / ms / 1e6, 1),
                     "frac_hbm": round(byts / ms / 1e6 / HBM_PEAK_GBS, 4)}
    return out


def codec_leg(torch, fb, g, steps, warmup):
    """Transport codec on one shard's K' ([16, 8, 8192, 128] bf16): quantise to 8 bits and back, bytes = read + write."""
    X = g["Ks"][0]
    n = X.numel() // X.shape[-1]
    d = X.shape[-1]
    out = {}
    for bits in (8, 4):
        codes, params = fb.fedrag_quantize_rows(X, bits)
        Xh = torch.empty_like(X)
        q = lambda: fb.fedrag_quantize_rows(X, bits, codes=codes, params=params)
        dq = lambda: fb.fedrag_dequantize_rows(codes, params, bits, X.dtype, X_out=Xh)
        for _ in range(warmup):
            q(); dq()
        torch.cuda.synchronize()
        timer = CallTimer(torch)
        for _ in range(steps):
            timer.run("q", q)
            timer.run("dq", dq)
        torch.cuda.synchronize()
        t = timer.summary()
        nbytes = n * (d * 2 + d * bits // 8 + 8)
        out[f"{bits}bit"] = {"quantize_us": round(t["q"]["avg_us"], 2), "dequantize_us": round(t["dq"]["avg_us"], 2),
                             "bytes": nbytes, "quantize_GB/s": round(nbytes / t["q"]["avg_us"] / 1e3, 1),
                             "dequantize_GB/s": round(nbytes / t["dq"]["avg_us"] / 1e3, 1)}
    # Enc with the codec as its epilogue (what a Context Owner sends): one shard, K and V
    cfg = g["cfg"]
    outs = fb.fedrag_scramble_kv_quantized(g["K"][0], g["V"][0], g["phi_k"], g["phi_v"], g["perm_kv"][0], 8,
                                           n_q_heads=cfg.n_q_heads)
    call = lambda: fb.fedrag_scramble_kv_quantized(g["K"][0], g["V"][0], g["phi_k"], g["phi_v"], g["perm_kv"][0], 8,
                                                   n_q_heads=cfg.n_q_heads, out=outs)
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(steps):
        timer.run("f", call)
    torch.cuda.synchronize()
    us = timer.summary()["f"]["avg_us"]
    nb = 2 * n * (d * 2 + d + 8) + 4 * cfg.L_kv
    out["scramble_kv_quantized_8bit"] = {"avg_us": round(us, 2), "bytes": nb, "GB/s": round(nb / us / 1e3, 1)}
    # the Compute Node's decode call reading the codes directly (one shard)
    for bits in (8, 4):
        Kc, Kp, Vc, Vp = fb.fedrag_scramble_kv_quantized(g["K"][0], g["V"][0], g["phi_k"], g["phi_v"], g["perm_kv"][0],
                                                         bits, n_q_heads=cfg.n_q_heads)
        call = lambda: fb.fedrag_partial_attn_quantized(g["Qs"], Kc, Kp, Vc, Vp, bits, None, O_part=g["O_parts"][0],
                                                        lse=g["lses"][0], workspace=g["ws"])
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        timer = CallTimer(torch)
        for _ in range(steps):
            timer.run("a", call)
        torch.cuda.synchronize()
        us = timer.summary()["a"]["avg_us"]
        nb = 2 * n * (d * bits // 8 + 8)
        out[f"partial_attn_quantized_{bits}bit"] = {"avg_us": round(us, 2), "bytes_read": nb,
                                                    "GB/s": round(nb / us / 1e3, 1)}
    return out


def prefill_leg(torch, W, fb, dev, steps, warmup):
    """RAG prefill: partial_attn alone, 2048 queries x 16384 keys, 32/8 heads, d 128, bf16."""
    cfg = W.CONFIGS["rag_prefill"]
    dt = W.torch_dtype(cfg.dtype)
    mk = lambda H, L, tid, oid: W.activations(cfg.batch, H, L, cfg.d_head, seed=cfg.seed, tensor_id=tid, outliers=True,
                                              outlier_id=oid, dtype=dt, device=dev)
    Q, K, V = mk(cfg.n_q_heads, cfg.L_q, W.TID_Q, W.TID_Q), mk(cfg.n_kv_heads, cfg.L_kv, W.TID_K, W.TID_K), \
        mk(cfg.n_kv_heads, cfg.L_kv, W.TID_V, W.TID_V)
    keys = W.make_keys(cfg.n_kv_heads, cfg.d_head, cfg.L_q, cfg.L_kv, 1, seed=cfg.seed, dtype=dt)
    Qs = fb.fedrag_scramble_q(Q, keys.phi_q.to(dev), keys.perm_q.to(dev))
    Ks, Vs = fb.fedrag_scramble_kv(K, V, keys.phi_k.to(dev), keys.phi_v.to(dev), keys.perm_kv[0].to(dev))
    O = torch.empty((cfg.batch, cfg.n_q_heads, cfg.L_q, cfg.d_head), dtype=torch.float32, device=dev)
    lse = torch.empty((cfg.batch, cfg.n_q_heads, cfg.L_q), dtype=torch.float32, device=dev)
    for _ in range(warmup):
        fb.fedrag_partial_attn(Qs, Ks, Vs, None, O_part=O, lse=lse)
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(steps):
        timer.run("partial_attn", lambda: fb.fedrag_partial_attn(Qs, Ks, Vs, None, O_part=O, lse=lse))
    torch.cuda.synchronize()
    t = timer.summary()["partial_attn"]
    # the Inquirer's two calls around it at this size (a2 before, a5 after)
    phi_q, perm_q, phi_vi = keys.phi_q.to(dev), keys.perm_q.to(dev), keys.phi_v_inv.to(dev)
    out = torch.empty_like(O)
    for _ in range(steps):
        timer.run("scramble_q", lambda: fb.fedrag_scramble_q(Q, phi_q, perm_q, Q_out=Qs))
        timer.run("unscramble", lambda: fb.fedrag_unscramble(O, phi_vi, perm_q, O_out=out))
    torch.cuda.synchronize()
    around = {k: round(v["avg_us"], 2) for k, v in timer.summary().items() if k != "partial_attn"}
    flop = 4.0 * cfg.L_q * cfg.L_kv * cfg.d_head * cfg.n_q_heads * cfg.batch
    tflops = flop / (t["avg_us"] * 1e-6) / 1e12
    return {"workload": "rag_prefill: B1 Hq32 Hkv8 d128 Lq2048 Lkv16384 bf16, non-causal", "flop": flop,
            "avg_us": t["avg_us"], "value": tflops, "unit": "TFLOP/s", "inquirer_calls_avg_us": around,
            "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": tflops / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
                         "kernel": "prefill_attn_kernel<BF16,128>"}}


def cpu_leg(torch, W, g, n_shards):
    """The oracle, as it stands, on the first n_shards KV shards (all sequences): scramble_q, then per shard scramble
    of K and V and partial attention, then merge and unscramble - the same step the GPU is timed on."""
    import numpy as np
    import oracle
    cfg = g["cfg"]
    n_shards = max(1, min(n_shards, cfg.n_shards))
    k = g["keys"]
    Q = g["Q"].cpu()
    Kc = [g["K"][s].cpu() for s in range(n_shards)]
    Vc = [g["V"][s].cpu() for s in range(n_shards)]
    t0 = time.perf_counter()
    Qs = oracle.scramble(Q, k.phi_q, None)
    parts, lses = [], []
    for s in range(n_shards):
        Ks = oracle.scramble(Kc[s], k.phi_k, k.perm_kv[s])
        Vs = oracle.scramble(Vc[s], k.phi_v, k.perm_kv[s])
        o, l = oracle.partial_attn(Qs, Ks, Vs)
        parts.append(o); lses.append(l)
        del Ks, Vs
    O, lse = oracle.lse_merge(np.stack(parts), np.stack(lses))
    out = oracle.unscramble(O, k.phi_v_inv, None)
    dt = time.perf_counter() - t0
    b = g["bytes"]
    nbytes = b["scramble_q"] + n_shards * (b["scramble_kv"] + b["partial_attn"]) + \
        b["lse_merge"] * (n_shards + 1) / (cfg.n_shards + 1) + b["unscramble"]
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": oracle.get_threads(), "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"KV shards 0..{n_shards - 1} of {cfg.n_shards}, all {cfg.batch} sequences: the whole step in fp64 "
                      f"({nbytes / 2**30:.2f} GiB of the step's {g['step_bytes'] / 2**30:.2f} GiB algorithmic bytes)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (federation nodes are simulated as sequential KV shards "
              "on that GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2605_25716_amd import binding as fb
    from paper_2605_25716_amd import build as fbuild
    from paper_2605_25716_amd import workloads as W
    if not os.path.exists(fbuild.LIB_PATH):
        fbuild.build_library(force=True)
    fb.load()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    torch.cuda.set_device(0)

    g = decode_workload(torch, W, fb, dev)
    if args.pmc_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        b.copy_(a)          # the reference kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        decode_step(fb, g)
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        decode_step(fb, g, timer)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = 1e3 * wall / args.steps
    value = g["step_bytes"] / (ms_per_step * 1e-3) / 1e9

    # the same K steps once more, replayed from a HIP graph (what a serving loop would do): no host time between launches
    graph_ms = None
    if not args.no_graph:
        graph_ms = graph_leg(torch, fb, g, args.steps)

    calls = timer.summary()
    per_call = {}
    for name, t in calls.items():
        gbs = g["bytes"][name] / (t["avg_us"] * 1e-6) / 1e9
        per_call[name] = {"avg_us": round(t["avg_us"], 2), "calls_per_step": t["calls"] // args.steps,
                          "bytes": g["bytes"][name], "GB/s": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
    kernel_of = {"scramble_kv": "scramble_rows_kernel<BF16,128,false,0>", "partial_attn": "decode_attn_kernel<BF16,128>"}
    dom = max(kernel_of, key=lambda n: calls[n]["total_ms"])
    roofline = {"bound": "hbm", "achieved": per_call[dom]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(per_call[dom]["GB/s"] / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(dom),
                "kernel": kernel_of[dom], "call": dom, "avg_us": per_call[dom]["avg_us"],
                "bytes_per_launch": g["bytes"][dom]}
    # the spec kernel on its own: K'/V' streaming of partial_attn (+ split merge) over the 4 shards
    attn = per_call["partial_attn"]

    line = {
        "metric": "scrambled partial-attn: decode HBM GB/s + prefill TFLOP/s (% of peak)",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "llama8b_decode: B16 Hq32 Hkv8 d128 Lq1, 4 shards x 8192 tokens, bf16; "
                               "step = scramble_q + 4x(scramble_kv + partial_attn) + lse_merge + unscramble",
                   "step_bytes": g["step_bytes"]},
        "roofline": roofline,
        "decode_partial_attn": {"GB/s": attn["GB/s"], "frac_hbm": attn["frac_hbm"], "avg_us": attn["avg_us"]},
        "calls": per_call,
    }
    line["config"]["launch"] = "eager: one C-ABI call after the other from Python, HIP events around each call"
    if graph_ms is not None:
        # headline = the K steps replayed from a HIP graph (same kernels, same buffers, no host time between launches);
        # the eager loop, which also carries the per-call events the roofline is computed from, is kept beside it
        line["eager"] = {"ms_per_step": line["ms_per_step"], "GB/s": line["value"],
                         "frac_hbm": round(line["value"] / HBM_PEAK_GBS, 4)}
        line["ms_per_step"] = round(graph_ms, 4)
        line["value"] = round(g["step_bytes"] / (graph_ms * 1e-3) / 1e9, 1)
        line["config"]["launch"] = ("the step recorded once into a HIP graph and replayed K times between "
                                    "synchronisations (outputs checked equal to the eager ones bit for bit); "
                                    "'eager' = the same K steps launched call by call from Python")
    line["frac_hbm"] = round(line["value"] / HBM_PEAK_GBS, 4)
    all_legs = ("shards", "codec", "structured", "rerank", "local_attn", "request", "mixed70b", "prefill",
                "long_decode")
    want = set(all_legs) if args.legs == "all" else {x for x in args.legs.split(",") if x and x != "none"}
    unknown = want - set(all_legs)
    if unknown:
        print(f"bench.py: unknown legs {sorted(unknown)}; known: {', '.join(all_legs)}", file=sys.stderr)
        sys.exit(2)
    if args.no_prefill:
        want -= {"rerank", "local_attn", "request", "mixed70b", "prefill", "long_decode"}
    half = max(5, args.steps // 2)

    def leg(name, fn):
        """The extra legs must not cost the headline its JSON line: a leg that fails reports its error instead."""
        if name not in want:
            return
        try:
            line[name] = fn()
        except Exception as e:  # noqa: BLE001 - reported in the line, the step above is already measured
            torch.cuda.synchronize()
            line[name] = {"error": f"{type(e).__name__}: {e}"}
            print(f"bench.py: leg {name} failed: {e}", file=sys.stderr)

    leg("shards", lambda: shards_leg(torch, fb, g, args.steps, args.warmup))
    leg("codec", lambda: codec_leg(torch, fb, g, args.steps, args.warmup))
    leg("structured", lambda: structured_leg(torch, W, fb, g, dev, args.steps, args.warmup))
    leg("rerank", lambda: rerank_leg(torch, W, fb, dev, half, args.warmup))
    leg("local_attn", lambda: local_attn_leg(torch, W, fb, dev, half, args.warmup))
    leg("request", lambda: request_leg(torch, W, fb, dev, half, args.warmup))
    leg("mixed70b", lambda: mixed_leg(torch, W, fb, dev, half, args.warmup))
    leg("prefill", lambda: prefill_leg(torch, W, fb, dev, half, args.warmup))
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_leg(torch, W, g, args.cpu_shards)
    if "long_decode" in want:   # last: it takes 64 GiB of device memory
        del g
        torch.cuda.empty_cache()
        leg("long_decode", lambda: long_decode_leg(torch, W, fb, dev, 5, args.warmup))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
