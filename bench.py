#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of all five calls over the Llama-3-8B-shaped decode workload (batch 16, 32 query / 8 KV
heads, d 128, 4 shards of 8192 tokens, bf16): scramble_q, then per shard scramble_kv and partial_attn, then
lse_merge and unscramble.  `value` is the step's algorithmic HBM bytes divided by the step time.  The same
JSON line carries the roofline of the kernel that dominates the step (`roofline`) and of the two attention kernels
a target is stated for (`rooflines`), per-call figures, what a plain copy and a bare MFMA loop reach on the device in
the same run (`achievable`), one leg per other configuration (RAG prefill, long-context decode, the 70B-shaped mixed
batch, request-sized chains, re-ranking, codec, structured keys; medians of at least 20 iterations) and the CPU
oracle timed on the host cores: on the whole step, and on the other configurations in full or on a scaled sample.

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

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy kernel of known size.
# Counters cannot be read from inside this program: the figures are those of the named profile, which was taken
# with this file's own command line, and they go stale when the kernel changes (re-run the profile then).
TRAFFIC_PROFILE = "profiles/bench_llama8b_decode_hbm_traffic.txt"
MEASURED_TRAFFIC_BYTES = {
    "scramble_kv": int((516.48 + 512.03) * 2**20),
    "partial_attn": int((512.57 + 0.51) * 2**20),
}
MIN_ITERS = 20   # timed iterations of every extra leg (medians are reported beside the means)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-prefill", action="store_true", help="skip the RAG-prefill leg")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay of the step")
    ap.add_argument("--legs", default="all",
                    help="comma-separated extra legs to run after the decode step: achievable, shards, codec, structured, "
                         "rerank, local_attn, request, mixed70b, prefill, long_decode (default: all; 'none' for the "
                         "step alone)")
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
            ms = sorted(a.elapsed_time(b) for a, b in pairs)
            med = (ms[len(ms) // 2] + ms[(len(ms) - 1) // 2]) / 2
            # an event pair also spans whatever held the host or the device up between its two records; a sample
            # beyond three medians is such a stall, not the call: it is left out of the mean and counted instead
            kept = [x for x in ms if x <= 3.0 * med]
            out[name] = {"calls": len(ms), "avg_us": 1e3 * sum(kept) / len(kept), "total_ms": sum(kept),
                         "med_us": 1e3 * med, "stalls_left_out": len(ms) - len(kept), "max_us": 1e3 * ms[-1]}
        return out


def measure(torch, fn, iters, warmup):
    """`warmup` untimed calls of fn, then `iters` calls each between its own pair of HIP events on the current
    stream.  Returns {"avg_us", "med_us", "iters"}."""
    for _ in range(max(1, warmup)):
        fn()
    torch.cuda.synchronize()
    timer = CallTimer(torch)
    for _ in range(iters):
        timer.run("x", fn)
    torch.cuda.synchronize()
    t = timer.summary()["x"]
    out = {"avg_us": t["avg_us"], "med_us": t["med_us"], "iters": iters}
    if t["stalls_left_out"]:
        out["stalls_left_out"] = t["stalls_left_out"]
        out["max_us"] = t["max_us"]
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
    `steps` replays between synchronisations.  Returns (ms per step, the three regions), or None if the replay does
    not reproduce."""
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
    # three timed regions of exactly `steps` replays, each between synchronisations; the middle one is reported, so
    # that one stall of the host or the box (seen once: 25 ms) does not decide the headline; all three are printed
    regions = []
    for _ in range(3):
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        regions.append(1e3 * (time.perf_counter() - t0) / steps)
    return sorted(regions)[1], regions


def shards_leg(torch, fb, g, steps, warmup):
    """Rows a3 + a4 of the decode step as one call over the 4 shards (after the step has left K', V' in place)."""
    cfg = g["cfg"]
    need = fb.fedrag_partial_attn_shards_workspace_bytes(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head,
                                                         g["Qs"].dtype, cfg.L_q, [cfg.L_kv] * cfg.n_shards)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=g["Qs"].device)
    O, lse = torch.empty_like(g["O"]), torch.empty_like(g["lse"])
    call = lambda: fb.fedrag_partial_attn_shards(g["Qs"], g["Ks"], g["Vs"], None, O=O, lse=lse, workspace=ws)
    t = measure(torch, call, max(steps, MIN_ITERS), warmup)
    us = t["med_us"]
    nb = cfg.n_shards * g["bytes"]["partial_attn"]
    # the aggregation adds the partials in another order than per shard + across shards: equal to rounding
    err = float((O - g["O"]).abs().max())
    return {"call": "partial_attn_shards (4 shards + aggregation)", "med_us": round(us, 2),
            "avg_us": round(t["avg_us"], 2), "iters": t["iters"], "bytes": nb,
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
    t = measure(torch, call, max(steps, MIN_ITERS), warmup)
    gbs = g["bytes"]["scramble_kv"] / (t["med_us"] * 1e-6) / 1e9
    return {"call": "scramble_kv_structured", "med_us": round(t["med_us"], 2), "avg_us": round(t["avg_us"], 2),
            "iters": t["iters"], "bytes": g["bytes"]["scramble_kv"], "GB/s": round(gbs, 1),
            "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}


def local_attn_leg(torch, W, fb, dev, steps, warmup):
    """The Inquirer's own part of a segment's attention: plaintext tokens attending to themselves and their
    predecessors, Llama-3-8B head shape, segments of 2048 and 4096 tokens.  Counted flops: 4 d Hq Lq (Lq + 1) / 2
    (visible pairs only).  The kernel feeds the second product two storage-type terms per probability (plaintext V
    keeps its outlier channels), i.e. 1.5 x the matrix work of the counted flops."""
    B, Hq, Hkv, d = 1, 32, 8, 128
    dt = torch.bfloat16
    out = {"workload": "local_attn: B1 Hq32 Hkv8 d128 bf16, whole segment attends to itself (causal), plaintext "
                       "Q, K, V with outlier channels"}
    for L in (2048, 4096):
        mk = lambda H, tid: W.activations(B, H, L, d, seed=W.BASE_SEED + 6, tensor_id=tid, outliers=True,
                                          outlier_id=tid, dtype=dt, device=dev)
        Q, K, V = mk(Hq, W.TID_Q), mk(Hkv, W.TID_K), mk(Hkv, W.TID_V)
        O = torch.empty((B, Hq, L, d), dtype=torch.float32, device=dev)
        lse = torch.empty((B, Hq, L), dtype=torch.float32, device=dev)
        need = fb.fedrag_local_attn_workspace_bytes(B, Hq, Hkv, d, dt, L, L) \
            if hasattr(fb, "fedrag_local_attn_workspace_bytes") else 0
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
        t = measure(torch, lambda: fb.fedrag_local_attn(Q, K, V, None, O_part=O, lse=lse, workspace=ws),
                    max(steps, MIN_ITERS), warmup)
        flop = 4.0 * d * Hq * B * (L * (L + 1) / 2)
        tflops = flop / (t["med_us"] * 1e-6) / 1e12
        out[f"segment_{L}"] = {"flop": flop, "med_us": round(t["med_us"], 2), "avg_us": round(t["avg_us"], 2),
                               "iters": t["iters"], "value": round(tflops, 1), "unit": "TFLOP/s",
                               "frac_mfma": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4)}
    return out


def rerank_leg(torch, W, fb, dev, steps, warmup):
    """Re-ranking shape (Section 7.1: 10 candidate documents): 10 query-document pairs of unequal length, 16 heads of
    64 channels, bidirectional attention of every token of a pair over the pair, padded to 1024 tokens; on 16-bit
    K', V' and on their 4-bit transport codes (Section 7.5 recommends 4 bits for re-ranking)."""
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
    t = measure(torch, call, max(steps, MIN_ITERS), warmup)
    flop = sum(4.0 * n * n * d * H for n in lens)   # real pairs only: n queries x n keys
    out = {"workload": "rerank: 10 pairs of 130..1024 tokens padded to 1024, 16 heads x 64, bf16, bidirectional",
           "flop_valid_pairs": flop, "med_us": round(t["med_us"], 2), "avg_us": round(t["avg_us"], 2),
           "iters": t["iters"], "value": round(flop / (t["med_us"] * 1e-6) / 1e12, 1), "unit": "TFLOP/s"}
    if hasattr(fb, "fedrag_partial_attn_varlen_quantized"):
        for bits in (8, 4):
            Kc, Kp = fb.fedrag_quantize_rows(Ks, bits)
            Vc, Vp = fb.fedrag_quantize_rows(Vs, bits)
            O2, l2 = torch.empty_like(O), torch.empty_like(lse)
            callq = lambda: fb.fedrag_partial_attn_varlen_quantized(Qs, Kc, Kp, Vc, Vp, bits, kv, None, O_part=O2,
                                                                    lse=l2, q_lens=kv)
            tq = measure(torch, callq, max(steps, MIN_ITERS), warmup)
            out[f"on_{bits}bit_codes"] = {"med_us": round(tq["med_us"], 2), "avg_us": round(tq["avg_us"], 2),
                                          "value": round(flop / (tq["med_us"] * 1e-6) / 1e12, 1), "unit": "TFLOP/s"}
    return out


def mixed_leg(torch, W, fb, dev, steps, warmup):
    """70B-shaped mixed batch (64 query heads over 8 KV heads, 8 shards x 8192 tokens, 33 sequences): 32 decoding
    sequences and one 4096-token prefill chunk.  Enc of one shard at this shape (all 33 sequences in one call);
    partial_attn over the 8 shards + lse_merge for each part, shard by shard and as one call, alone and with the two
    parts issued on two streams at once.  Inputs: the seeded generator with outlier channels, scrambled on the GPU."""
    cd, cp = W.CONFIGS["mixed70b_decode"], W.CONFIGS["mixed70b_prefill"]
    dt = W.torch_dtype(cd.dtype)
    S, d, Hkv, L = cd.n_shards, cd.d_head, cd.n_kv_heads, cd.L_kv
    Bd, Bp = cd.batch, cp.batch
    Ball = Bd + Bp
    iters = max(steps, MIN_ITERS)
    keys = W.make_keys(Hkv, d, cp.L_q, L, S, seed=cd.seed, dtype=dt)
    phi_k, phi_v, phi_q = keys.phi_k.to(dev), keys.phi_v.to(dev), keys.phi_q.to(dev)
    act = lambda B, H, n, tid, oid: W.activations(B, H, n, d, seed=cd.seed, tensor_id=tid, outliers=True,
                                                  outlier_id=oid, dtype=dt, device=dev)
    Ks, Vs = [], []
    enc = None
    for s_ in range(S):
        K, V = act(Ball, Hkv, L, W.TID_K + s_, W.TID_K), act(Ball, Hkv, L, W.TID_V + s_, W.TID_V)
        perm = keys.perm_kv[s_].to(dev)
        Ko, Vo = torch.empty_like(K), torch.empty_like(V)
        call = lambda: fb.fedrag_scramble_kv(K, V, phi_k, phi_v, perm, n_q_heads=cd.n_q_heads, K_out=Ko, V_out=Vo)
        if s_ == 0:   # Enc of one shard at this configuration's own shape, timed on its own
            enc = measure(torch, call, iters, warmup)
        else:
            call()
        Ks.append(Ko)
        Vs.append(Vo)
        torch.cuda.synchronize()
        del K, V
    enc_bytes = 8.0 * d * Ball * Hkv * L + 4 * L
    Qd = fb.fedrag_scramble_q(act(Bd, cd.n_q_heads, 1, W.TID_Q, W.TID_Q), phi_q, None)
    Qp = fb.fedrag_scramble_q(act(Bp, cp.n_q_heads, cp.L_q, W.TID_Q + 1, W.TID_Q), phi_q, keys.perm_q.to(dev))

    def part(cfg, Q, lo, hi):
        KV = [(Ks[s_][lo:hi], Vs[s_][lo:hi]) for s_ in range(S)]   # the part's sequences: a contiguous slab
        O = torch.empty((S, cfg.batch, cfg.n_q_heads, cfg.L_q, d), dtype=torch.float32, device=dev)
        lse = torch.empty((S, cfg.batch, cfg.n_q_heads, cfg.L_q), dtype=torch.float32, device=dev)
        Om, lm = torch.empty_like(O[0]), torch.empty_like(lse[0])
        O1, l1 = torch.empty_like(O[0]), torch.empty_like(lse[0])
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
            fb.fedrag_partial_attn_shards(Q, [kv[0] for kv in KV], [kv[1] for kv in KV], None, O=O1, lse=l1,
                                          workspace=ws1)
        diff = lambda: (float((Om - O1).abs().max()), float((lm - l1).abs().max()))
        return run, run_one_call, diff

    (run_d, run_d1, diff_d), (run_p, run_p1, diff_p) = part(cd, Qd, 0, Bd), part(cp, Qp, Bd, Ball)
    s_d, s_p = torch.cuda.Stream(), torch.cuda.Stream()   # default priority, both

    def both():
        cur = torch.cuda.current_stream()
        s_p.wait_stream(cur)
        s_d.wait_stream(cur)
        with torch.cuda.stream(s_p):
            run_p()
        with torch.cuda.stream(s_d):
            run_d()
        cur.wait_stream(s_p)
        cur.wait_stream(s_d)

    t_d, t_p = measure(torch, run_d, iters, warmup), measure(torch, run_p, iters, warmup)
    t_b = measure(torch, both, iters, warmup)
    t_d1, t_p1 = measure(torch, run_d1, iters, warmup), measure(torch, run_p1, iters, warmup)
    torch.cuda.synchronize()
    dd, dp = diff_d(), diff_p()
    byts = 4.0 * d * Bd * Hkv * L * S              # K' + V', 16-bit, read once per KV head
    flop = 4.0 * cp.L_q * L * S * d * cp.n_q_heads * Bp
    ms = lambda t: t["med_us"] / 1e3
    hbm = lambda t: {"ms": round(ms(t), 4), "avg_ms": round(t["avg_us"] / 1e3, 4), "GB/s": round(byts / ms(t) / 1e6, 1),
                     "frac_hbm": round(byts / ms(t) / 1e6 / HBM_PEAK_GBS, 4)}
    mf = lambda t: {"ms": round(ms(t), 4), "avg_ms": round(t["avg_us"] / 1e3, 4),
                    "TFLOP/s": round(flop / ms(t) / 1e9, 1),
                    "frac_mfma": round(flop / ms(t) / 1e9 / MFMA_BF16_PEAK_TFLOPS, 4)}
    return {"workload": "mixed70b: Hq64 Hkv8 d128, 8 shards x 8192 tokens, bf16, 33 sequences: 32 decoding + one "
                        "4096-token prefill chunk; partial_attn x 8 + lse_merge per part; medians of "
                        f"{iters} iterations",
            "scramble_kv_one_shard": {"ms": round(ms(enc), 4), "avg_ms": round(enc["avg_us"] / 1e3, 4),
                                      "bytes": enc_bytes, "GB/s": round(enc_bytes / ms(enc) / 1e6, 1),
                                      "frac_hbm": round(enc_bytes / ms(enc) / 1e6 / HBM_PEAK_GBS, 4)},
            "decode": hbm(t_d), "prefill": mf(t_p), "decode_one_call": hbm(t_d1), "prefill_one_call": mf(t_p1),
            "max_abs_diff_one_call_vs_shard_by_shard": {"decode_O": dd[0], "decode_lse": dd[1],
                                                        "prefill_O": dp[0], "prefill_lse": dp[1]},
            "both_on_two_streams_ms": round(ms(t_b), 4), "sum_ms": round(ms(t_d) + ms(t_p), 4),
            "max_ms": round(max(ms(t_d), ms(t_p)), 4)}


def request_leg(torch, W, fb, dev, steps, warmup, n_layers=32):
    """The attention path of one request at the largest length configuration of Section 7.1 (context 4096 + 4096 on
    two Context Owners, 128-token query segment), Llama-3-8B-shaped (32 layers, 32/8 heads of 128), batch 1:
    per layer scramble_q -> attention on the two shards and their aggregation -> the Inquirer's own causal attention
    -> Dec and the aggregation of the two.  Once for the 128-token segment (prefill) and once for one decoded token
    (the segment's 128 + 64 generated tokens local), each as one HIP graph of all layers; with the fused calls
    (partial_attn_shards, unscramble_merge: 4 calls per layer) and call by call (8 calls per layer)."""
    B, Hq, Hkv, d, S, Lc, Lseg, Lgen = 1, 32, 8, 128, 2, 4096, 128, 64
    dt = torch.bfloat16
    tid = [1000]

    def rnd(b, h, n, dd, kind=W.TID_K):   # plaintext from the seeded generator, outlier channels fixed per tensor kind
        tid[0] += 1
        return W.activations(b, h, n, dd, seed=W.BASE_SEED + 9, tensor_id=tid[0], outliers=True, outlier_id=kind,
                             dtype=dt, device=dev)
    keys = W.make_keys(Hkv, d, Lseg, Lc, S, seed=W.BASE_SEED + 9, dtype=dt)
    phi_q, phi_vi = keys.phi_q.to(dev), keys.phi_v_inv.to(dev)
    phi_k, phi_v = keys.phi_k.to(dev), keys.phi_v.to(dev)
    perms = [p_.to(dev) for p_ in keys.perm_kv]
    # per layer: the scrambled caches the Compute Node holds (distinct memory per layer, 1 GiB in all)
    Ks, Vs = [], []
    for _ in range(n_layers):
        enc = [fb.fedrag_scramble_kv(rnd(B, Hkv, Lc, d, W.TID_K), rnd(B, Hkv, Lc, d, W.TID_V), phi_k, phi_v, perms[s_],
                                     n_q_heads=Hq) for s_ in range(S)]
        Ks.append([e[0] for e in enc])
        Vs.append([e[1] for e in enc])

    def chain(Lq, L_local, fused):
        Q = rnd(B, Hq, Lq, d, W.TID_Q)
        Kl = [rnd(B, Hkv, L_local, d, W.TID_K) for _ in range(n_layers)]   # the Inquirer's own plaintext K, V per layer
        Vl = [rnd(B, Hkv, L_local, d, W.TID_V) for _ in range(n_layers)]
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
        steps = max(steps, MIN_ITERS)
        eager_ms = measure(torch, run, steps, warmup)["med_us"] / 1e3
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
        graph_ms = measure(torch, graph.replay, steps, 1)["med_us"] / 1e3
        res[name] = {"eager_ms": round(eager_ms, 4), "graph_ms": round(graph_ms, 4),
                     "graph_us_per_layer": round(1e3 * graph_ms / n_layers, 2), "replay_equals_eager": same}
    res["decode_token"]["tokens_per_s_attention_path"] = round(1e3 / res["decode_token"]["graph_ms"], 1)
    return res


def long_decode_leg(torch, W, fb, dev, steps, warmup):
    """Long-context decode (B64, 32/8 heads, d128, 8 shards x 32768 tokens, bf16): Enc of one shard at this size, then
    rows a3 + a4 with all 64 GiB of K', V' resident, as one call over the 8 shards and shard by shard.  Inputs: the
    seeded generator with outlier channels, scrambled on the GPU shard by shard."""
    cfg = W.CONFIGS["long_decode"]
    dt = W.torch_dtype(cfg.dtype)
    B, Hq, Hkv, d, S, L = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.d_head, cfg.n_shards, cfg.L_kv
    iters = max(steps, MIN_ITERS)
    keys = W.make_keys(Hkv, d, 1, L, S, seed=cfg.seed, dtype=dt)
    phi_k, phi_v = keys.phi_k.to(dev), keys.phi_v.to(dev)
    act = lambda H, n, tid, oid: W.activations(B, H, n, d, seed=cfg.seed, tensor_id=tid, outliers=True,
                                               outlier_id=oid, dtype=dt, device=dev)
    out = {"workload": "long_decode: B64 Hq32 Hkv8 d128 Lq1, 8 shards x 32768 tokens, bf16 (64 GiB of K', V'); "
                       f"medians of {iters} iterations"}
    Ks, Vs = [], []
    for s_ in range(S):
        K, V = act(Hkv, L, W.TID_K + s_, W.TID_K), act(Hkv, L, W.TID_V + s_, W.TID_V)
        perm = keys.perm_kv[s_].to(dev)
        Ko, Vo = torch.empty_like(K), torch.empty_like(V)
        enc = lambda: fb.fedrag_scramble_kv(K, V, phi_k, phi_v, perm, n_q_heads=Hq, K_out=Ko, V_out=Vo)
        if s_ == 0:   # Enc of one shard at this size (8 GiB read, 8 GiB written)
            t = measure(torch, enc, iters, 2)
            enc_bytes = 8.0 * d * B * Hkv * L + 4 * L
            ms = t["med_us"] / 1e3
            out["scramble_kv_one_shard"] = {"ms": round(ms, 3), "avg_ms": round(t["avg_us"] / 1e3, 3),
                                            "GB/s": round(enc_bytes / ms / 1e6, 1),
                                            "frac_hbm": round(enc_bytes / ms / 1e6 / HBM_PEAK_GBS, 4)}
        else:
            enc()
        Ks.append(Ko)
        Vs.append(Vo)
        torch.cuda.synchronize()
        del K, V
    Q = fb.fedrag_scramble_q(act(Hq, 1, W.TID_Q, W.TID_Q), keys.phi_q.to(dev), None)
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
    O, lse, O2, lse2 = f32(B, Hq, 1, d), f32(B, Hq, 1), f32(B, Hq, 1, d), f32(B, Hq, 1)
    Op, lp = f32(S, B, Hq, 1, d), f32(S, B, Hq, 1)
    need = fb.fedrag_partial_attn_shards_workspace_bytes(B, Hq, Hkv, d, dt, 1, [L] * S)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)
    need1 = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dt, 1, L)
    ws1 = torch.empty(max(need1, 16), dtype=torch.uint8, device=dev)

    def one_call():
        fb.fedrag_partial_attn_shards(Q, Ks, Vs, None, O=O, lse=lse, workspace=ws)

    def per_shard():
        for s_ in range(S):
            fb.fedrag_partial_attn(Q, Ks[s_], Vs[s_], None, O_part=Op[s_], lse=lp[s_], workspace=ws1)
        fb.fedrag_lse_merge(Op, lp, n_kv_heads=Hkv, O_out=O2, lse_out=lse2)

    byts = 4.0 * d * B * Hkv * L * S
    for name, fn in (("one_call", one_call), ("shard_by_shard", per_shard)):
        t = measure(torch, fn, iters, max(1, warmup // 2))
        ms = t["med_us"] / 1e3
        out[name] = {"ms": round(ms, 3), "avg_ms": round(t["avg_us"] / 1e3, 3), "GB/s": round(byts / ms / 1e6, 1),
                     "frac_hbm": round(byts / ms / 1e6 / HBM_PEAK_GBS, 4)}
    torch.cuda.synchronize()
    out["max_abs_diff_one_call_vs_shard_by_shard"] = {"O": float((O - O2).abs().max()),
                                                      "lse": float((lse - lse2).abs().max())}
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
        steps = max(steps, MIN_ITERS)
        tq, tdq = measure(torch, q, steps, warmup), measure(torch, dq, steps, warmup)
        nbytes = n * (d * 2 + d * bits // 8 + 8)
        out[f"{bits}bit"] = {"quantize_us": round(tq["med_us"], 2), "dequantize_us": round(tdq["med_us"], 2),
                             "bytes": nbytes, "quantize_GB/s": round(nbytes / tq["med_us"] / 1e3, 1),
                             "dequantize_GB/s": round(nbytes / tdq["med_us"] / 1e3, 1)}
    # Enc with the codec as its epilogue (what a Context Owner sends): one shard, K and V
    cfg = g["cfg"]
    outs = fb.fedrag_scramble_kv_quantized(g["K"][0], g["V"][0], g["phi_k"], g["phi_v"], g["perm_kv"][0], 8,
                                           n_q_heads=cfg.n_q_heads)
    call = lambda: fb.fedrag_scramble_kv_quantized(g["K"][0], g["V"][0], g["phi_k"], g["phi_v"], g["perm_kv"][0], 8,
                                                   n_q_heads=cfg.n_q_heads, out=outs)
    us = measure(torch, call, steps, warmup)["med_us"]
    nb = 2 * n * (d * 2 + d + 8) + 4 * cfg.L_kv
    out["scramble_kv_quantized_8bit"] = {"med_us": round(us, 2), "bytes": nb, "GB/s": round(nb / us / 1e3, 1)}
    # the Compute Node's decode call reading the codes directly (one shard)
    for bits in (8, 4):
        Kc, Kp, Vc, Vp = fb.fedrag_scramble_kv_quantized(g["K"][0], g["V"][0], g["phi_k"], g["phi_v"], g["perm_kv"][0],
                                                         bits, n_q_heads=cfg.n_q_heads)
        call = lambda: fb.fedrag_partial_attn_quantized(g["Qs"], Kc, Kp, Vc, Vp, bits, None, O_part=g["O_parts"][0],
                                                        lse=g["lses"][0], workspace=g["ws"])
        us = measure(torch, call, steps, warmup)["med_us"]
        nb = 2 * n * (d * bits // 8 + 8)
        out[f"partial_attn_quantized_{bits}bit"] = {"med_us": round(us, 2), "bytes_read": nb,
                                                    "GB/s": round(nb / us / 1e3, 1)}
    return out


def prefill_leg(torch, W, fb, dev, steps, warmup, keep=None):
    """RAG prefill: partial_attn alone, 2048 queries x 16384 keys, 32/8 heads, d 128, bf16.  `keep`, a dict, receives
    host copies of Q', K', V' for the oracle's timing leg."""
    cfg = W.CONFIGS["rag_prefill"]
    dt = W.torch_dtype(cfg.dtype)
    mk = lambda H, L, tid, oid: W.activations(cfg.batch, H, L, cfg.d_head, seed=cfg.seed, tensor_id=tid, outliers=True,
                                              outlier_id=oid, dtype=dt, device=dev)
    Q, K, V = mk(cfg.n_q_heads, cfg.L_q, W.TID_Q, W.TID_Q), mk(cfg.n_kv_heads, cfg.L_kv, W.TID_K, W.TID_K), \
        mk(cfg.n_kv_heads, cfg.L_kv, W.TID_V, W.TID_V)
    keys = W.make_keys(cfg.n_kv_heads, cfg.d_head, cfg.L_q, cfg.L_kv, 1, seed=cfg.seed, dtype=dt)
    Qs = fb.fedrag_scramble_q(Q, keys.phi_q.to(dev), keys.perm_q.to(dev))
    Ks, Vs = fb.fedrag_scramble_kv(K, V, keys.phi_k.to(dev), keys.phi_v.to(dev), keys.perm_kv[0].to(dev))
    if keep is not None:
        keep.update(Qs=Qs.cpu(), Ks=Ks.cpu(), Vs=Vs.cpu())
    O = torch.empty((cfg.batch, cfg.n_q_heads, cfg.L_q, cfg.d_head), dtype=torch.float32, device=dev)
    lse = torch.empty((cfg.batch, cfg.n_q_heads, cfg.L_q), dtype=torch.float32, device=dev)
    iters = max(steps, MIN_ITERS)
    t = measure(torch, lambda: fb.fedrag_partial_attn(Qs, Ks, Vs, None, O_part=O, lse=lse), iters, warmup)
    # the Inquirer's two calls around it at this size (a2 before, a5 after)
    phi_q, perm_q, phi_vi = keys.phi_q.to(dev), keys.perm_q.to(dev), keys.phi_v_inv.to(dev)
    out = torch.empty_like(O)
    Q2 = torch.empty_like(Qs)
    around = {"scramble_q": round(measure(torch, lambda: fb.fedrag_scramble_q(Q, phi_q, perm_q, Q_out=Q2), iters, 2)["med_us"], 2),
              "unscramble": round(measure(torch, lambda: fb.fedrag_unscramble(O, phi_vi, perm_q, O_out=out), iters, 2)["med_us"], 2)}
    flop = 4.0 * cfg.L_q * cfg.L_kv * cfg.d_head * cfg.n_q_heads * cfg.batch
    tflops = flop / (t["avg_us"] * 1e-6) / 1e12
    return {"workload": "rag_prefill: B1 Hq32 Hkv8 d128 Lq2048 Lkv16384 bf16, non-causal", "flop": flop,
            "avg_us": round(t["avg_us"], 2), "med_us": round(t["med_us"], 2), "iters": iters,
            "value": round(tflops, 1), "unit": "TFLOP/s",
            "inquirer_calls_med_us": around,
            "roofline": {"bound": "mfma", "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                         "kernel": "prefill_attn_kernel<BF16,128,false>", "avg_us": round(t["avg_us"], 2),
                         "flop_per_launch": flop}}


def achievable_leg(torch, dev):
    """What plain kernels reach on this device in this run, beside the published peaks the fractions are quoted
    against: a streaming copy and a streaming read of 1 GiB (beyond the 256 MB last-level cache) and a bare bf16 MFMA
    issue loop.  The kernels live in libfedrag_probes.so (csrc/probes/rate_probes.hip)."""
    import ctypes
    from paper_2605_25716_amd import build as fbuild
    if not os.path.exists(fbuild.PROBES_LIB):
        fbuild.build_probes(force=True)
    lib = ctypes.CDLL(fbuild.PROBES_LIB)
    vp = ctypes.c_void_p
    lib.fedrag_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.fedrag_probe_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
    lib.fedrag_probe_mfma_bf16.argtypes = [vp, ctypes.c_int, vp]
    lib.fedrag_probe_mfma_bf16_random.argtypes = [vp, ctypes.c_int, vp]
    lib.fedrag_probe_mfma_bf16_flop.argtypes = [ctypes.c_int]
    lib.fedrag_probe_mfma_bf16_flop.restype = ctypes.c_double
    n = 1 << 30
    gen = torch.Generator(device=dev)
    gen.manual_seed(0xFED2A6)
    a = torch.randint(0, 256, (n,), dtype=torch.uint8, device=dev, generator=gen)  # bytes that toggle, as real data do
    b = torch.empty_like(a)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    stream = lambda: vp(torch.cuda.current_stream().cuda_stream)

    def chk(rc):
        if rc != 0:
            raise RuntimeError(f"probe launch failed ({rc})")
    tc = measure(torch, lambda: chk(lib.fedrag_probe_copy(b.data_ptr(), a.data_ptr(), n, stream())), MIN_ITERS, 3)
    tr = measure(torch, lambda: chk(lib.fedrag_probe_read(a.data_ptr(), n, sink.data_ptr(), stream())), MIN_ITERS, 3)
    iters = 4096
    tm = measure(torch, lambda: chk(lib.fedrag_probe_mfma_bf16(sink.data_ptr(), iters, stream())), MIN_ITERS, 3)
    tmr = measure(torch, lambda: chk(lib.fedrag_probe_mfma_bf16_random(sink.data_ptr(), iters, stream())), MIN_ITERS, 3)
    flop = float(lib.fedrag_probe_mfma_bf16_flop(iters))
    ok = bool(torch.equal(a, b))
    del a, b
    return {"copy_GB/s": round(2.0 * n / tc["med_us"] / 1e3, 1), "copy_frac_of_hbm_peak": round(2.0 * n / tc["med_us"] / 1e3 / HBM_PEAK_GBS, 4),
            "read_GB/s": round(1.0 * n / tr["med_us"] / 1e3, 1), "read_frac_of_hbm_peak": round(1.0 * n / tr["med_us"] / 1e3 / HBM_PEAK_GBS, 4),
            "mfma_bf16_TFLOP/s": round(flop / tm["med_us"] / 1e6, 1),
            "mfma_frac_of_peak": round(flop / tm["med_us"] / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
            "mfma_bf16_random_operands_TFLOP/s": round(flop / tmr["med_us"] / 1e6, 1),
            "mfma_random_operands_frac_of_peak": round(flop / tmr["med_us"] / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
            "copy_verified": ok,
            "what": "medians of 20 launches: 1 GiB device copy of random bytes (read + write bytes) and 1 GiB streaming "
                    "read, one 256-thread workgroup per compute unit; 256 workgroups x 8 waves x 4096 x 8 independent "
                    "32x32x16 bf16 MFMAs on register operands, first with the same two smooth operands for every MFMA, "
                    "then with hashed bell-shaped operands per accumulator (the chip clocks lower when operand bits toggle)"}


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


def cpu_other_configs(torch, W, kept):
    """The oracle (partial attention per shard + aggregation, fp64, its own thread pool) on the other configurations:
    the RAG prefill in full; the long-context decode and the two parts of the 70B-shaped batch on a seeded sample of
    (sequence, KV head) units of every shard, scaled linearly to the whole configuration (the work per unit is
    uniform) and marked as extrapolated."""
    import numpy as np
    import oracle
    out = {}
    if kept:   # configuration 3, whole: the same Q', K', V' bits the GPU leg consumed
        cfg = W.CONFIGS["rag_prefill"]
        t0 = time.perf_counter()
        oracle.partial_attn(kept["Qs"], kept["Ks"], kept["Vs"])
        dt = time.perf_counter() - t0
        flop = 4.0 * cfg.L_q * cfg.L_kv * cfg.d_head * cfg.n_q_heads * cfg.batch
        out["rag_prefill"] = {"value": round(flop / dt / 1e12, 5), "unit": "TFLOP/s", "seconds": round(dt, 3),
                              "extrapolated": False, "sample": "the whole configuration (2048 x 16384, 32 heads)"}

    def sampled(cfg, n_units, q_rows):
        dt_ = W.torch_dtype(cfg.dtype)
        G, S, d = cfg.group, cfg.n_shards, cfg.d_head
        act = lambda H, n, tid: W.activations(n_units, H, n, d, seed=cfg.seed + 77, tensor_id=tid, outliers=False, dtype=dt_)
        Q = act(G, q_rows, W.TID_Q)                      # the sampled units as a batch of single-KV-head sequences
        KV = [(act(1, cfg.L_kv, W.TID_K + s_), act(1, cfg.L_kv, W.TID_V + s_)) for s_ in range(S)]
        t0 = time.perf_counter()
        parts = [oracle.partial_attn(Q, k, v) for k, v in KV]
        oracle.lse_merge(np.stack([p_[0] for p_ in parts]), np.stack([p_[1] for p_ in parts]))
        return time.perf_counter() - t0

    cfg = W.CONFIGS["long_decode"]
    n = 8
    dt = sampled(cfg, n, 1)
    scale = cfg.batch * cfg.n_kv_heads / n
    byts = 4.0 * cfg.d_head * cfg.batch * cfg.n_kv_heads * cfg.L_kv * cfg.n_shards
    out["long_decode"] = {"value": round(byts / (dt * scale) / 1e9, 4), "unit": "GB/s", "seconds": round(dt, 3),
                          "extrapolated": True, "seconds_whole_configuration": round(dt * scale, 1),
                          "sample": f"{n} of {cfg.batch * cfg.n_kv_heads} (sequence, KV head) units of each of the "
                                    f"{cfg.n_shards} shards, scaled by {scale:g}"}
    cfg = W.CONFIGS["mixed70b_decode"]
    dt = sampled(cfg, n, 1)
    scale = cfg.batch * cfg.n_kv_heads / n
    byts = 4.0 * cfg.d_head * cfg.batch * cfg.n_kv_heads * cfg.L_kv * cfg.n_shards
    out["mixed70b_decode"] = {"value": round(byts / (dt * scale) / 1e9, 4), "unit": "GB/s", "seconds": round(dt, 3),
                              "extrapolated": True, "seconds_whole_configuration": round(dt * scale, 1),
                              "sample": f"{n} of {cfg.batch * cfg.n_kv_heads} units of each of the {cfg.n_shards} "
                                        f"shards, scaled by {scale:g}"}
    cfg = W.CONFIGS["mixed70b_prefill"]
    rows = 32
    dt = sampled(cfg, cfg.n_kv_heads, rows)
    scale = cfg.L_q / rows
    flop = 4.0 * cfg.L_q * cfg.L_kv * cfg.n_shards * cfg.d_head * cfg.n_q_heads * cfg.batch
    out["mixed70b_prefill"] = {"value": round(flop / (dt * scale) / 1e12, 5), "unit": "TFLOP/s", "seconds": round(dt, 3),
                               "extrapolated": True, "seconds_whole_configuration": round(dt * scale, 1),
                               "sample": f"all {cfg.n_kv_heads} KV-head units of each of the {cfg.n_shards} shards, "
                                         f"{rows} of the {cfg.L_q} query rows per head, scaled by {scale:g}"}
    return out


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
        got = graph_leg(torch, fb, g, args.steps)
        if got is not None:
            graph_ms, graph_regions = got

    calls = timer.summary()
    per_call = {}
    for name, t in calls.items():
        gbs = g["bytes"][name] / (t["avg_us"] * 1e-6) / 1e9
        per_call[name] = {"avg_us": round(t["avg_us"], 2), "med_us": round(t["med_us"], 2),
                          "calls_per_step": t["calls"] // args.steps,
                          "bytes": g["bytes"][name], "GB/s": round(gbs, 1), "frac_hbm": round(gbs / HBM_PEAK_GBS, 4)}
        if t["stalls_left_out"]:
            per_call[name]["stalls_left_out"] = t["stalls_left_out"]
            per_call[name]["max_us"] = round(t["max_us"], 2)
    kernel_of = {"scramble_kv": "scramble_rows_kernel<BF16,128,false,0>", "partial_attn": "decode_attn_kernel<BF16,128>"}
    dom = max(kernel_of, key=lambda n: calls[n]["total_ms"])
    def hbm_roofline(name):
        return {"bound": "hbm", "achieved": per_call[name]["GB/s"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(per_call[name]["GB/s"] / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC_BYTES.get(name),
                "traffic_source": f"{TRAFFIC_PROFILE} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this command, scaled "
                                  "by a 1 GiB copy; not re-read in this run)",
                "kernel": kernel_of[name], "call": name, "avg_us": per_call[name]["avg_us"],
                "med_us": per_call[name]["med_us"], "bytes_per_launch": g["bytes"][name]}
    # the kernel with the largest share of the step's time
    roofline = hbm_roofline(dom)
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
        # every kernel a target is stated for: the decode attention kernel (HBM) here, the prefill one (MFMA) is added
        # by the prefill leg below
        "rooflines": {"scramble_kv": hbm_roofline("scramble_kv"), "decode_partial_attn": hbm_roofline("partial_attn")},
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
        line["graph_regions_ms_per_step"] = [round(x, 4) for x in graph_regions]
        line["value"] = round(g["step_bytes"] / (graph_ms * 1e-3) / 1e9, 1)
        line["config"]["launch"] = ("the step recorded once into a HIP graph and replayed K times between "
                                    "synchronisations (outputs checked equal to the eager ones bit for bit), three "
                                    "such regions of K steps, the middle one reported; "
                                    "'eager' = the same K steps launched call by call from Python")
    line["frac_hbm"] = round(line["value"] / HBM_PEAK_GBS, 4)
    all_legs = ("achievable", "shards", "codec", "structured", "rerank", "local_attn", "request", "mixed70b", "prefill",
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

    leg("achievable", lambda: achievable_leg(torch, dev))
    leg("shards", lambda: shards_leg(torch, fb, g, args.steps, args.warmup))
    leg("codec", lambda: codec_leg(torch, fb, g, args.steps, args.warmup))
    leg("structured", lambda: structured_leg(torch, W, fb, g, dev, args.steps, args.warmup))
    leg("rerank", lambda: rerank_leg(torch, W, fb, dev, half, args.warmup))
    leg("local_attn", lambda: local_attn_leg(torch, W, fb, dev, half, args.warmup))
    leg("request", lambda: request_leg(torch, W, fb, dev, half, args.warmup))
    leg("mixed70b", lambda: mixed_leg(torch, W, fb, dev, half, args.warmup))
    kept = {}
    leg("prefill", lambda: prefill_leg(torch, W, fb, dev, half, args.warmup, keep=None if args.no_cpu else kept))
    if isinstance(line.get("prefill"), dict) and "roofline" in line["prefill"]:
        line["rooflines"]["prefill_partial_attn"] = line["prefill"]["roofline"]
    ach = line.get("achievable")
    if isinstance(ach, dict) and "copy_GB/s" in ach:
        # each kernel's rate beside what the plain probe of its kind reached in this run (`frac` stays against the
        # published peak): a copy for the read + write kernel, a read stream for the read-only one, the MFMA issue
        # loop on hashed operands for the contraction
        for key, probe in (("scramble_kv", "copy_GB/s"), ("decode_partial_attn", "read_GB/s"),
                           ("prefill_partial_attn", "mfma_bf16_random_operands_TFLOP/s")):
            r = line["rooflines"].get(key)
            if isinstance(r, dict) and ach.get(probe):
                r["frac_of_probe"] = round(r["achieved"] / ach[probe], 4)
                r["probe"] = f"achievable.{probe}"
        dom_key = {"scramble_kv": "scramble_kv", "partial_attn": "decode_partial_attn"}.get(line["roofline"]["call"])
        if dom_key:
            line["roofline"] = dict(line["rooflines"][dom_key])
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_leg(torch, W, g, args.cpu_shards)
        try:
            line["cpu_baseline"]["other_configs"] = cpu_other_configs(torch, W, kept)
        except Exception as e:  # noqa: BLE001 - the headline baseline above is already measured
            line["cpu_baseline"]["other_configs"] = {"error": f"{type(e).__name__}: {e}"}
    kept.clear()
    if "long_decode" in want:   # last: it takes 64 GiB of device memory
        del g
        torch.cuda.empty_cache()
        leg("long_decode", lambda: long_decode_leg(torch, W, fb, dev, half, args.warmup))
    print(json.dumps(line))


if __name__ == "__main__":
    main()
