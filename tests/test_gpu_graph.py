"""The decode chain enqueues only kernels on the caller's stream (no allocation, no host synchronisation, no memset
nodes), so a caller can record it into a HIP graph.  Replays are checked against the eager result, several times, with
eager work and synchronisations between them."""
import pytest
import torch

from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def chain(g):
    fb.fedrag_scramble_q(g["Q"], g["phi_q"], None, Q_out=g["Qs"])
    for s in range(g["S"]):
        fb.fedrag_scramble_kv(g["K"][s], g["V"][s], g["phi_k"], g["phi_v"], g["perm"][s], n_q_heads=g["Hq"],
                              K_out=g["Ks"], V_out=g["Vs"])
        fb.fedrag_partial_attn(g["Qs"], g["Ks"], g["Vs"], None, O_part=g["parts"][s], lse=g["lses"][s],
                               workspace=g["ws"])
    fb.fedrag_lse_merge(g["parts"], g["lses"], n_kv_heads=g["Hkv"], O_out=g["O"], lse_out=g["lse"])
    fb.fedrag_unscramble(g["O"], g["phi_v_inv"], None, O_out=g["out"])


def make(seed):
    B, Hq, Hkv, d, Lq, L, S = 3, 8, 2, 128, 1, 4096 + 37, 3
    dt = torch.bfloat16
    keys = W.make_keys(Hkv, d, Lq, L, S, seed=seed, dtype=dt)
    g = {"S": S, "Hq": Hq, "Hkv": Hkv}
    g["Q"] = W.activations(B, Hq, Lq, d, seed=seed, tensor_id=W.TID_Q, outliers=True, dtype=dt, device=DEV)
    g["K"] = [W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_K + s, outliers=True, outlier_id=W.TID_K, dtype=dt,
                            device=DEV) for s in range(S)]
    g["V"] = [W.activations(B, Hkv, L, d, seed=seed, tensor_id=W.TID_V + s, outliers=True, outlier_id=W.TID_V, dtype=dt,
                            device=DEV) for s in range(S)]
    for k in ("phi_q", "phi_k", "phi_v", "phi_v_inv"):
        g[k] = getattr(keys, k).to(DEV)
    g["perm"] = [p.to(DEV) for p in keys.perm_kv]
    g["Qs"] = torch.empty_like(g["Q"])
    g["Ks"] = torch.empty_like(g["K"][0])
    g["Vs"] = torch.empty_like(g["V"][0])
    g["parts"] = torch.empty((S, B, Hq, Lq, d), dtype=torch.float32, device=DEV)
    g["lses"] = torch.empty((S, B, Hq, Lq), dtype=torch.float32, device=DEV)
    g["O"] = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=DEV)
    g["lse"] = torch.empty((B, Hq, Lq), dtype=torch.float32, device=DEV)
    g["out"] = torch.empty((B, Hq, Lq, d), dtype=torch.float32, device=DEV)
    ws = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dt, Lq, L)
    g["ws"] = torch.empty(max(ws, 16), dtype=torch.uint8, device=DEV)
    return g


def test_decode_chain_replays_from_a_hip_graph():
    g = make(seed=4242)
    chain(g)                     # eager: also warms up everything the first call of a kernel sets up
    torch.cuda.synchronize()
    ref_out, ref_lse = g["out"].clone(), g["lse"].clone()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            chain(g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(4):
        # eager work of the program's own between replays: overwrite every intermediate and output
        for k in ("Qs", "Ks", "Vs", "parts", "lses", "O", "lse", "out"):
            g[k].fill_(float(rep + 1))
        g["ws"].fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g["out"], ref_out), f"replay {rep}: output differs from the eager result"
        assert torch.equal(g["lse"], ref_lse), f"replay {rep}: lse differs from the eager result"


def fused_chain(g):
    """scramble_q -> attention over all shards with their aggregation -> the Inquirer's own attention -> Dec and the
    aggregation of the two, for a 70-token segment (prefill kernel with key runs, fp32 matrix-core Dec)."""
    fb.fedrag_scramble_q(g["Q"], g["phi_q"], g["perm_q"], Q_out=g["Qs"])
    fb.fedrag_partial_attn_shards(g["Qs"], g["Ksl"], g["Vsl"], None, O=g["O"], lse=g["lse"], workspace=g["ws"])
    fb.fedrag_local_attn(g["Q"], g["Kl"], g["Vl"], None, O_part=g["Ol"], lse=g["ll"])
    fb.fedrag_unscramble_merge(g["O"], g["lse"], g["phi_v_inv"], g["perm_q"], g["Ol"], g["ll"], O_out=g["out"],
                               lse_out=g["out_l"], n_kv_heads=g["Hkv"])


def test_fused_segment_chain_replays_from_a_hip_graph():
    B, Hq, Hkv, d, Lq, Ls = 1, 8, 2, 128, 70, [1500, 700, 64]
    dt = torch.bfloat16
    keys = W.make_keys(Hkv, d, Lq, max(Ls), len(Ls), seed=777, dtype=dt, permute_q=True)
    mk = lambda H, L, tid: W.activations(B, H, L, d, seed=777, tensor_id=tid, outliers=False, dtype=dt, device=DEV)
    g = {"Hkv": Hkv, "Q": mk(Hq, Lq, W.TID_Q), "Kl": mk(Hkv, Lq, 50), "Vl": mk(Hkv, Lq, 51),
         "Ksl": [mk(Hkv, L, W.TID_K + i) for i, L in enumerate(Ls)],
         "Vsl": [mk(Hkv, L, W.TID_V + i) for i, L in enumerate(Ls)],
         "phi_q": keys.phi_q.to(DEV), "phi_v_inv": keys.phi_v_inv.to(DEV), "perm_q": keys.perm_q.to(DEV)}
    f32 = lambda *s: torch.empty(s, dtype=torch.float32, device=DEV)
    g["Qs"] = torch.empty_like(g["Q"])
    g["O"], g["lse"], g["Ol"], g["ll"] = f32(B, Hq, Lq, d), f32(B, Hq, Lq), f32(B, Hq, Lq, d), f32(B, Hq, Lq)
    g["out"], g["out_l"] = f32(B, Hq, Lq, d), f32(B, Hq, Lq)
    need = fb.fedrag_partial_attn_shards_workspace_bytes(B, Hq, Hkv, d, dt, Lq, Ls)
    assert need > 0
    g["ws"] = torch.empty(need, dtype=torch.uint8, device=DEV)
    fused_chain(g)
    torch.cuda.synchronize()
    ref_out, ref_lse = g["out"].clone(), g["out_l"].clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fused_chain(g)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        for k in ("Qs", "O", "lse", "Ol", "ll", "out", "out_l"):
            g[k].fill_(float(rep + 1))
        g["ws"].fill_(rep + 1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(g["out"], ref_out) and torch.equal(g["out_l"], ref_lse), f"replay {rep} differs"
