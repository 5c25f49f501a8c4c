"""fedrag_partial_attn_static (the entry point that allocates nothing: its key-run partials live in the library's
static device array) against fedrag_partial_attn, through the C ABI: two calls in a row, the second on a smaller
input, so that the second finds the first call's contents in the shared array."""
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _inputs(B, Hq, Hkv, d, Lq, L, dtype, seed):
    mk = lambda H, n, tid: W.activations(B, H, n, d, seed=seed, tensor_id=tid, outliers=True, dtype=dtype).to(DEV)
    return mk(Hq, Lq, W.TID_Q), mk(Hkv, L, W.TID_K), mk(Hkv, L, W.TID_V)


# (first call, second smaller call); every one of them is cut into key runs, i.e. uses the scratch array
PAIRS = [
    ("decode", (2, 8, 2, 128, 1, 6000), (1, 8, 2, 128, 1, 1500)),
    ("decode_rows16_d64", (1, 8, 2, 64, 4, 3000), (1, 8, 2, 64, 2, 700)),
    ("prefill_runs", (1, 4, 2, 128, 70, 2500), (1, 4, 2, 128, 33, 600)),
]


@pytest.mark.parametrize("pair", PAIRS, ids=[p[0] for p in PAIRS])
def test_static_scratch_equals_workspace_call(oracle, pair):
    name, first, second = pair
    dtype = torch.bfloat16
    for i, (B, Hq, Hkv, d, Lq, L) in enumerate((first, second)):
        need = fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dtype, Lq, L)
        assert 0 < need <= fb.STATIC_SCRATCH_BYTES, "the case must use the scratch array and fit into it"
        Q, K, V = _inputs(B, Hq, Hkv, d, Lq, L, dtype, seed=100 + i)
        O_ref, l_ref = fb.fedrag_partial_attn(Q, K, V)
        O = torch.full((B, Hq, Lq, d), 7.0, dtype=torch.float32, device=DEV)
        lse = torch.full((B, Hq, Lq), 7.0, dtype=torch.float32, device=DEV)
        before = torch.cuda.memory_allocated()
        fb.fedrag_partial_attn_static(Q, K, V, O, lse)
        assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        # same kernels, same plan, same order of operations: bit for bit
        assert torch.equal(O, O_ref) and torch.equal(lse, l_ref), f"{name} call {i}"
        # and both to the oracle's bound
        Or, lr = oracle.partial_attn(Q.cpu(), K.cpu(), V.cpu())
        PT.check_attn(O, lse, Or, lr, dtype, f"{name} call {i}")


def test_static_scratch_refuses_what_does_not_fit():
    dtype = torch.bfloat16
    B, Hq, Hkv, d, Lq, L = 1, 32, 8, 128, 128, 8192   # a 128-token segment: 16 runs of 4096 rows, about 34 MB
    assert fb.fedrag_partial_attn_workspace_bytes(B, Hq, Hkv, d, dtype, Lq, L) > fb.STATIC_SCRATCH_BYTES
    Q = torch.zeros((B, Hq, Lq, d), dtype=dtype, device=DEV)
    K = torch.zeros((B, Hkv, L, d), dtype=dtype, device=DEV)
    O = torch.full((B, Hq, Lq, d), 7.0, dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq, Lq), 7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(fb.FedragError) as e:
        fb.fedrag_partial_attn_static(Q, K, K, O, lse)
    assert e.value.status == fb.ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((O == 7.0).all()) and bool((lse == 7.0).all())  # nothing was launched
