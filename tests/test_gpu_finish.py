"""GPU parity of fedrag_unscramble_merge: Dec of the remote result plus the aggregation with the Inquirer's own
partial (Sections 4.2 and 4.1) against the oracle's stages, and bit for bit against the three separate calls."""
import numpy as np
import pytest
import torch

import parity as PT
from paper_2605_25716_amd import binding as fb
from paper_2605_25716_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("B,Hq,Hkv,d,Lq,permute", [(2, 8, 2, 128, 1, False), (1, 4, 2, 128, 77, True),
                                                   (2, 4, 4, 64, 40, True), (1, 32, 8, 128, 128, True)])
def test_unscramble_merge(oracle, B, Hq, Hkv, d, Lq, permute):
    keys = W.make_keys(Hkv, d, Lq, 64, 1, seed=4242 + Lq, dtype=torch.float32, permute_q=permute)
    g = torch.Generator().manual_seed(99 + Lq)
    O_scr = torch.randn((B, Hq, Lq, d), generator=g)
    O_loc = torch.randn((B, Hq, Lq, d), generator=g)
    l_scr = 3.0 * torch.randn((B, Hq, Lq), generator=g)
    l_loc = 3.0 * torch.randn((B, Hq, Lq), generator=g)
    # degenerate rows: no remote keys, no local keys, neither (their outputs are never read: poison them)
    flat_s, flat_l = l_scr.view(-1), l_loc.view(-1)
    n = flat_s.numel()
    if n >= 4:
        flat_s[0] = -np.inf
        O_scr.view(-1, d)[0] = float("nan")
        flat_l[1] = -np.inf
        O_loc.view(-1, d)[1] = float("nan")
    perm = keys.perm_q
    if n >= 4 and perm is None:
        flat_s[2] = -np.inf
        flat_l[2] = -np.inf
    dv = lambda t: None if t is None else t.to(DEV)
    O, lse = fb.fedrag_unscramble_merge(dv(O_scr), dv(l_scr), dv(keys.phi_v_inv), dv(perm), dv(O_loc), dv(l_loc))
    # the three calls
    O1 = fb.fedrag_unscramble(dv(O_scr), dv(keys.phi_v_inv), dv(perm))
    l1 = fb.fedrag_unpermute_lse(dv(l_scr), dv(perm))
    O3, l3 = fb.fedrag_lse_merge(torch.stack([O1, dv(O_loc)]), torch.stack([l1, dv(l_loc)]), n_kv_heads=Hkv)
    torch.cuda.synchronize()
    assert torch.equal(torch.nan_to_num(O, nan=7.0), torch.nan_to_num(O3, nan=7.0)) and torch.equal(lse, l3)
    # the oracle's stages on the same inputs (poisoned rows replaced: the oracle multiplies before it weighs)
    Os = torch.nan_to_num(O_scr, nan=0.0)
    Ol = torch.nan_to_num(O_loc, nan=0.0)
    Ou = oracle.unscramble(Os, keys.phi_v_inv, perm)
    lu = np.empty((B, Hq, Lq))
    p = np.arange(Lq) if perm is None else perm.numpy()
    lu[:, :, p] = l_scr.double().numpy()
    Or, lr = oracle.lse_merge(np.stack([Ou, Ol.double().numpy()]), np.stack([lu, l_loc.double().numpy()]))
    assert PT.rel_normwise(O, Or) <= PT.TOL_F32_REL
    assert PT.rel_normwise(lse, lr) <= PT.TOL_F32_REL
