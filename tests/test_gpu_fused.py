"""GPU parity of the fused on-the-fly-weights path (trigram context, shared-embedding weight
function) against the float64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2304_13134_amd import binding as lb
from paper_2304_13134_amd import workloads
from gpu_util import announce, assert_dist_close

pytestmark = pytest.mark.gpu


def dev_bf16(bits):
    return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)


def fused_inputs(s):
    return lb.SharedEmb(dev_bf16(s["f"]), dev_bf16(s["e"]), dev_bf16(s["W"]))


@pytest.mark.parametrize("B,T,V,H,seed", [(1, 4, 2, 32, 1), (3, 9, 3, 64, 2), (2, 12, 6, 96, 3),
                                           (2, 7, 17, 128, 4), (5, 10, 5, 512, 5)])
def test_fused_shortest_distance_small(B, T, V, H, seed):
    announce("fused forward", B, T, V, H)
    s = workloads.shared_emb(B=B, T=T, V=V, order=2, H=H, seed=seed, len_lo=max(1, T - 3), len_hi=T)
    st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    dist = lb.last_shortest_distance(fused_inputs(s), torch.from_numpy(s["lengths"]).cuda(), order=2,
                                     item_status=st)
    torch.cuda.synchronize()
    o = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=False)
    assert st.cpu().tolist() == [0] * B
    assert_dist_close(dist.cpu().numpy(), o["D"])


def test_fused_shortest_distance_config4_shape_short():
    """Config 4's lattice (V=64, C=4161, hidden 512) on a few frames: every tile is full size."""
    announce("fused forward, config 4 shape, T=6")
    s = workloads.config(4, B=2, T=6)
    st = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    dist = lb.last_shortest_distance(fused_inputs(s), torch.from_numpy(s["lengths"]).cuda(), order=2,
                                     item_status=st)
    torch.cuda.synchronize()
    o = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=False)
    assert st.cpu().tolist() == [0, 0]
    assert_dist_close(dist.cpu().numpy(), o["D"])
