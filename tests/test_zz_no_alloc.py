"""The entry point that allocates nothing (last_shortest_distance_static): same results as
last_shortest_distance, on two calls in a row, the second with a smaller input, in both semirings."""
import numpy as np
import pytest
import torch

from paper_2304_13134_amd import binding as lb
from paper_2304_13134_amd import workloads
from gpu_util import announce, dev



def _case(B, T, V, seed):
    rng = np.random.default_rng(seed)
    lengths = rng.integers(max(1, T // 2), T + 1, size=B).astype(np.int32)
    w = rng.standard_normal((B, T, V + 1, V + 1)).astype(np.float32)
    return dev(w), dev(lengths)


@pytest.mark.gpu
def test_static_scratch_entry_matches_workspace_entry():
    lb.load_library()
    # first a lattice that takes the clustered kernels (exchange buffers, stored state vectors in
    # the scratch array), then a smaller one that takes the one-workgroup kernels
    for (B, T, V) in ((5, 40, 200), (3, 12, 7)):
        w, lengths = _case(B, T, V, 11 + V)
        for semiring in ("log", "tropical"):
            announce("static scratch", B, T, V, semiring)
            want = lb.last_shortest_distance(w, lengths, order=1, semiring=semiring)
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            got = torch.full((B,), float("nan"), dtype=torch.float32, device="cuda")
            mid = torch.cuda.memory_allocated()
            lb.last_shortest_distance_static(w, lengths, got, order=1, semiring=semiring)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == mid and mid >= before
            g, x = got.cpu().numpy().astype(np.float64), want.cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(g))
            assert np.max(np.abs(g - x) / np.maximum(1.0, np.abs(x))) <= 1e-5, (g, x)


def test_static_scratch_entry_rejects_what_does_not_fit():
    lb.load_library()
    # [B][T+1][C] stored state vectors, twice, beyond the 32 MiB of the static array
    B, T, V = 16, 1200, 256
    wt = lb.LastWeights(lb.WEIGHTS_DENSE, B, T, 0x1000, None, None, None, 0)
    cx = lb.context(V, 1)
    assert lb.last_workspace_bytes(wt, cx, lb.OP_SHORTEST_DISTANCE) > lb.STATIC_SCRATCH_BYTES
    import ctypes
    rc = lb.load_library().last_shortest_distance_static(ctypes.byref(wt), ctypes.c_void_p(0x2000), ctypes.byref(cx),
                                                         0, ctypes.c_void_p(0x3000), None, None)
    assert rc == 5
