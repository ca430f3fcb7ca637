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


@pytest.mark.parametrize("B,T,V,H,seed", [(1, 4, 2, 128, 1), (3, 9, 3, 128, 2), (2, 12, 6, 256, 3),
                                           (2, 7, 17, 384, 4), (5, 10, 5, 512, 5), (2, 5, 40, 128, 6)])
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


@pytest.mark.parametrize("B,T,V,H,lens,seed", [(2, 1, 4, 128, [1, 0], 11), (3, 5, 8, 128, [5, 4, 1], 12),
                                                (2, 9, 20, 256, [9, 2], 13), (4, 12, 33, 384, [12, 11, 7, 3], 14),
                                                (2, 7, 64, 512, [7, 6], 15)])
def test_fused_frames_per_tile(B, T, V, H, lens, seed):
    """Weights of one or of two frames at a time in the forward kernel (the library's
    LAST_OPT_FUSED_FRAMES_PER_TILE): both against the oracle, odd and even lengths, a length of one
    and of zero, full-size tiles; the two settings give the same bits (each frame's weights and the
    recursion are computed by the same instructions, only their order in time differs)."""
    from gpu_util import library_option
    announce("fused forward, frames per tile 1 and 2", B, T, V, H, lens)
    s = workloads.shared_emb(B=B, T=T, V=V, order=2, H=H, seed=seed)
    s["lengths"] = np.asarray(lens, dtype=np.int32)
    se, lengths = fused_inputs(s), torch.from_numpy(s["lengths"]).cuda()
    o = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=True)
    got = {}
    for frames in (1, 2):
        with library_option(lb.OPT_FUSED_FRAMES_PER_TILE, frames):
            st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
            dist = lb.last_shortest_distance(se, lengths, order=2, item_status=st)
            dist2, grads = lb.last_arc_posteriors(se, lengths, order=2, item_status=st)
            torch.cuda.synchronize()
        assert st.cpu().tolist() == [0] * B
        assert_dist_close(dist.cpu().numpy(), o["D"])
        assert torch.equal(dist, dist2)
        for name, a, b in zip(("df", "de", "dW"), grads, (o["df"], o["de"], o["dW"])):
            assert_grad_close(name, a.cpu().numpy(), b.astype(np.float64))
        got[frames] = dist.cpu()
    assert torch.equal(got[1], got[2])


@pytest.mark.parametrize("keep", [0, 1])
@pytest.mark.parametrize("B,T,V,H,seed", [(3, 9, 3, 128, 21), (2, 7, 17, 384, 22), (2, 6, 64, 512, 23)])
def test_fused_gradients_with_and_without_kept_marginals(B, T, V, H, seed, keep):
    """dW from the marginals the backward kernel kept in the workspace (LAST_OPT_FUSED_KEEP_MARGINALS = 1,
    the default) and from marginals rebuilt with a third evaluation of the weights (0): both against the
    oracle; the workspace the library asks for follows the setting."""
    from gpu_util import library_option
    announce("fused gradients, kept marginals", keep, B, T, V, H)
    s = workloads.shared_emb(B=B, T=T, V=V, order=2, H=H, seed=seed, len_lo=max(1, T - 3), len_hi=T)
    se, lengths = fused_inputs(s), torch.from_numpy(s["lengths"]).cuda()
    o = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=True)
    wt = lb.LastWeights(lb.WEIGHTS_SHARED_EMB, B, T, None, se[0].data_ptr(), se[1].data_ptr(), se[2].data_ptr(), H)
    cx = lb.context(V, 2)
    with library_option(lb.OPT_FUSED_KEEP_MARGINALS, 0):
        n0 = lb.last_workspace_bytes(wt, cx, lb.OP_ARC_POSTERIORS)
    with library_option(lb.OPT_FUSED_KEEP_MARGINALS, 1):
        n1 = lb.last_workspace_bytes(wt, cx, lb.OP_ARC_POSTERIORS)
    assert n1 >= n0 + B * T * V * (V + 2) * (V + 1) * 4
    with library_option(lb.OPT_FUSED_KEEP_MARGINALS, keep):
        st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        dist, grads = lb.last_arc_posteriors(se, lengths, order=2, item_status=st)
        torch.cuda.synchronize()
    assert st.cpu().tolist() == [0] * B
    assert_dist_close(dist.cpu().numpy(), o["D"])
    for name, a, b in zip(("df", "de", "dW"), grads, (o["df"], o["de"], o["dW"])):
        assert_grad_close(name, a.cpu().numpy(), b.astype(np.float64))


# Gradients of the fused path: the marginals enter two bf16 matrix-core contractions as hi + lo
# halves (16 significant bits), tanh is evaluated in float32 before the bf16 rounding (a value
# that lands within ~1e-6 of a rounding boundary may round the other way than the float64
# oracle's: one 2^-9 relative step on one hidden unit), and sums run in float32 in a different
# order.  Bound used: 1e-4 * max(1, largest magnitude of the tensor); measured deviations are 3e-6 of
# that magnitude at most (sizes from a handful of frames to the full configurations).
def assert_grad_close(name, got, want):
    got = np.asarray(got, dtype=np.float64)
    tol = 1e-4 * max(1.0, float(np.max(np.abs(want))))
    err = float(np.max(np.abs(got - want)))
    assert np.all(np.isfinite(got)), name
    assert err <= tol, "%s: max abs error %.3g > %.3g (max |ref| %.3g)" % (name, err, tol, np.max(np.abs(want)))


def run_fused_grads(s, scale=1.0):
    B = s["f"].shape[0]
    st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    dist, (df, de, dW) = lb.last_arc_posteriors(fused_inputs(s), torch.from_numpy(s["lengths"]).cuda(),
                                                order=2, scale=scale, item_status=st)
    torch.cuda.synchronize()
    o = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=True)
    assert st.cpu().tolist() == [0] * B
    assert_dist_close(dist.cpu().numpy(), o["D"])
    assert_grad_close("df", df.cpu().numpy(), scale * o["df"])
    assert_grad_close("de", de.cpu().numpy(), scale * o["de"])
    assert_grad_close("dW", dW.cpu().numpy(), scale * o["dW"])
    return o, (df, de, dW)


@pytest.mark.parametrize("B,T,V,H,seed", [(1, 4, 2, 128, 11), (3, 9, 3, 128, 12), (2, 12, 6, 256, 13),
                                           (2, 7, 17, 384, 14), (5, 10, 5, 512, 15), (2, 5, 40, 128, 16)])
def test_fused_gradients_small(B, T, V, H, seed):
    announce("fused forward-backward", B, T, V, H)
    s = workloads.shared_emb(B=B, T=T, V=V, order=2, H=H, seed=seed, len_lo=max(1, T - 3), len_hi=T)
    o, (df, de, dW) = run_fused_grads(s)
    # frames past the length of an item get no gradient
    for b in range(B):
        assert float(df[b, int(s["lengths"][b]):].abs().max() if s["lengths"][b] < T else 0.0) == 0.0


def test_fused_gradients_scale_and_accumulate():
    announce("fused forward-backward, scale and accumulate")
    s = workloads.shared_emb(B=2, T=6, V=4, order=2, H=128, seed=21, len_lo=4, len_hi=6)
    o, (df, de, dW) = run_fused_grads(s, scale=-0.5)
    lengths = torch.from_numpy(s["lengths"]).cuda()
    lb.last_arc_posteriors(fused_inputs(s), lengths, order=2, dw=(df, de, dW), scale=1.5, accumulate=True)
    torch.cuda.synchronize()
    assert_grad_close("df", df.cpu().numpy(), o["df"])
    assert_grad_close("de", de.cpu().numpy(), o["de"])
    assert_grad_close("dW", dW.cpu().numpy(), o["dW"])


def test_fused_gradients_config4_shape_short():
    announce("fused forward-backward, config 4 shape, T=6")
    s = workloads.config(4, B=2, T=6)
    run_fused_grads(s)


def test_fused_full_size_against_stored_oracle_results():
    """Config 4 at full size (B=4, T=1000, V=64, hidden 512), the launch configuration the
    benchmark times.  The float64 oracle needs about 20 core-minutes for it, so its results are
    stored: tests/golden/config4_fused.npz, written by tests/golden/make_config4_fused.py, which
    calls only the oracle (D, dW whole, 4096 seeded samples each of df and de)."""
    import os
    announce("fused forward-backward, config 4 full size")
    gold = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config4_fused.npz"))
    s = workloads.config(4)
    B = s["f"].shape[0]
    st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    dist, (df, de, dW) = lb.last_arc_posteriors(fused_inputs(s), torch.from_numpy(s["lengths"]).cuda(),
                                                order=2, item_status=st)
    torch.cuda.synchronize()
    assert st.cpu().tolist() == [0] * B
    assert_dist_close(dist.cpu().numpy(), gold["D"])
    assert_grad_close("dW", dW.cpu().numpy(), gold["dW"])
    dfs = df.cpu().numpy().ravel()[gold["idx_f"]].astype(np.float64)
    des = de.cpu().numpy().ravel()[gold["idx_e"]].astype(np.float64)
    for name, got, want, mx in (("df", dfs, gold["df"], float(gold["df_max"])),
                                ("de", des, gold["de"], float(gold["de_max"]))):
        tol = 1e-4 * max(1.0, mx)
        err = float(np.max(np.abs(got - want)))
        assert np.all(np.isfinite(got)), name
        assert err <= tol, "%s: max abs error %.3g > %.3g (max |ref| %.3g)" % (name, err, tol, mx)
    # frames past the length of an item get no gradient; the total is finite
    assert bool(torch.isfinite(df).all()) and bool(torch.isfinite(de).all())


# ------------------------------------------------- numerator on on-the-fly weights
def run_fused_loss(s, order=2):
    """Denominator forward-backward, then the numerator accumulated with scale -1: (D, N, grads)."""
    se = fused_inputs(s)
    lengths = torch.from_numpy(s["lengths"]).cuda()
    refs, ulen = torch.from_numpy(s["refs"]).cuda(), torch.from_numpy(s["ref_lengths"]).cuda()
    B = s["f"].shape[0]
    st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    dist, grads = lb.last_arc_posteriors(se, lengths, order=order)
    num = lb.last_intersect_reference(se, lengths, refs, ulen, order=order, dw=grads, scale=-1.0,
                                      accumulate=True, item_status=st)
    torch.cuda.synchronize()
    return dist.cpu().numpy(), num.cpu().numpy(), [g.cpu().numpy() for g in grads], st.cpu().numpy()


@pytest.mark.parametrize("B,T,V,H,U,seed", [(2, 9, 3, 128, 4, 11), (3, 20, 6, 256, 9, 12),
                                             (2, 14, 17, 384, 14, 13), (2, 40, 5, 512, 21, 14)])
def test_fused_numerator_small(B, T, V, H, U, seed):
    announce("numerator on on-the-fly weights", B, T, V, H, U)
    s = workloads.shared_emb(B=B, T=T, V=V, order=2, H=H, seed=seed, len_lo=max(U, T - 3), len_hi=T)
    rng = np.random.default_rng(seed)
    s["refs"], s["ref_lengths"] = workloads.references(rng, B, V, U, max(0, U - 3), U)
    se = fused_inputs(s)
    lengths = torch.from_numpy(s["lengths"]).cuda()
    refs, ulen = torch.from_numpy(s["refs"]).cuda(), torch.from_numpy(s["ref_lengths"]).cuda()
    st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    g = [torch.full(t.shape, 7.0, dtype=torch.float32, device="cuda") for t in se]
    num = lb.last_intersect_reference(se, lengths, refs, ulen, order=2, dw=g, scale=1.0, accumulate=False,
                                      item_status=st)
    num2 = lb.last_intersect_reference(se, lengths, refs, ulen, order=2)          # without gradients
    torch.cuda.synchronize()
    o = oracle.fused_numerator(s["f"], s["e"], s["W"], s["lengths"], s["refs"], s["ref_lengths"], 2)
    assert st.cpu().tolist() == [0] * B
    assert_dist_close(num.cpu().numpy(), o["N"], "numerator")
    assert torch.equal(num, num2)
    for name, got, want in zip(("df", "de", "dW"), g, (o["df"], o["de"], o["dW"])):
        assert_grad_close(name, got.cpu().numpy(), want)
    # the full loss gradient: denominator marginals minus numerator marginals through the weight function
    D, N, grads, st2 = run_fused_loss(s)
    den = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=True)
    assert np.all(st2 == 0)
    assert_dist_close(D, den["D"])
    for name, got, a, b in zip(("df", "de", "dW"), grads, (den["df"], den["de"], den["dW"]),
                               (o["df"], o["de"], o["dW"])):
        tol = 1e-4 * max(1.0, np.max(np.abs(a)) + np.max(np.abs(b)))      # a difference of two such terms
        assert np.max(np.abs(got - (a - b))) <= tol, name


def test_fused_numerator_bigram_context_and_edge_cases():
    announce("numerator on on-the-fly weights: context size 1, wide vocabulary, U=0, U=len, U>len, bad label")
    s = workloads.shared_emb(B=5, T=12, V=100, order=1, H=128, seed=21)
    s["lengths"] = np.array([12, 7, 4, 12, 12], np.int32)
    rng = np.random.default_rng(21)
    refs, _ = workloads.references(rng, 5, 100, 13, 1, 5)
    ulen = np.array([0, 7, 5, 3, 14], np.int32)
    refs[3, 1] = 101
    se = fused_inputs(s)
    st = torch.full((5,), -1, dtype=torch.int32, device="cuda")
    g = [torch.full(t.shape, 3.0, dtype=torch.float32, device="cuda") for t in se]
    num = lb.last_intersect_reference(se, torch.from_numpy(s["lengths"]).cuda(), torch.from_numpy(refs).cuda(),
                                      torch.from_numpy(ulen).cuda(), order=1, dw=g, scale=1.0, accumulate=False,
                                      item_status=st).cpu().numpy()
    assert st.cpu().tolist() == [0, 0, 4, 2, 3]
    assert num[2] == -np.inf and np.isnan(num[3]) and np.isnan(num[4])
    o = oracle.fused_numerator(s["f"][:2], s["e"], s["W"], s["lengths"][:2], refs[:2], ulen[:2], 1)
    assert_dist_close(num[:2], o["N"])
    assert_grad_close("df", g[0].cpu().numpy()[:2], o["df"])
    assert torch.all(g[0][2:] == 0)
    assert_grad_close("de", g[1].cpu().numpy(), o["de"])
    assert_grad_close("dW", g[2].cpu().numpy(), o["dW"])


def test_fused_numerator_table2_shape_two_items():
    """The paper's benchmark shape (Table 2: 32 labels, 1057 states, 512 hidden units, 1024 frames,
    256 output labels) on two items, numerator and its gradients against the oracle."""
    announce("numerator on on-the-fly weights, Table 2 shape, B=2")
    s = workloads.config(5, B=2)
    se = fused_inputs(s)
    st = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    g = [torch.empty(t.shape, dtype=torch.float32, device="cuda") for t in se]
    num = lb.last_intersect_reference(se, torch.from_numpy(s["lengths"]).cuda(), torch.from_numpy(s["refs"]).cuda(),
                                      torch.from_numpy(s["ref_lengths"]).cuda(), order=2, dw=g, scale=1.0,
                                      accumulate=False, item_status=st)
    torch.cuda.synchronize()
    o = oracle.fused_numerator(s["f"], s["e"], s["W"], s["lengths"], s["refs"], s["ref_lengths"], 2)
    assert st.cpu().tolist() == [0, 0]
    assert_dist_close(num.cpu().numpy(), o["N"], "numerator")
    for name, got, want in zip(("df", "de", "dW"), g, (o["df"], o["de"], o["dW"])):
        assert_grad_close(name, got.cpu().numpy(), want)


def test_table2_shape_full_loss_against_stored_oracle_results():
    """One training step at the shape of the paper's benchmark (Table 2), all 16 items: D, N and the
    gradient of D - N against tests/golden/table2_fused.npz, written by
    tests/golden/make_table2_fused.py, which calls only the oracle (D, N, dW whole, 4096 seeded
    samples each of df and de)."""
    import os
    announce("Table 2 shape, full loss, B=16 T=1024 V=32 U=256 hidden 512")
    gold = np.load(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "table2_fused.npz"))
    s = workloads.config(5)
    D, N, (df, de, dW), st = run_fused_loss(s)
    assert np.all(st == 0)
    assert_dist_close(D, gold["D"])
    assert_dist_close(N, gold["N"], "numerator")
    assert np.all(N <= D)
    dfs = df.ravel()[gold["idx_f"]].astype(np.float64)
    des = de.ravel()[gold["idx_e"]].astype(np.float64)
    # the gradient is a difference of two terms of these magnitudes, each within the bound above
    for name, got, want, mx in (("dW", dW.astype(np.float64), gold["dW"], float(np.max(np.abs(gold["dW"])))),
                                ("df", dfs, gold["df"], float(gold["df_max"])),
                                ("de", des, gold["de"], float(gold["de_max"]))):
        tol = 1e-4 * max(1.0, mx)
        err = float(np.max(np.abs(got - want)))
        assert np.all(np.isfinite(got)), name
        assert err <= tol, "%s: max abs error %.3g > %.3g (max |ref| %.3g)" % (name, err, tol, mx)


def test_fused_loss_in_one_call():
    announce("loss in one call on on-the-fly weights")
    s = workloads.shared_emb(B=3, T=20, V=6, order=2, H=256, seed=31, len_lo=17, len_hi=20)
    rng = np.random.default_rng(31)
    s["refs"], s["ref_lengths"] = workloads.references(rng, 3, 6, 9, 4, 9)
    D, N, grads, st = run_fused_loss(s)
    se = fused_inputs(s)
    st1 = torch.full((3,), -1, dtype=torch.int32, device="cuda")
    d1, n1, g1 = lb.last_globally_normalized_loss(se, torch.from_numpy(s["lengths"]).cuda(),
                                                  torch.from_numpy(s["refs"]).cuda(),
                                                  torch.from_numpy(s["ref_lengths"]).cuda(), order=2, item_status=st1)
    torch.cuda.synchronize()
    assert st1.cpu().tolist() == [0, 0, 0]
    assert np.array_equal(d1.cpu().numpy(), D) and np.array_equal(n1.cpu().numpy(), N)
    for name, a, b in zip(("df", "de", "dW"), g1, grads):
        assert_grad_close(name, a.cpu().numpy(), b.astype(np.float64))


@pytest.mark.parametrize("frames", [1, 2])
def test_fused_bounded_waits_end_every_kernel_and_are_reported(frames):
    """Spin limit of one poll on the fused kernels: every kernel ends, items that gave up carry status 5."""
    from gpu_util import library_option
    announce("spin limit 1, fused forward-backward, frames per tile", frames)
    s = workloads.shared_emb(B=3, T=12, V=6, order=2, H=256, seed=77)
    se, lengths = fused_inputs(s), torch.from_numpy(s["lengths"]).cuda()
    with library_option(lb.OPT_SPIN_LIMIT, 1), library_option(lb.OPT_FUSED_FRAMES_PER_TILE, frames):
        st = torch.full((3,), -1, dtype=torch.int32, device="cuda")
        dist, grads = lb.last_arc_posteriors(se, lengths, order=2, item_status=st)
        torch.cuda.synchronize()
    st = st.cpu().numpy()
    assert set(st.tolist()) <= {0, 5}
    o = oracle.fused_forward_backward(s["f"], s["e"], s["W"], s["lengths"], 2, round_h=True, grads=False)
    for b in range(3):
        if st[b] == 0:
            assert abs(float(dist[b]) - o["D"][b]) <= 1e-5 * abs(o["D"][b])
        else:
            assert torch.isnan(dist[b])
    st2 = torch.full((3,), -1, dtype=torch.int32, device="cuda")
    dist2 = lb.last_shortest_distance(se, lengths, order=2, item_status=st2)
    torch.cuda.synchronize()
    assert st2.cpu().tolist() == [0, 0, 0]
    assert_dist_close(dist2.cpu().numpy(), o["D"])
