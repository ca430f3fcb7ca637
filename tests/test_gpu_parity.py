"""GPU parity: the HIP path (through the C ABI) against the float64 CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from oracle import brute_force as bf
from paper_2304_13134_amd import binding as lb
from paper_2304_13134_amd import workloads
from gpu_util import TOL_POST_ABS, announce, assert_dist_close, dev, library_option

pytestmark = pytest.mark.gpu


def run_posteriors(cfg, order=1):
    w = dev(cfg["w"])
    lengths = dev(cfg["lengths"])
    status = torch.full((cfg["B"],), -1, dtype=torch.int32, device="cuda")
    dist, dw = lb.last_arc_posteriors(w, lengths, order=order, item_status=status)
    torch.cuda.synchronize()
    return dist.cpu().numpy(), dw.cpu().numpy(), status.cpu().numpy()


def check_posteriors(cfg, order=1):
    D, gamma, status = run_posteriors(cfg, order)
    alpha, D_o = oracle.forward(cfg["w"], cfg["lengths"], order)
    gamma_o = oracle.posteriors(cfg["w"], cfg["lengths"], order)
    assert np.all(status == 0)
    assert_dist_close(D, D_o)
    assert not np.any(np.isnan(gamma))
    assert np.max(np.abs(gamma - gamma_o)) <= TOL_POST_ABS
    # exact zeros where the oracle has exact zeros (padding, unreachable states)
    assert np.all(gamma[gamma_o == 0.0] == 0.0)
    return D, gamma


def check_path(cfg, order=1):
    w = dev(cfg["w"])
    lengths = dev(cfg["lengths"])
    labels, states, score = lb.last_shortest_path(w, lengths, order=order)
    dist = lb.last_shortest_distance(w, lengths, order=order, semiring="tropical")
    torch.cuda.synchronize()
    l_o, s_o, sc_o = oracle.viterbi(cfg["w"], cfg["lengths"], order, "f32")
    assert np.array_equal(labels.cpu().numpy(), l_o)
    assert np.array_equal(states.cpu().numpy(), s_o)
    assert np.array_equal(score.cpu().numpy(), sc_o)          # same float32 adds: bit-exact
    assert np.array_equal(dist.cpu().numpy(), sc_o)


def test_config0_against_oracle_and_enumeration():
    announce("config 0: B=1 T=8 V=3 bigram")
    cfg = workloads.config(0)
    D, gamma = check_posteriors(cfg)
    labels, states, scores = bf.enumerate_paths(cfg["w"][0], 1)
    D_bf, g_bf = bf.arc_marginals(labels, states, scores, cfg["w"][0].shape)
    assert abs(D[0] - D_bf) <= 1e-5 * abs(D_bf)
    assert np.max(np.abs(gamma[0] - g_bf)) <= TOL_POST_ABS
    check_path(cfg)
    dist = lb.last_shortest_distance(dev(cfg["w"]), dev(cfg["lengths"]))
    assert_dist_close(dist.cpu().numpy(), [D_bf])


def test_config1_full():
    announce("config 1: B=8 T<=200 V=32 bigram, variable lengths")
    cfg = workloads.config(1)
    check_posteriors(cfg)
    check_path(cfg)


def test_config1_nan_padding_is_ignored():
    announce("config 1 with NaN in the padded frames")
    cfg = workloads.config(1, pad_nan=True)
    assert np.isnan(cfg["w"]).any()
    check_posteriors(cfg)
    check_path(cfg)


@pytest.mark.parametrize("V,T,B", [(4, 25, 3), (12, 14, 2)])
def test_order2_dense(V, T, B):
    announce("dense trigram context", V, T, B)
    cfg = workloads.dense(B=B, T=T, V=V, order=2, sigma=1.5, seed=77, len_lo=T - 5, len_hi=T)
    check_posteriors(cfg, order=2)
    check_path(cfg, order=2)


def test_config2_reduced_spans_several_tiles():
    announce("config 2 reduced: B=3 T=40 V=256 sigma=2")
    cfg = workloads.config(2, B=3, T=40)
    check_posteriors(cfg)
    check_path(cfg)


def test_ragged_vocabulary_sizes():
    # (3 and 4: the smallest label sets on either side of the clustered kernel's four-column accesses)
    for V in (1, 2, 3, 4, 5, 8, 32, 33, 34, 63, 64, 65, 130):
        announce("ragged V", V)
        cfg = workloads.dense(B=2, T=9, V=V, order=1, sigma=1.0, seed=V, len_lo=5, len_hi=9)
        check_posteriors(cfg)
        check_path(cfg)


def test_state_counts_around_256_and_every_pair_parity():
    # the clustered kernels give columns and rows beyond 256 to the last wave's tail, walk frames in
    # pairs from either end and meet in the middle: cover the sizes and the lengths around those edges
    for V in (254, 255, 256, 257, 263, 264):
        announce("clustered path, V", V)
        cfg = workloads.dense(B=6, T=9, V=V, order=1, sigma=2.0, seed=300 + V, len_lo=1, len_hi=9)
        cfg["lengths"] = np.array([1, 2, 3, 4, 8, 9], dtype=np.int32)
        check_posteriors(cfg)
        check_path(cfg)


def test_first_generation_clustered_kernel():
    # the kernel with one exchange per frame stays covered
    with library_option(lb.OPT_CLUSTER_GENERATION, 1):
        announce("first-generation clustered kernel: B=3 T=40 V=256")
        check_posteriors(workloads.config(2, B=3, T=40))
        for V in (65, 130, 263):
            cfg = workloads.dense(B=2, T=9, V=V, order=1, sigma=1.0, seed=V, len_lo=5, len_hi=9)
            check_posteriors(cfg)


@pytest.mark.parametrize("generation", [2, 3])
def test_clustered_kernel_generations_at_256_labels(generation):
    # both kernels that take 256 labels (eight / sixteen workgroups per direction and item) stay covered
    with library_option(lb.OPT_CLUSTER_GENERATION, generation):
        announce("clustered kernel generation", generation, ": B=3 T=40 V=256, every pair parity, B=37")
        check_posteriors(workloads.config(2, B=3, T=40))
        cfg = workloads.dense(B=6, T=9, V=256, order=1, sigma=2.0, seed=556, len_lo=1, len_hi=9)
        cfg["lengths"] = np.array([1, 2, 3, 4, 8, 9], dtype=np.int32)
        check_posteriors(cfg)
        check_posteriors(workloads.dense(B=37, T=6, V=256, order=1, sigma=2.0, seed=3737, len_lo=0, len_hi=6))


def test_more_items_than_clusters():
    # 37 items on 16 clusters: every cluster walks several items one after the other, with ragged lengths
    announce("clustered path: B=37 T=6 V=256")
    cfg = workloads.dense(B=37, T=6, V=256, order=1, sigma=2.0, seed=3737, len_lo=0, len_hi=6)
    check_posteriors(cfg)
    check_path(cfg)


def test_one_workgroup_shortest_path_kernels():
    # the shortest-path kernels with one workgroup per item stay covered
    with library_option(lb.OPT_CLUSTER_VITERBI, 0):
        announce("one-workgroup shortest path: B=3 T=40 V=256, and ragged sizes")
        check_path(workloads.config(2, B=3, T=40))
        for V in (5, 130, 200, 263):
            check_path(workloads.dense(B=2, T=9, V=V, order=1, sigma=1.0, seed=V, len_lo=5, len_hi=9))


def test_both_clustered_shortest_path_kernels_at_256_labels():
    """256 labels take the kernel with the work cut down to the wave (LAST_OPT_CLUSTER_VITERBI = 1, the
    default); 2 selects the older clustered kernel, which other label counts use anyway.  Both against the
    oracle: random weights with ragged lengths (a length of 1, of 2, odd and even ones), integer weights
    with many ties, all-equal weights, forbidden arcs."""
    rng = np.random.default_rng(11)
    for mode in (1, 2):
        with library_option(lb.OPT_CLUSTER_VITERBI, mode):
            announce("clustered shortest path at 256 labels, kernel", mode)
            cfg = workloads.config(2, B=9, T=21)
            cfg["lengths"] = np.array([21, 20, 1, 2, 3, 0, 17, 8, 21], np.int32)
            check_path(cfg)
            wc = rng.integers(-1, 2, size=(3, 12, 257, 257)).astype(np.float32)
            check_path(dict(w=wc, lengths=np.array([12, 7, 11], np.int32), B=3))
            check_path(dict(w=np.zeros((2, 6, 257, 257), np.float32), lengths=np.array([6, 5], np.int32), B=2))
            check_path(forbid_arcs(workloads.config(2, B=2, T=10), 5))
            # more items than clusters: every cluster walks several items one after the other
            many = workloads.config(2, B=35, T=6)
            many["lengths"] = (np.arange(35) % 7).astype(np.int32)
            check_path(many)


def forbid_arcs(cfg, seed):
    """A third of the arcs, every arc out of state 5 and label 7 at frame 3 get weight -1e4."""
    rng = np.random.default_rng(seed)
    w = cfg["w"]
    w[rng.random(w.shape) < 0.3] = -1.0e4
    w[:, :, 5, :] = -1.0e4
    w[:, 3, :, 7] = -1.0e4
    return cfg


def test_wide_dynamic_range_is_exact_or_flagged():
    # weights of up to about +-50 with forbidden arcs: exact on the bandwidth path, status 0
    announce("wide range: sigma 12 with forbidden arcs")
    cfg = forbid_arcs(workloads.dense(B=3, T=14, V=256, order=1, sigma=12.0, seed=1200, len_lo=11, len_hi=14), 5)
    check_posteriors(cfg)
    check_path(cfg)
    # far beyond what scaled float32 state vectors hold (weights of +-180): the distance is still right and
    # every item says that its marginals may not be (status 6), without NaN
    announce("wide range: sigma 40")
    cfg = forbid_arcs(workloads.dense(B=2, T=11, V=130, order=1, sigma=40.0, seed=4130, len_lo=8, len_hi=11), 5)
    D, gamma, status = run_posteriors(cfg)
    _, D_o = oracle.forward(cfg["w"], cfg["lengths"], 1)
    gamma_o = oracle.posteriors(cfg["w"], cfg["lengths"], 1)
    assert_dist_close(D, D_o)
    assert not np.any(np.isnan(gamma))
    for b in range(cfg["B"]):
        assert status[b] in (0, 6)
        if status[b] == 0:
            assert np.max(np.abs(gamma[b] - gamma_o[b])) <= TOL_POST_ABS
    check_path(cfg)
    # the log-domain kernels take the same input without a flag; float32 weights of this size resolve
    # 2^-16, so the marginals agree to a few 1e-5 only
    announce("wide range: sigma 40, one workgroup per item")
    with library_option(lb.OPT_FORCE_SOLO, 1):
        D, gamma, status = run_posteriors(cfg)
    assert np.all(status == 0)
    assert_dist_close(D, D_o)
    assert np.max(np.abs(gamma - gamma_o)) <= 5.0e-5


def test_edge_lengths_and_status():
    announce("edge lengths: 0, 1, T, invalid")
    cfg = workloads.dense(B=5, T=6, V=5, order=1, seed=5)
    cfg["lengths"] = np.array([0, 1, 6, 7, -1], dtype=np.int32)
    D, gamma, status = run_posteriors(cfg)
    assert list(status) == [0, 0, 0, 1, 1]
    assert np.isnan(D[3]) and np.isnan(D[4])
    assert np.all(gamma[3:] == 0.0) and np.all(gamma[0] == 0.0)
    ok = dict(cfg, w=cfg["w"][:3], lengths=cfg["lengths"][:3], B=3)
    alpha, D_o = oracle.forward(ok["w"], ok["lengths"], 1)
    g_o = oracle.posteriors(ok["w"], ok["lengths"], 1)
    assert_dist_close(D[:3], D_o)
    assert D[0] == 0.0
    assert np.max(np.abs(gamma[:3] - g_o)) <= TOL_POST_ABS
    labels, states, score = lb.last_shortest_path(dev(cfg["w"]), dev(cfg["lengths"]))
    l_o, s_o, sc_o = oracle.viterbi(ok["w"], ok["lengths"], 1, "f32")
    assert np.array_equal(labels.cpu().numpy()[:3], l_o)
    assert np.array_equal(states.cpu().numpy()[:3], s_o)
    assert np.all(labels.cpu().numpy()[3:] == -1) and np.all(states.cpu().numpy()[3:] == -1)


def test_scale_and_accumulate():
    announce("scale / accumulate semantics of the gradient output")
    # (6: one workgroup per direction; 130, 256: several workgroups whose lanes share columns at the
    # edges of their blocks, which adding must count once)
    for V, T in ((6, 7), (130, 9), (256, 10)):
        cfg = workloads.dense(B=2, T=T, V=V, order=1, seed=9 + V, len_lo=T - 2, len_hi=T)
        w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
        _, g1 = lb.last_arc_posteriors(w, lengths)
        base = torch.full_like(w, 0.5)
        lb.last_arc_posteriors(w, lengths, dw=base, scale=-2.0, accumulate=True)
        torch.cuda.synchronize()
        want = 0.5 - 2.0 * g1
        # frames beyond an item's length are left as they were
        for b in range(cfg["B"]):
            want[b, int(cfg["lengths"][b]):] = 0.5
        assert torch.max(torch.abs(base - want)).item() < 1e-6


def test_viterbi_ties_follow_the_lowest_flat_index():
    announce("tie rules on integer weights")
    rng = np.random.default_rng(3)
    w = rng.integers(-2, 3, size=(4, 30, 9, 9)).astype(np.float32)   # many exact ties
    cfg = dict(w=w, lengths=np.array([30, 17, 1, 30], np.int32), B=4)
    check_path(cfg)
    # the streaming kernel of the full 1-gram context dependency (both of its tilings)
    for C in (129, 200, 256, 257, 264):
        announce("tie rules on integer weights, C =", C)
        wc = rng.integers(-1, 2, size=(2, 11, C, C)).astype(np.float32)
        check_path(dict(w=wc, lengths=np.array([11, 6], np.int32), B=2))
    w0 = np.zeros((1, 5, 4, 4), np.float32)
    labels, states, score = lb.last_shortest_path(dev(w0), dev(np.array([5], np.int32)))
    assert labels.cpu().tolist() == [[0] * 5] and states.cpu().tolist() == [[0] * 6]


def check_loss(cfg, order=1):
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    refs, ulen = dev(cfg["refs"]), dev(cfg["ref_lengths"])
    st = torch.full((cfg["B"],), -1, dtype=torch.int32, device="cuda")
    dist, dw = lb.last_arc_posteriors(w, lengths, order=order)
    num = lb.last_intersect_reference(w, lengths, refs, ulen, order=order, dw=dw, scale=-1.0,
                                      accumulate=True, item_status=st)
    torch.cuda.synchronize()
    o = oracle.numerator(cfg["w"], cfg["lengths"], cfg["refs"], cfg["ref_lengths"], order)
    assert_dist_close(num.cpu().numpy(), o["N"], "numerator")
    gden = oracle.posteriors(cfg["w"], cfg["lengths"], order)
    gnum = oracle.numerator_posteriors_dense(o, cfg["refs"], cfg["ref_lengths"], cfg["w"].shape)
    grad = dw.cpu().numpy()
    assert np.max(np.abs(grad - (gden - gnum))) <= 2 * TOL_POST_ABS   # two 1e-5 terms
    _, D_o = oracle.forward(cfg["w"], cfg["lengths"], order)
    loss = dist.cpu().numpy().astype(np.float64) - num.cpu().numpy().astype(np.float64)
    fin = np.isfinite(o["N"])
    assert np.max(np.abs(loss[fin] - (D_o - o["N"])[fin]) / np.maximum(1, np.abs(D_o[fin]))) <= 2e-5
    # numerator-only gradient, overwrite mode
    only = torch.full_like(w, 7.0)
    lb.last_intersect_reference(w, lengths, refs, ulen, order=order, dw=only, scale=1.0, accumulate=False)
    torch.cuda.synchronize()
    assert np.max(np.abs(only.cpu().numpy() - gnum)) <= TOL_POST_ABS
    return st.cpu().numpy()


def test_full_loss_reduced_config3():
    announce("config 3 reduced: B=4 T=60 V=40 U in [5,30]")
    cfg = workloads.config(3, B=4, T=60, V=40, Umax=30, u_lo=5, u_hi=30)
    assert np.all(check_loss(cfg) == 0)


def test_full_loss_order2():
    announce("numerator with trigram context")
    cfg = workloads.config(3, B=2, T=20, V=5, order=2, Umax=12, u_lo=3, u_hi=12)
    assert np.all(check_loss(cfg, order=2) == 0)


def test_numerator_edge_cases():
    announce("numerator: U=0, U=len, U>len, bad label, bad ref length")
    cfg = workloads.config(3, B=5, T=10, V=6, Umax=12, u_lo=1, u_hi=5)
    cfg["lengths"] = np.array([10, 7, 4, 10, 10], np.int32)
    cfg["ref_lengths"] = np.array([0, 7, 5, 3, 13], np.int32)
    cfg["refs"][3, 1] = 9                                  # label outside 1..V
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    refs, ulen = dev(cfg["refs"]), dev(cfg["ref_lengths"])
    st = torch.full((5,), -1, dtype=torch.int32, device="cuda")
    dw = torch.zeros_like(w)
    num = lb.last_intersect_reference(w, lengths, refs, ulen, dw=dw, scale=1.0, accumulate=True,
                                      item_status=st)
    torch.cuda.synchronize()
    num = num.cpu().numpy()
    assert st.cpu().tolist() == [0, 0, 4, 2, 3]
    assert num[2] == -np.inf and np.isnan(num[3]) and np.isnan(num[4])
    assert torch.all(dw[2:] == 0)
    good = dict(w=cfg["w"][:2], lengths=cfg["lengths"][:2], refs=cfg["refs"][:2],
                ref_lengths=cfg["ref_lengths"][:2])
    o = oracle.numerator(good["w"], good["lengths"], good["refs"], good["ref_lengths"], 1)
    assert_dist_close(num[:2], o["N"])
    gnum = oracle.numerator_posteriors_dense(o, good["refs"], good["ref_lengths"], good["w"].shape)
    assert np.max(np.abs(dw.cpu().numpy()[:2] - gnum)) <= TOL_POST_ABS


# ------------------------------------------------------------------ full sizes
@pytest.fixture(scope="module")
def config3_full():
    """Configs 2 and 3 at full size (B=16, T=500, V=256): the lattice the benchmark times."""
    announce("building config 3 (2.1 GB) and its oracle forward / backward weights")
    cfg = workloads.config(3)
    alpha, D = oracle.forward(cfg["w"], cfg["lengths"], 1)
    beta = oracle.backward(cfg["w"], cfg["lengths"], 1)
    return cfg, alpha, beta, D


def test_config2_full_size_sampled_marginals_and_invariants(config3_full):
    announce("config 2 full size: D, sampled marginals, per-frame sums")
    cfg, alpha, beta, D_o = config3_full
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    st = torch.full((cfg["B"],), -1, dtype=torch.int32, device="cuda")
    dist, dw = lb.last_arc_posteriors(w, lengths, item_status=st)
    dist2 = lb.last_shortest_distance(w, lengths)
    torch.cuda.synchronize()
    assert torch.all(st == 0)
    assert_dist_close(dist.cpu().numpy(), D_o)
    assert_dist_close(dist2.cpu().numpy(), D_o)
    # every frame's marginals sum to 1 (one arc per frame in a frame dependent lattice)
    sums = dw.sum(dim=(2, 3), dtype=torch.float64).cpu().numpy()
    assert np.max(np.abs(sums - 1.0)) < 1e-4
    assert not torch.isnan(dw).any()
    # 400k sampled arcs + the largest marginals, each checked against Eq. 1 one by one
    rng = np.random.default_rng(11)
    n = 400_000
    idx = np.stack([rng.integers(0, cfg["B"], n), rng.integers(0, cfg["T"], n),
                    rng.integers(0, cfg["C"], n), rng.integers(0, cfg["V"] + 1, n)], axis=1)
    top = torch.topk(dw.view(-1), 20000).indices.cpu().numpy()
    tidx = np.stack(np.unravel_index(top, cfg["w"].shape), axis=1)
    idx = np.concatenate([idx, tidx])
    want = oracle.posterior_samples(cfg["w"], cfg["lengths"], 1, alpha, beta, D_o, idx)
    got = dw[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
    assert np.max(np.abs(got - want)) <= TOL_POST_ABS
    # frames 0 and 1: unreachable states carry exact zeros
    assert torch.all(dw[:, 0, 1:, :] == 0)


def test_config2_and_3_full_size_every_element(config3_full):
    """All 5.28e8 arc marginals of config 2 and the whole loss gradient of config 3 against the
    oracle's dense tensors, item by item (the oracle's forward and backward weights are reused)."""
    announce("configs 2 and 3 full size: every marginal and every element of the loss gradient")
    cfg, alpha, beta, D_o = config3_full
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    refs, ulen = dev(cfg["refs"]), dev(cfg["ref_lengths"])
    dist, dw = lb.last_arc_posteriors(w, lengths)
    d2, num, gl = lb.last_globally_normalized_loss(w, lengths, refs, ulen)
    torch.cuda.synchronize()
    o = oracle.numerator(cfg["w"], cfg["lengths"], cfg["refs"], cfg["ref_lengths"], 1)
    worst_den = worst_loss = 0.0
    for b in range(cfg["B"]):
        sl = slice(b, b + 1)
        gamma = oracle.posteriors(cfg["w"][sl], cfg["lengths"][sl], 1, alpha[sl], beta[sl], D_o[sl])
        got = dw[b].cpu().numpy()
        worst_den = max(worst_den, float(np.max(np.abs(got - gamma[0]))))
        assert np.all(got[gamma[0] == 0.0] == 0.0)
        one = dict(ctx=o["ctx"][sl], pb=o["pb"][sl], pl=o["pl"][sl])
        gnum = oracle.numerator_posteriors_dense(one, cfg["refs"][sl], cfg["ref_lengths"][sl], gamma.shape)
        worst_loss = max(worst_loss, float(np.max(np.abs(gl[b].cpu().numpy() - (gamma[0] - gnum[0])))))
        del gamma, gnum, got
    announce("largest deviation: marginals %.3g, loss gradient %.3g" % (worst_den, worst_loss))
    assert worst_den <= TOL_POST_ABS
    assert worst_loss <= 2 * TOL_POST_ABS
    assert_dist_close(d2.cpu().numpy(), D_o)
    assert_dist_close(num.cpu().numpy(), o["N"], "numerator")


def test_config2_full_size_shortest_path(config3_full):
    announce("config 2 full size: tropical shortest path, bit-exact indices")
    cfg, _, _, _ = config3_full
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    labels, states, score = lb.last_shortest_path(w, lengths)
    torch.cuda.synchronize()
    l_o, s_o, sc_o = oracle.viterbi(cfg["w"], cfg["lengths"], 1, "f32")
    assert np.array_equal(labels.cpu().numpy(), l_o)
    assert np.array_equal(states.cpu().numpy(), s_o)
    assert np.array_equal(score.cpu().numpy(), sc_o)


def test_config3_full_size_loss_and_gradient(config3_full):
    announce("config 3 full size: numerator, loss, gradient on the numerator's arcs")
    cfg, alpha, beta, D_o = config3_full
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    refs, ulen = dev(cfg["refs"]), dev(cfg["ref_lengths"])
    dist, dw = lb.last_arc_posteriors(w, lengths)
    num = lb.last_intersect_reference(w, lengths, refs, ulen, dw=dw, scale=-1.0, accumulate=True)
    torch.cuda.synchronize()
    o = oracle.numerator(cfg["w"], cfg["lengths"], cfg["refs"], cfg["ref_lengths"], 1)
    assert_dist_close(num.cpu().numpy(), o["N"], "numerator")
    assert np.all(o["N"] <= D_o)
    # gradient on every arc the intersected lattice rides on, for two items
    for b in (0, 9):
        U = int(cfg["ref_lengths"][b])
        T = cfg["T"]
        gnum = {}
        for u in range(U + 1):
            q = int(o["ctx"][b, u])
            for t in range(T):
                gnum[(t, q, 0)] = gnum.get((t, q, 0), 0.0) + o["pb"][b, t, u]
                if u < U:
                    y = int(cfg["refs"][b, u])
                    gnum[(t, q, y)] = gnum.get((t, q, y), 0.0) + o["pl"][b, t, u]
        keys = np.array(list(gnum.keys()))
        idx = np.concatenate([np.full((len(keys), 1), b), keys], axis=1)
        den = oracle.posterior_samples(cfg["w"], cfg["lengths"], 1, alpha, beta, D_o, idx)
        want = den - np.array(list(gnum.values()))
        got = dw[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy()
        assert np.max(np.abs(got - want)) <= 2 * TOL_POST_ABS
    sums = dw.sum(dim=(2, 3), dtype=torch.float64).cpu().numpy()
    assert np.max(np.abs(sums)) < 1e-4                 # denominator and numerator marginals cancel


# ------------------------------------------------------- loss in one call
def check_loss_one_call(cfg, order=1, g_order=None):
    """last_globally_normalized_loss against the two calls in sequence and against the oracle."""
    g_order = order if g_order is None else g_order
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    refs, ulen = dev(cfg["refs"]), dev(cfg["ref_lengths"])
    B = cfg["w"].shape[0]
    st = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    dist, num, dw = lb.last_globally_normalized_loss(w, lengths, refs, ulen, order=g_order, item_status=st)
    d2, dw2 = lb.last_arc_posteriors(w, lengths, order=g_order)
    n2 = lb.last_intersect_reference(w, lengths, refs, ulen, order=g_order, dw=dw2, scale=-1.0, accumulate=True)
    torch.cuda.synchronize()
    assert torch.equal(dist, d2) and torch.equal(num, n2)
    assert float((dw - dw2).abs().max()) <= 1e-6          # same kernels; float atomics may land in another order
    o = oracle.numerator(cfg["w"], cfg["lengths"], cfg["refs"], cfg["ref_lengths"], order)
    gden = oracle.posteriors(cfg["w"], cfg["lengths"], order)
    gnum = oracle.numerator_posteriors_dense(o, cfg["refs"], cfg["ref_lengths"], cfg["w"].shape)
    assert np.max(np.abs(dw.cpu().numpy() - (gden - gnum))) <= 2 * TOL_POST_ABS
    assert_dist_close(num.cpu().numpy(), o["N"], "numerator")
    # scale and accumulate; several calls in a row on the same stream
    acc = torch.full_like(w, 0.25)
    for _ in range(3):
        lb.last_globally_normalized_loss(w, lengths, refs, ulen, order=g_order, dw=acc, scale=0.5, accumulate=True)
    assert np.max(np.abs(acc.cpu().numpy() - (0.25 + 1.5 * (gden - gnum)))) <= 4 * TOL_POST_ABS
    return st.cpu().numpy()


def test_loss_in_one_call():
    announce("loss in one call: config 3 reduced (clustered denominator), B=4 T=60 V=256")
    cfg = workloads.config(3, B=4, T=60, V=256, Umax=30, u_lo=5, u_hi=30)
    assert np.all(check_loss_one_call(cfg) == 0)
    announce("loss in one call: context size 2, B=2 T=20 V=5")
    cfg = workloads.config(3, B=2, T=20, V=5, order=2, Umax=12, u_lo=3, u_hi=12)
    assert np.all(check_loss_one_call(cfg, order=2) == 0)
    announce("loss in one call: status of either part")
    cfg = workloads.config(3, B=4, T=10, V=6, Umax=12, u_lo=1, u_hi=5)
    cfg["lengths"] = np.array([10, 11, 4, 10], np.int32)
    cfg["ref_lengths"] = np.array([3, 2, 5, 13], np.int32)
    st = torch.full((4,), -1, dtype=torch.int32, device="cuda")
    dist, num, dw = lb.last_globally_normalized_loss(dev(cfg["w"]), dev(cfg["lengths"]), dev(cfg["refs"]),
                                                     dev(cfg["ref_lengths"]), item_status=st)
    assert st.cpu().tolist() == [0, 1, 4, 3]
    assert torch.isnan(dist[1]) and float(num[2]) == -np.inf and torch.isnan(num[3])


# ------------------------------------------------ bounded waits, driven from the host
def test_bounded_waits_end_every_kernel_and_are_reported():
    """With a spin limit of one poll the cooperating workgroups give up waiting for each other almost
    at once: every kernel must still end, every item must either be right or carry status 5 and NaN,
    and the next call with the normal limit must be right again."""
    cfg = workloads.dense(B=6, T=24, V=256, order=1, sigma=2.0, seed=4242, len_lo=20, len_hi=24)
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    _, D_o = oracle.forward(cfg["w"], cfg["lengths"], 1)
    gamma_o = oracle.posteriors(cfg["w"], cfg["lengths"], 1)
    l_o, s_o, sc_o = oracle.viterbi(cfg["w"], cfg["lengths"], 1, "f32")
    seen_timeouts = 0
    for generation in (3, 2, 1):
        announce("spin limit 1, clustered forward-backward, generation", generation)
        with library_option(lb.OPT_CLUSTER_GENERATION, generation), library_option(lb.OPT_SPIN_LIMIT, 1):
            st = torch.full((6,), -1, dtype=torch.int32, device="cuda")
            dist, dw = lb.last_arc_posteriors(w, lengths, item_status=st)
            torch.cuda.synchronize()
        st, dist, dw = st.cpu().numpy(), dist.cpu().numpy(), dw.cpu().numpy()
        assert set(st.tolist()) <= {0, 5}
        for b in range(6):
            if st[b] == 5:
                assert np.isnan(dist[b])
                seen_timeouts += 1
            else:
                assert abs(dist[b] - D_o[b]) <= 1e-5 * abs(D_o[b])
                assert np.max(np.abs(dw[b] - gamma_o[b])) <= TOL_POST_ABS
    for mode in (1, 2):
        announce("spin limit 1, clustered shortest path, kernel", mode)
        with library_option(lb.OPT_CLUSTER_VITERBI, mode), library_option(lb.OPT_SPIN_LIMIT, 1):
            st = torch.full((6,), -1, dtype=torch.int32, device="cuda")
            labels, states, score = lb.last_shortest_path(w, lengths, item_status=st)
            torch.cuda.synchronize()
        st = st.cpu().numpy()
        assert set(st.tolist()) <= {0, 5}
        for b in range(6):
            if st[b] == 5:
                assert torch.isnan(score[b]) and torch.all(labels[b] == -1) and torch.all(states[b] == -1)
                seen_timeouts += 1
            else:
                assert np.array_equal(labels[b].cpu().numpy(), l_o[b]) and float(score[b]) == sc_o[b]
    assert seen_timeouts > 0, "the bounded-wait path was not exercised"
    announce("normal spin limit again")
    check_posteriors(cfg)
    check_path(cfg)


def test_dense_context_size_2_with_more_than_1024_states():
    # 32 labels, context size 2: 1057 states, more than the 1024 threads of the one-workgroup kernels
    # (the state loop takes a second sweep); the lattice of the paper's Table 2 with dense weights
    announce("dense weights, context size 2, V=32 (C=1057), B=2 T<=9")
    cfg = workloads.config(3, B=2, T=9, V=32, order=2, Umax=6, u_lo=2, u_hi=6, len_lo=6, len_hi=9)
    check_posteriors(cfg, order=2)
    check_path(cfg, order=2)
    assert np.all(check_loss(cfg, order=2) == 0)


def test_calls_under_graph_capture_replay_like_eager():
    """The loss in one call (with its fork to the library's side stream and the join back) and the
    entry point that allocates nothing, captured into a HIP graph: every replay, with eager work
    between the replays, gives the eager results bit for bit."""
    announce("graph capture: loss in one call, static-scratch shortest distance; three replays")
    cfg = workloads.config(3, B=4, T=60, V=256, Umax=30, u_lo=5, u_hi=30)
    w, lengths = dev(cfg["w"]), dev(cfg["lengths"])
    refs, ulen = dev(cfg["refs"]), dev(cfg["ref_lengths"])
    st = torch.zeros(4, dtype=torch.int32, device="cuda")
    d0, n0, g0 = lb.last_globally_normalized_loss(w, lengths, refs, ulen, item_status=st)
    s0 = lb.last_shortest_distance(w, lengths)
    torch.cuda.synchronize()
    dw = torch.empty_like(w)
    sd = torch.empty(4, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up on a side stream, as graph capture asks for
        lb.last_globally_normalized_loss(w, lengths, refs, ulen, dw=dw, item_status=st)
        lb.last_shortest_distance_static(w, lengths, sd, item_status=st)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        d1, n1, _ = lb.last_globally_normalized_loss(w, lengths, refs, ulen, dw=dw, item_status=st)
        lb.last_shortest_distance_static(w, lengths, sd, item_status=st)
    for _ in range(3):
        dw.fill_(7.0)
        d1.fill_(0.0)
        n1.fill_(0.0)
        sd.fill_(0.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(d1, d0) and torch.equal(n1, n0) and torch.equal(sd, s0)
        assert float((dw - g0).abs().max()) <= 1e-6       # (float atomics of the numerator's scatter)
        assert torch.all(st == 0)
        float(torch.randn(1000, device="cuda").sum())     # eager work between the replays


def test_placement_probe_and_fallback_routing():
    """The probe of what the cooperating-workgroup kernels rely on (all workgroups resident at once,
    workgroup i on XCD i mod 8) passes on this chip, the binding has run it, and the library routes by
    its result: with the one-workgroup kernels forced the same inputs still give the oracle's values."""
    announce("placement probe")
    assert lb.verify_placement() is True
    assert lb._placement[torch.cuda.current_device()] is True
    cx = lb.context(256, 1)
    wt = lb.LastWeights(lb.WEIGHTS_DENSE, 16, 500, 0x1000, None, None, None, 0)
    assert lb.load_library().last_kernel_variant(wt, cx, lb.OP_ARC_POSTERIORS) == 1
    c = workloads.config(0)
    w, lengths = dev(c["w"]), dev(c["lengths"])
    _, want = oracle.forward(c["w"], c["lengths"], 1)
    dist = lb.last_shortest_distance(w, lengths, order=1)
    with library_option(lb.OPT_FORCE_SOLO, 1):
        dist_solo = lb.last_shortest_distance(w, lengths, order=1)
    torch.cuda.synchronize()
    assert_dist_close(dist.cpu().numpy(), want)
    assert_dist_close(dist_solo.cpu().numpy(), want)
