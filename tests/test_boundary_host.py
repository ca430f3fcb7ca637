"""Host-only checks of the C-ABI boundary: the library loads without a GPU,
exports every symbol include/last.h declares, and rejects bad arguments before
anything is enqueued."""
import ctypes
import os
import re

import pytest

from paper_2304_13134_amd import binding as lb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lb.LIB_PATH):
        from paper_2304_13134_amd.build import build_library
        build_library()
    return lb.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "last.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(last_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(lb.EXPORTS) == set(names)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    for code in range(8):
        assert len(lib.last_status_string(code)) > 0
    assert lib.last_version() >= 1


def _wt(B=2, T=5, w=0x1000):
    return lb.LastWeights(lb.WEIGHTS_DENSE, B, T, w, None, None, None, 0)


def test_workspace_bytes_and_context_validation(lib):
    cx = lb.context(3, 1)
    wt = _wt()
    n = lb.last_workspace_bytes(wt, cx, lb.OP_ARC_POSTERIORS)
    assert n >= 2 * 6 * 4 * 4 and n % 256 == 0
    assert lb.last_workspace_bytes(wt, cx, lb.OP_SHORTEST_PATH) >= 2 * 5 * 4 * 4
    assert lb.last_workspace_bytes(wt, cx, lb.OP_INTERSECT_REFERENCE, 3) > 0
    assert lb.last_workspace_bytes(wt, cx, 99) == 0
    bad = lb.LastContext(3, 1, 5)
    assert lb.last_workspace_bytes(wt, bad, lb.OP_ARC_POSTERIORS) == 0
    assert lb.context(32, 2).num_states == 1057          # Table 2 of the paper
    assert lb.last_workspace_bytes(_wt(), lb.LastContext(3, 3, 40), 0) == 0


def test_argument_errors_are_reported_before_any_launch(lib):
    cx = lb.context(3, 1)
    wt = _wt()
    vp = ctypes.c_void_p
    dummy = vp(0x2000)
    # null pointers
    assert lib.last_shortest_distance(None, dummy, ctypes.byref(cx), 0, dummy, None, dummy, 1 << 20, None) == 1
    assert lib.last_shortest_distance(ctypes.byref(wt), None, ctypes.byref(cx), 0, dummy, None, dummy, 1 << 20, None) == 1
    nullw = _wt(w=None)
    assert lib.last_shortest_distance(ctypes.byref(nullw), dummy, ctypes.byref(cx), 0, dummy, None, dummy, 1 << 20, None) == 1
    # shape, context, semiring
    assert lib.last_shortest_distance(ctypes.byref(_wt(B=0)), dummy, ctypes.byref(cx), 0, dummy, None, dummy, 1 << 20, None) == 2
    bad = lb.LastContext(3, 1, 7)
    assert lib.last_shortest_distance(ctypes.byref(wt), dummy, ctypes.byref(bad), 0, dummy, None, dummy, 1 << 20, None) == 3
    assert lib.last_shortest_distance(ctypes.byref(wt), dummy, ctypes.byref(cx), 7, dummy, None, dummy, 1 << 20, None) == 4
    # workspace: null, misaligned, too small
    g = lb.LastGrads(0x3000, None, None, None, 0, 1.0)
    assert lib.last_arc_posteriors(ctypes.byref(wt), dummy, ctypes.byref(cx), dummy, ctypes.byref(g), None, None, 1 << 20, None) == 5
    assert lib.last_arc_posteriors(ctypes.byref(wt), dummy, ctypes.byref(cx), dummy, ctypes.byref(g), None, vp(0x2001), 1 << 20, None) == 5
    assert lib.last_arc_posteriors(ctypes.byref(wt), dummy, ctypes.byref(cx), dummy, ctypes.byref(g), None, dummy, 16, None) == 5
    gnull = lb.LastGrads(None, None, None, None, 0, 1.0)
    assert lib.last_arc_posteriors(ctypes.byref(wt), dummy, ctypes.byref(cx), dummy, ctypes.byref(gnull), None, dummy, 1 << 20, None) == 1
    # unsupported weight kind
    unk = lb.LastWeights(9, 2, 5, 0x1000, None, None, None, 0)
    assert lib.last_shortest_path(ctypes.byref(unk), dummy, ctypes.byref(cx), dummy, dummy, dummy, None, dummy, 1 << 20, None) == 6
    assert lib.last_intersect_reference(ctypes.byref(wt), dummy, ctypes.byref(cx), dummy, dummy, -1, dummy, None, None, dummy, 1 << 20, None) == 2


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(TypeError):
        lb.last_shortest_distance(torch.zeros(1, 2, 4, 4), torch.zeros(1, dtype=torch.int32))


def _se(B=4, T=10, H=512):
    return lb.LastWeights(lb.WEIGHTS_SHARED_EMB, B, T, None, 0x1000, 0x2000, 0x3000, H)


def test_shared_embedding_plan_is_checked_on_the_host(lib):
    cx = lb.context(64, 2)
    assert cx.num_states == 4161
    need_d = lb.last_workspace_bytes(_se(), cx, lb.OP_SHORTEST_DISTANCE)
    need_g = lb.last_workspace_bytes(_se(), cx, lb.OP_ARC_POSTERIORS)
    # the gradient pass keeps the forward and backward weights of every state-frame
    assert need_d > 0 and need_g >= need_d + 2 * 4 * 11 * 4161 * 4
    assert lb.last_kernel_variant(_se(), cx, lb.OP_ARC_POSTERIORS) == 2
    # unsupported combinations: hidden size, vocabulary, context size, operation
    assert lb.last_workspace_bytes(_se(H=96), cx, lb.OP_ARC_POSTERIORS) == 0
    assert lb.last_workspace_bytes(_se(H=640), cx, lb.OP_ARC_POSTERIORS) == 0
    assert lb.last_workspace_bytes(_se(), lb.context(65, 2), lb.OP_ARC_POSTERIORS) == 0
    assert lb.last_workspace_bytes(_se(), lb.context(64, 1), lb.OP_ARC_POSTERIORS) == 0
    assert lb.last_workspace_bytes(_se(), cx, lb.OP_SHORTEST_PATH) == 0
    assert lb.last_kernel_variant(_se(H=96), cx, lb.OP_ARC_POSTERIORS) == -1
    vp = ctypes.c_void_p
    dummy = vp(0x4000)
    se, bad = _se(), _se(H=96)
    g = lb.LastGrads(None, 0x5000, 0x6000, 0x7000, 0, 1.0)
    assert lib.last_arc_posteriors(ctypes.byref(bad), dummy, ctypes.byref(cx), dummy, ctypes.byref(g), None,
                                   dummy, 1 << 30, None) == 6
    assert lib.last_shortest_distance(ctypes.byref(se), dummy, ctypes.byref(cx), lb.LAST_TROPICAL, dummy, None,
                                      dummy, 1 << 30, None) == 6
    gnull = lb.LastGrads(None, None, 0x6000, 0x7000, 0, 1.0)
    assert lib.last_arc_posteriors(ctypes.byref(se), dummy, ctypes.byref(cx), dummy, ctypes.byref(gnull), None,
                                   dummy, 1 << 30, None) == 1
    assert lib.last_arc_posteriors(ctypes.byref(se), dummy, ctypes.byref(cx), dummy, ctypes.byref(g), None,
                                   dummy, 4096, None) == 5


def test_table_context_is_checked_on_the_host(lib):
    vp = ctypes.c_void_p
    dummy = vp(0x2000)
    wt = _wt()
    tab = lb.LastContext(3, 0, 40, 0x8000)                 # 40 states, any automaton
    for op in (lb.OP_SHORTEST_DISTANCE, lb.OP_ARC_POSTERIORS, lb.OP_SHORTEST_PATH):
        assert lb.last_workspace_bytes(wt, tab, op) > 0
    assert lb.last_workspace_bytes(wt, tab, lb.OP_LOCAL_LOG_LIKELIHOOD, 5) > \
        lb.last_workspace_bytes(wt, tab, lb.OP_INTERSECT_REFERENCE, 5) > 0
    assert lb.last_kernel_variant(wt, tab, lb.OP_ARC_POSTERIORS) == 0
    # a table context without a table, without states, or with on-the-fly weights
    assert lib.last_shortest_distance(ctypes.byref(wt), dummy, ctypes.byref(lb.LastContext(3, 0, 40, None)), 0,
                                      dummy, None, dummy, 1 << 20, None) == 1
    assert lib.last_shortest_distance(ctypes.byref(wt), dummy, ctypes.byref(lb.LastContext(3, 0, 0, 0x8000)), 0,
                                      dummy, None, dummy, 1 << 20, None) == 3
    assert lb.last_workspace_bytes(_se(), lb.LastContext(64, 0, 4161, 0x8000), lb.OP_ARC_POSTERIORS) == 0
    # more states than the LDS of a compute unit holds
    big = lb.LastContext(3, 0, 20000, 0x8000)
    assert lib.last_shortest_distance(ctypes.byref(wt), dummy, ctypes.byref(big), 0, dummy, None, dummy,
                                      1 << 30, None) == 6
    g = lb.LastGrads(0x3000, None, None, None, 0, 1.0)
    assert lib.last_arc_posteriors(ctypes.byref(wt), dummy, ctypes.byref(big), dummy, ctypes.byref(g), None,
                                   dummy, 1 << 30, None) == 6
    assert lib.last_local_log_likelihood(ctypes.byref(wt), dummy, ctypes.byref(tab), dummy, dummy, -1, dummy,
                                         None, None, dummy, 1 << 20, None) == 2


def test_options_are_validated(lib):
    """last_set_option refuses unknown options and values and leaves the setting as it was."""
    for option, good, bad in [(lb.OPT_CLUSTER_GENERATION, (0, 1, 2, 3), (-1, 4)),
                              (lb.OPT_CLUSTER_VITERBI, (0, 1, 2), (-1, 3)),
                              (lb.OPT_SPIN_LIMIT, (1, 1 << 20), (0, -5)),
                              (lb.OPT_FUSED_FRAMES_PER_TILE, (1, 2), (0, 3)),
                              (lb.OPT_FUSED_KEEP_MARGINALS, (0, 1), (-1, 2))]:
        before = lib.last_get_option(option)
        for v in bad:
            assert lib.last_set_option(option, v) != 0
            assert lib.last_get_option(option) == before
        for v in good:
            assert lib.last_set_option(option, v) == 0
            assert lib.last_get_option(option) == v
        assert lib.last_set_option(option, before) == 0
    assert lib.last_set_option(99, 0) != 0
    assert lib.last_get_option(99) == -1
    assert lib.last_get_option(lb.OPT_FUSED_FRAMES_PER_TILE) == 2     # the default


def test_placement_probe_checks_its_arguments(lib):
    assert lib.last_verify_placement(None, 4096, None) == 1              # LAST_ERR_NULL
    assert lib.last_verify_placement(ctypes.c_void_p(0x1000), 64, None) == 5    # workspace too small
    assert lib.last_verify_placement(ctypes.c_void_p(0x1002), 4096, None) == 5  # misaligned
