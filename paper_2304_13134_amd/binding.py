"""Thin ctypes binding of the C-ABI library declared in ``include/last.h``.

Argument marshalling only: every step of the computation runs in the HIP
kernels.  PyTorch supplies device memory and the current stream, nothing else.
There is no CPU fallback: if ``liblast_hip.so`` has not been built
(``python -m paper_2304_13134_amd.build``) the first call raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# LAST_HIP_LIB selects another build of the same library (e.g. one compiled with other tuning macros)
LIB_PATH = os.environ.get("LAST_HIP_LIB") or os.path.join(_HERE, "liblast_hip.so")

LAST_LOG, LAST_TROPICAL = 0, 1
OP_SHORTEST_DISTANCE, OP_ARC_POSTERIORS, OP_INTERSECT_REFERENCE, OP_SHORTEST_PATH = 0, 1, 2, 3
OP_LOCAL_LOG_LIKELIHOOD = 4
OP_LOSS = 5
WEIGHTS_DENSE, WEIGHTS_SHARED_EMB = 0, 1

EXPORTS = ["last_workspace_bytes", "last_shortest_distance", "last_arc_posteriors",
           "last_intersect_reference", "last_shortest_path", "last_status_string",
           "last_version", "last_kernel_variant", "last_hip_error_string",
           "last_shortest_distance_static", "last_set_option", "last_get_option",
           "last_local_log_likelihood", "last_probe_bandwidth", "last_globally_normalized_loss",
           "last_verify_placement"]
PROBE_READ, PROBE_COPY, PROBE_READ_ROWS, PROBE_READ_COLUMNS = 0, 1, 2, 3
OPT_FORCE_SOLO, OPT_CLUSTER_GENERATION, OPT_CLUSTER_VITERBI, OPT_SPIN_LIMIT, OPT_FUSED_FRAMES_PER_TILE = 0, 1, 2, 3, 4
OPT_FUSED_KEEP_MARGINALS = 5
STATIC_SCRATCH_BYTES = 32 << 20


class LastContext(ctypes.Structure):
    _fields_ = [("vocab", ctypes.c_int32), ("order", ctypes.c_int32),
                ("num_states", ctypes.c_int32), ("next_table", ctypes.c_void_p)]


class LastWeights(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("B", ctypes.c_int32), ("T", ctypes.c_int32),
                ("w", ctypes.c_void_p), ("f", ctypes.c_void_p), ("e", ctypes.c_void_p),
                ("W", ctypes.c_void_p), ("hidden", ctypes.c_int32)]


class LastGrads(ctypes.Structure):
    _fields_ = [("dw", ctypes.c_void_p), ("df", ctypes.c_void_p), ("de", ctypes.c_void_p),
                ("dW", ctypes.c_void_p), ("accumulate", ctypes.c_int32),
                ("scale", ctypes.c_float)]


class LastError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("liblast_hip: status %d (%s)" % (code, text))
        self.code = code


_lib = None


def load_library():
    """Load liblast_hip.so (no GPU needed to load it) and set the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("liblast_hip.so is not built; run `python -m paper_2304_13134_amd.build` "
                           "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.last_workspace_bytes.restype = sz
    lib.last_workspace_bytes.argtypes = [ctypes.POINTER(LastWeights), ctypes.POINTER(LastContext), i32, i32]
    lib.last_shortest_distance.restype = i32
    lib.last_shortest_distance.argtypes = [ctypes.POINTER(LastWeights), vp, ctypes.POINTER(LastContext),
                                           i32, vp, vp, vp, sz, vp]
    lib.last_shortest_distance_static.restype = i32
    lib.last_shortest_distance_static.argtypes = [ctypes.POINTER(LastWeights), vp, ctypes.POINTER(LastContext),
                                                  i32, vp, vp, vp]
    lib.last_arc_posteriors.restype = i32
    lib.last_arc_posteriors.argtypes = [ctypes.POINTER(LastWeights), vp, ctypes.POINTER(LastContext),
                                        vp, ctypes.POINTER(LastGrads), vp, vp, sz, vp]
    lib.last_intersect_reference.restype = i32
    lib.last_intersect_reference.argtypes = [ctypes.POINTER(LastWeights), vp, ctypes.POINTER(LastContext),
                                             vp, vp, i32, vp, ctypes.POINTER(LastGrads), vp, vp, sz, vp]
    lib.last_local_log_likelihood.restype = i32
    lib.last_local_log_likelihood.argtypes = lib.last_intersect_reference.argtypes
    lib.last_globally_normalized_loss.restype = i32
    lib.last_globally_normalized_loss.argtypes = [ctypes.POINTER(LastWeights), vp, ctypes.POINTER(LastContext),
                                                  vp, vp, i32, vp, vp, ctypes.POINTER(LastGrads), vp, vp, sz, vp]
    lib.last_shortest_path.restype = i32
    lib.last_shortest_path.argtypes = [ctypes.POINTER(LastWeights), vp, ctypes.POINTER(LastContext),
                                       vp, vp, vp, vp, vp, sz, vp]
    lib.last_probe_bandwidth.restype = i32
    lib.last_probe_bandwidth.argtypes = [i32, vp, vp, sz, vp]
    lib.last_verify_placement.restype = i32
    lib.last_verify_placement.argtypes = [vp, sz, vp]
    lib.last_status_string.restype = ctypes.c_char_p
    lib.last_status_string.argtypes = [i32]
    lib.last_version.restype = i32
    lib.last_hip_error_string.restype = ctypes.c_char_p
    lib.last_set_option.restype = i32
    lib.last_set_option.argtypes = [i32, i32]
    lib.last_get_option.restype = i32
    lib.last_get_option.argtypes = [i32]
    lib.last_kernel_variant.restype = i32
    lib.last_kernel_variant.argtypes = [ctypes.POINTER(LastWeights), ctypes.POINTER(LastContext), i32]
    _lib = lib
    return lib


def _check(code):
    if code != 0:
        text = load_library().last_status_string(code).decode()
        if code == 7:
            text += ": " + load_library().last_hip_error_string().decode()
        raise LastError(code, text)


def set_option(option, value):
    """Process-wide setting of the library (see last_set_option in include/last.h); returns the old value."""
    lib = load_library()
    old = int(lib.last_get_option(option))
    _check(lib.last_set_option(option, value))
    return old


def last_probe_bandwidth(kind, src, dst):
    """Plain read sweep (PROBE_READ; dst is any device tensor of >= 16 bytes) or copy (PROBE_COPY) of
    the bytes of `src`: the streaming yardstick of the benchmark."""
    nbytes = src.numel() * src.element_size()
    _check(load_library().last_probe_bandwidth(kind, _ptr(src), _ptr(dst), nbytes, _stream()))


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dev_tensor(t, dtype, name):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous device tensor of dtype %s" % (name, dtype))
    return t


_workspaces = {}
_placement = {}      # device index -> True (cooperating workgroups) / False (one workgroup per item)


def verify_placement(device=None):
    """Run the library's placement probe on `device` (default: the current one) and return whether the
    cooperating-workgroup kernels will be used there; waits for the device."""
    index = torch.cuda.current_device() if device is None else (torch.device(device).index or 0)
    with torch.cuda.device(index):
        buf = torch.empty(2048, dtype=torch.uint8, device="cuda")
        code = load_library().last_verify_placement(_ptr(buf), buf.numel(), _stream())
    if code not in (0, 6):          # LAST_OK / LAST_ERR_UNSUPPORTED
        _check(code)
    _placement[index] = code == 0
    return _placement[index]


def workspace(nbytes, device):
    """A cached device scratch buffer (grown on demand, 256-byte aligned by the allocator), one per
    device and stream: calls enqueued on different streams may overlap and must not share scratch."""
    index = torch.device(device).index or 0
    if index not in _placement and not torch.cuda.is_current_stream_capturing():
        verify_placement(index)     # once per device, before the first kernel that relies on it
    key = (index, torch.cuda.current_stream().cuda_stream)
    buf = _workspaces.get(key)
    if buf is None or buf.numel() < nbytes:
        buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        _workspaces[key] = buf
    return buf


def context(V, order):
    """order: 1 or 2 (full n-gram in closed form), or a device int32 tensor [C, V], the next-state
    table of any deterministic automaton (table[q, y-1] = state after label y; start state 0)."""
    if isinstance(order, torch.Tensor):
        _dev_tensor(order, torch.int32, "next_table")
        if order.dim() != 2 or order.shape[1] != V:
            raise ValueError("next_table must be [C, V]")
        return LastContext(V, 0, order.shape[0], order.data_ptr())
    C = 1 + V if order == 1 else 1 + V + V * V
    return LastContext(V, order, C, None)


# item_status of the most recent call that was not given one (device int32 [B])
last_item_status = None


def _status(item_status, B, device):
    """Every call gets an item_status array, so that data-dependent failures are never silent."""
    global last_item_status
    if item_status is None:
        item_status = torch.empty(B, dtype=torch.int32, device=device)
        last_item_status = item_status
    return _dev_tensor(item_status, torch.int32, "item_status")


def check_item_status(item_status=None):
    """Synchronises and raises if any item of the call reported a problem (see include/last.h)."""
    st = last_item_status if item_status is None else item_status
    if st is not None:
        bad = torch.nonzero(st).flatten().tolist()
        if bad:
            raise LastError(100 + int(st[bad[0]]), "item_status %d on items %s" % (int(st[bad[0]]), bad[:8]))


def dense_weights(w):
    _dev_tensor(w, torch.float32, "w")
    B, T, C, V1 = w.shape
    return LastWeights(WEIGHTS_DENSE, B, T, w.data_ptr(), None, None, None, 0)


def shared_emb_weights(f, e, W):
    for t, n in ((f, "f"), (e, "e"), (W, "W")):
        _dev_tensor(t, torch.bfloat16, n)
    B, T, H = f.shape
    return LastWeights(WEIGHTS_SHARED_EMB, B, T, None, f.data_ptr(), e.data_ptr(), W.data_ptr(), H)


class SharedEmb(tuple):
    """Inputs of the on-the-fly weight function: (f [B,T,H], e [C,H], W [H,V+1]), bfloat16."""

    def __new__(cls, f, e, W):
        return super().__new__(cls, (f, e, W))


def _weights_and_context(w, order):
    """(LastWeights, LastContext, device, B) for a dense tensor or a SharedEmb triple."""
    if isinstance(w, SharedEmb):
        f, e, W = w
        wt = shared_emb_weights(f, e, W)
        V = W.shape[1] - 1
        cx = context(V, order)
        if cx.num_states != e.shape[0] or e.shape[1] != f.shape[2] or W.shape[0] != f.shape[2]:
            raise ValueError("f, e, W do not match the context dependency")
        return wt, cx, f.device, f.shape[0]
    return dense_weights(w), _dense_ctx(w, order), w.device, w.shape[0]


def _dense_ctx(w, order):
    V = w.shape[3] - 1
    cx = context(V, order)
    if cx.num_states != w.shape[2]:
        raise ValueError("w.shape[2] does not match the context dependency")
    return cx


def last_workspace_bytes(weights, cx, op, Umax=0):
    return int(load_library().last_workspace_bytes(ctypes.byref(weights), ctypes.byref(cx), op, Umax))


def last_kernel_variant(weights, cx, op):
    return int(load_library().last_kernel_variant(ctypes.byref(weights), ctypes.byref(cx), op))


def last_shortest_distance(w, lengths, order=1, semiring="log", item_status=None):
    """dist [B] float32 (device).  semiring: "log" or "tropical"."""
    lib = load_library()
    wt, cx, device, B = _weights_and_context(w, order)
    _dev_tensor(lengths, torch.int32, "lengths")
    dist = torch.empty(B, dtype=torch.float32, device=device)
    item_status = _status(item_status, B, device)
    nbytes = last_workspace_bytes(wt, cx, OP_SHORTEST_DISTANCE)
    if nbytes == 0:
        raise LastError(6, "combination not supported")
    ws = workspace(nbytes, device)
    sr = LAST_LOG if semiring == "log" else LAST_TROPICAL
    _check(lib.last_shortest_distance(ctypes.byref(wt), _ptr(lengths), ctypes.byref(cx), sr,
                                      _ptr(dist), _ptr(item_status), _ptr(ws), ws.numel(), _stream()))
    return dist


def last_shortest_distance_static(w, lengths, dist, order=1, semiring="log", item_status=None):
    """last_shortest_distance into the caller's `dist` [B] with the library's static scratch array:
    nothing is allocated, here or in the library."""
    lib = load_library()
    wt, cx, device, B = _weights_and_context(w, order)
    _dev_tensor(lengths, torch.int32, "lengths")
    _dev_tensor(dist, torch.float32, "dist")
    sr = LAST_LOG if semiring == "log" else LAST_TROPICAL
    _check(lib.last_shortest_distance_static(ctypes.byref(wt), _ptr(lengths), ctypes.byref(cx), sr,
                                             _ptr(dist), _ptr(item_status), _stream()))
    return dist


def last_arc_posteriors(w, lengths, order=1, dw=None, scale=1.0, accumulate=False,
                        item_status=None):
    """Dense weights: (dist [B], dw [B,T,C,V+1]) on the device; dw = scale * arc marginals.
    SharedEmb weights: (dist [B], (df [B,T,H], de [C,H], dW [H,V+1])), float32, the chain of
    the marginals through the weight function; `dw` may be such a triple to write into."""
    lib = load_library()
    wt, cx, device, B = _weights_and_context(w, order)
    _dev_tensor(lengths, torch.int32, "lengths")
    dist = torch.empty(B, dtype=torch.float32, device=device)
    if isinstance(w, SharedEmb):
        f, e, W = w
        if dw is None:
            dw = tuple(torch.empty(t.shape, dtype=torch.float32, device=device) for t in (f, e, W))
        for t, n in zip(dw, ("df", "de", "dW")):
            _dev_tensor(t, torch.float32, n)
        g = LastGrads(None, dw[0].data_ptr(), dw[1].data_ptr(), dw[2].data_ptr(),
                      int(bool(accumulate)), float(scale))
    else:
        if dw is None:
            dw = torch.empty_like(w)
        _dev_tensor(dw, torch.float32, "dw")
        g = LastGrads(dw.data_ptr(), None, None, None, int(bool(accumulate)), float(scale))
    item_status = _status(item_status, B, device)
    nbytes = last_workspace_bytes(wt, cx, OP_ARC_POSTERIORS)
    if nbytes == 0:
        raise LastError(6, "combination not supported")
    ws = workspace(nbytes, device)
    _check(lib.last_arc_posteriors(ctypes.byref(wt), _ptr(lengths), ctypes.byref(cx), _ptr(dist),
                                   ctypes.byref(g), _ptr(item_status), _ptr(ws), ws.numel(),
                                   _stream()))
    return dist, dw


def _intersect(entry, op, w, lengths, refs, ref_lengths, order, dw, scale, accumulate, item_status):
    lib = load_library()
    wt, cx, device, B = _weights_and_context(w, order)
    _dev_tensor(lengths, torch.int32, "lengths")
    _dev_tensor(refs, torch.int32, "refs")
    _dev_tensor(ref_lengths, torch.int32, "ref_lengths")
    Umax = refs.shape[1]
    num = torch.empty(B, dtype=torch.float32, device=device)
    item_status = _status(item_status, B, device)
    g = None
    if dw is not None and isinstance(w, SharedEmb):
        for t, n in zip(dw, ("df", "de", "dW")):
            _dev_tensor(t, torch.float32, n)
        g = LastGrads(None, dw[0].data_ptr(), dw[1].data_ptr(), dw[2].data_ptr(),
                      int(bool(accumulate)), float(scale))
    elif dw is not None:
        _dev_tensor(dw, torch.float32, "dw")
        g = LastGrads(dw.data_ptr(), None, None, None, int(bool(accumulate)), float(scale))
    nbytes = last_workspace_bytes(wt, cx, op, Umax)
    if nbytes == 0:
        raise LastError(6, "combination not supported")
    ws = workspace(nbytes, device)
    _check(getattr(lib, entry)(ctypes.byref(wt), _ptr(lengths), ctypes.byref(cx),
                               _ptr(refs), _ptr(ref_lengths), Umax, _ptr(num),
                               ctypes.byref(g) if g is not None else None,
                               _ptr(item_status), _ptr(ws), ws.numel(), _stream()))
    return num


def last_intersect_reference(w, lengths, refs, ref_lengths, order=1, dw=None, scale=-1.0,
                             accumulate=True, item_status=None):
    """numerator [B] float32; if dw is given, scale * (marginals of the
    intersected lattice) is added to (accumulate) or written over dw.  With SharedEmb weights only
    the arcs of the intersected lattice are evaluated and dw is the triple (df, de, dW)."""
    return _intersect("last_intersect_reference", OP_INTERSECT_REFERENCE, w, lengths, refs, ref_lengths,
                      order, dw, scale, accumulate, item_status)


def last_globally_normalized_loss(w, lengths, refs, ref_lengths, order=1, dw=None, scale=1.0,
                                  accumulate=False, item_status=None):
    """(dist [B], numerator [B], dw): the globally normalised loss dist - numerator of every item and
    dw (+)= scale * its gradient (dense: a tensor like w; SharedEmb: the triple (df, de, dW)), in one
    call; the numerator's recursion runs beside the denominator."""
    lib = load_library()
    wt, cx, device, B = _weights_and_context(w, order)
    _dev_tensor(lengths, torch.int32, "lengths")
    _dev_tensor(refs, torch.int32, "refs")
    _dev_tensor(ref_lengths, torch.int32, "ref_lengths")
    Umax = refs.shape[1]
    dist = torch.empty(B, dtype=torch.float32, device=device)
    num = torch.empty(B, dtype=torch.float32, device=device)
    item_status = _status(item_status, B, device)
    if isinstance(w, SharedEmb):
        if dw is None:
            dw = tuple(torch.empty(t.shape, dtype=torch.float32, device=device) for t in w)
        for t, n in zip(dw, ("df", "de", "dW")):
            _dev_tensor(t, torch.float32, n)
        g = LastGrads(None, dw[0].data_ptr(), dw[1].data_ptr(), dw[2].data_ptr(),
                      int(bool(accumulate)), float(scale))
    else:
        if dw is None:
            dw = torch.empty_like(w)
        _dev_tensor(dw, torch.float32, "dw")
        g = LastGrads(dw.data_ptr(), None, None, None, int(bool(accumulate)), float(scale))
    nbytes = last_workspace_bytes(wt, cx, OP_LOSS, Umax)
    if nbytes == 0:
        raise LastError(6, "combination not supported")
    ws = workspace(nbytes, device)
    _check(lib.last_globally_normalized_loss(ctypes.byref(wt), _ptr(lengths), ctypes.byref(cx), _ptr(refs),
                                             _ptr(ref_lengths), Umax, _ptr(dist), _ptr(num), ctypes.byref(g),
                                             _ptr(item_status), _ptr(ws), ws.numel(), _stream()))
    return dist, num, dw


def last_local_log_likelihood(w, lengths, refs, ref_lengths, order=1, dw=None, scale=1.0,
                              accumulate=False, item_status=None):
    """Log-likelihood [B] float32 of the references under the locally normalised model on the same
    lattice; if dw is given, scale * d loglik / d w is written over (or added to) it."""
    return _intersect("last_local_log_likelihood", OP_LOCAL_LOG_LIKELIHOOD, w, lengths, refs, ref_lengths,
                      order, dw, scale, accumulate, item_status)


def last_shortest_path(w, lengths, order=1, item_status=None):
    """(labels [B,T] int32, states [B,T+1] int32, score [B] float32) on the device."""
    lib = load_library()
    wt, cx = dense_weights(w), _dense_ctx(w, order)
    _dev_tensor(lengths, torch.int32, "lengths")
    B, T = w.shape[0], w.shape[1]
    labels = torch.empty((B, T), dtype=torch.int32, device=w.device)
    states = torch.empty((B, T + 1), dtype=torch.int32, device=w.device)
    score = torch.empty(B, dtype=torch.float32, device=w.device)
    item_status = _status(item_status, B, w.device)
    nbytes = last_workspace_bytes(wt, cx, OP_SHORTEST_PATH)
    if nbytes == 0:
        raise LastError(6, "combination not supported")
    ws = workspace(nbytes, w.device)
    _check(lib.last_shortest_path(ctypes.byref(wt), _ptr(lengths), ctypes.byref(cx), _ptr(labels),
                                  _ptr(states), _ptr(score), _ptr(item_status), _ptr(ws),
                                  ws.numel(), _stream()))
    return labels, states, score
