"""TEST INFRASTRUCTURE -- not part of the product path.

Float64 CPU oracle for the lattice computations of arXiv 2304.13134 (LAST):
a ctypes front end to ``last_oracle.c`` plus a brute-force path enumerator
(``brute_force.py``).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the HIP library
and its Python binding never do, and this package never imports them.

Each function cites the passage of the paper it follows; the conventions
(label 0 = empty label, state 0 = empty history, all last-frame states final)
are stated at the top of ``last_oracle.c``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "last_oracle.c")
_LIB = os.path.join(_HERE, "liblast_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with the host compiler (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC",
               "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, "bfloat16 tensors are passed as uint16 bit patterns"
    return a


def max_threads() -> int:
    return int(_load().lo_max_threads())


def set_threads(n: int) -> None:
    _load().lo_set_threads(int(n))


def num_states(V: int, order: int) -> int:
    """Number of context states of the full n-gram context dependency (Section 3)."""
    return int(_load().lo_num_states(int(V), int(order)))


def next_state(V: int, order: int, q: int, y: int) -> int:
    """Destination context state of arc (q, y); the empty label y = 0 stays in q."""
    return int(_load().lo_next_state(int(V), int(order), int(q), int(y)))


_table_keepalive = None


def set_next_table(table) -> None:
    """Register a NextStateTable context dependency (Section 3): table [C, V] int32, table[q, y-1] =
    destination of label y out of state q.  Functions called with order = 0 use it."""
    global _table_keepalive
    table = np.ascontiguousarray(table, dtype=np.int32)
    C, V = table.shape
    assert table.min() >= 0 and table.max() < C
    _table_keepalive = table
    _load().lo_set_next_table(_p(table, ctypes.c_int32), int(C), int(V))


def next_state_table(V: int, order: int) -> np.ndarray:
    C = num_states(V, order)
    return np.array([[next_state(V, order, q, y) for y in range(V + 1)] for q in range(C)],
                    dtype=np.int64)


def _dims(w, order):
    w = _f32(w)
    B, T, C, V1 = w.shape
    V = V1 - 1
    assert num_states(V, order) == C, "weights do not match the context dependency"
    return w, B, T, C, V


def forward(w, lengths, order=1):
    """Eq. 2 in the log semiring over the complete lattice: (alpha [B,T+1,C], D [B])."""
    w, B, T, C, V = _dims(w, order)
    lengths = _i32(lengths)
    alpha = np.empty((B, T + 1, C), dtype=np.float64)
    D = np.empty((B,), dtype=np.float64)
    rc = _load().lo_forward(_p(w, ctypes.c_float), _p(lengths, ctypes.c_int32), B, T, V, order,
                            _p(alpha, ctypes.c_double), _p(D, ctypes.c_double))
    assert rc == 0
    return alpha, D


def backward(w, lengths, order=1):
    """Backward weights beta [B,T+1,C] (Section 4.2.2)."""
    w, B, T, C, V = _dims(w, order)
    lengths = _i32(lengths)
    beta = np.empty((B, T + 1, C), dtype=np.float64)
    rc = _load().lo_backward(_p(w, ctypes.c_float), _p(lengths, ctypes.c_int32), B, T, V, order,
                             _p(beta, ctypes.c_double))
    assert rc == 0
    return beta


def posteriors(w, lengths, order=1, alpha=None, beta=None, D=None):
    """Arc marginals of Eq. 1 as a dense float64 tensor [B,T,C,V+1]."""
    w, B, T, C, V = _dims(w, order)
    lengths = _i32(lengths)
    if alpha is None:
        alpha, D = forward(w, lengths, order)
    if beta is None:
        beta = backward(w, lengths, order)
    gamma = np.empty((B, T, C, V + 1), dtype=np.float64)
    rc = _load().lo_posteriors(_p(w, ctypes.c_float), _p(lengths, ctypes.c_int32), B, T, V, order,
                               _p(alpha, ctypes.c_double), _p(beta, ctypes.c_double),
                               _p(D, ctypes.c_double), _p(gamma, ctypes.c_double))
    assert rc == 0
    return gamma


def posterior_samples(w, lengths, order, alpha, beta, D, idx):
    """Eq. 1 evaluated one arc at a time at the rows of ``idx`` = (b, t, q, y)."""
    w = np.asarray(w)
    V = w.shape[3] - 1
    nx = next_state_table(V, order)
    b, t, q, y = (np.asarray(idx[:, i], dtype=np.int64) for i in range(4))
    a = alpha[b, t, q]
    e = a + w[b, t, q, y].astype(np.float64) + beta[b, t + 1, nx[q, y]] - D[b]
    out = np.where(np.isneginf(a), 0.0, np.exp(np.where(np.isneginf(a), 0.0, e)))
    out = np.where(t >= np.asarray(lengths)[b], 0.0, out)
    return out


def numerator(w, lengths, refs, ref_lengths, order=1):
    """Intersection with the reference + shortest distance on it (Section 2.1).

    Returns a dict: N [B], ctx [B,Umax+1], a / b [B,T+1,Umax+1] forward and
    backward weights on the (t,u) grid, pb / pl [B,T,Umax+1] marginals of the
    empty-label arc and of the label arc leaving (t,u)."""
    w, B, T, C, V = _dims(w, order)
    lengths = _i32(lengths)
    refs = _i32(refs)
    ref_lengths = _i32(ref_lengths)
    Umax = refs.shape[1]
    U1 = Umax + 1
    ctx = np.empty((B, U1), dtype=np.int32)
    a = np.empty((B, T + 1, U1), dtype=np.float64)
    bb = np.empty((B, T + 1, U1), dtype=np.float64)
    N = np.empty((B,), dtype=np.float64)
    pb = np.empty((B, T, U1), dtype=np.float64)
    pl = np.empty((B, T, U1), dtype=np.float64)
    rc = _load().lo_numerator(_p(w, ctypes.c_float), _p(lengths, ctypes.c_int32),
                              _p(refs, ctypes.c_int32), _p(ref_lengths, ctypes.c_int32),
                              B, T, V, order, Umax, _p(ctx, ctypes.c_int32),
                              _p(a, ctypes.c_double), _p(bb, ctypes.c_double),
                              _p(N, ctypes.c_double), _p(pb, ctypes.c_double),
                              _p(pl, ctypes.c_double))
    assert rc == 0
    return dict(N=N, ctx=ctx, a=a, b=bb, pb=pb, pl=pl)


def numerator_local(w, lengths, refs, ref_lengths, order=1, grad=True):
    """Locally normalised (RNN-T-style) log-likelihood of the reference on the intersected lattice
    (Section 2.1; Table 1, first row): the numerator recursion on w - logsumexp_y w.  Returns the
    dict of `numerator` plus grad [B,T,C,V+1] = dN/dw."""
    w, B, T, C, V = _dims(w, order)
    lengths = _i32(lengths)
    refs = _i32(refs)
    ref_lengths = _i32(ref_lengths)
    Umax = refs.shape[1]
    U1 = Umax + 1
    ctx = np.empty((B, U1), dtype=np.int32)
    a = np.empty((B, T + 1, U1), dtype=np.float64)
    bb = np.empty((B, T + 1, U1), dtype=np.float64)
    N = np.empty((B,), dtype=np.float64)
    pb = np.empty((B, T, U1), dtype=np.float64)
    pl = np.empty((B, T, U1), dtype=np.float64)
    g = np.empty((B, T, C, V + 1), dtype=np.float64) if grad else None
    rc = _load().lo_numerator_local(_p(w, ctypes.c_float), _p(lengths, ctypes.c_int32),
                                    _p(refs, ctypes.c_int32), _p(ref_lengths, ctypes.c_int32),
                                    B, T, V, order, Umax, _p(ctx, ctypes.c_int32),
                                    _p(a, ctypes.c_double), _p(bb, ctypes.c_double),
                                    _p(N, ctypes.c_double), _p(pb, ctypes.c_double),
                                    _p(pl, ctypes.c_double), _p(g, ctypes.c_double))
    assert rc == 0
    return dict(N=N, ctx=ctx, a=a, b=bb, pb=pb, pl=pl, grad=g)


def numerator_posteriors_dense(num, refs, ref_lengths, shape):
    """Scatter the (t,u) marginals onto the arcs (t, ctx(u), label) they ride on;
    several u may share one arc, their marginals add."""
    B, T, C, V1 = shape
    g = np.zeros(shape, dtype=np.float64)
    refs = np.asarray(refs)
    for b in range(B):
        U = int(ref_lengths[b])
        for u in range(U + 1):
            q = int(num["ctx"][b, u])
            np.add.at(g[b, :, q, 0], np.arange(T), num["pb"][b, :, u])
            if u < U:
                np.add.at(g[b, :, q, int(refs[b, u])], np.arange(T), num["pl"][b, :, u])
    return g


def viterbi(w, lengths, order=1, precision="f32"):
    """Tropical shortest path with arg-max backpointers (Sections 2.1, 4.2.3).

    Returns (labels [B,T], states [B,T+1], score [B]); ties go to the lowest
    flat arc index q*(V+1)+y, then to the lowest final state."""
    w, B, T, C, V = _dims(w, order)
    lengths = _i32(lengths)
    labels = np.empty((B, T), dtype=np.int32)
    states = np.empty((B, T + 1), dtype=np.int32)
    if precision == "f32":
        score = np.empty((B,), dtype=np.float32)
        fn, ct = _load().lo_viterbi_f32, ctypes.c_float
    else:
        score = np.empty((B,), dtype=np.float64)
        fn, ct = _load().lo_viterbi_f64, ctypes.c_double
    rc = fn(_p(w, ctypes.c_float), _p(lengths, ctypes.c_int32), B, T, V, order,
            _p(labels, ctypes.c_int32), _p(states, ctypes.c_int32), _p(score, ct))
    assert rc == 0
    return labels, states, score


def shared_emb_weights(f, e, W, round_h=True):
    """w[b,t,q,:] = tanh(f[b,t] + e[q]) @ W as float64 [B,T,C,V+1] (Table 2's
    shared-embedding weight function; formula from the benchmark definition)."""
    f, e, W = _u16(f), _u16(e), _u16(W)
    B, T, H = f.shape
    C = e.shape[0]
    V1 = W.shape[1]
    out = np.empty((B, T, C, V1), dtype=np.float64)
    rc = _load().lo_shared_emb_weights(_p(f, ctypes.c_uint16), _p(e, ctypes.c_uint16),
                                       _p(W, ctypes.c_uint16), B, T, C, H, V1, int(round_h),
                                       _p(out, ctypes.c_double))
    assert rc == 0
    return out


def fused_forward_backward(f, e, W, lengths, order=2, round_h=True, grads=True):
    """On-the-fly weights (Section 4.1) + forward-backward + chain of Eq. 1
    through the weight function.  Returns dict(D, alpha, df, de, dW)."""
    f, e, W = _u16(f), _u16(e), _u16(W)
    lengths = _i32(lengths)
    B, T, H = f.shape
    C = e.shape[0]
    V = W.shape[1] - 1
    assert num_states(V, order) == C
    alpha = np.empty((B, T + 1, C), dtype=np.float64)
    D = np.empty((B,), dtype=np.float64)
    df = np.empty((B, T, H), dtype=np.float64) if grads else None
    de = np.empty((C, H), dtype=np.float64) if grads else None
    dW = np.empty((H, V + 1), dtype=np.float64) if grads else None
    rc = _load().lo_fused_forward_backward(
        _p(f, ctypes.c_uint16), _p(e, ctypes.c_uint16), _p(W, ctypes.c_uint16),
        _p(lengths, ctypes.c_int32), B, T, V, order, H, int(round_h),
        _p(alpha, ctypes.c_double), _p(D, ctypes.c_double),
        _p(df, ctypes.c_double), _p(de, ctypes.c_double), _p(dW, ctypes.c_double))
    assert rc == 0
    return dict(D=D, alpha=alpha, df=df, de=de, dW=dW)


def fused_numerator(f, e, W, lengths, refs, ref_lengths, order=2, round_h=True, grads=True):
    """Numerator (Section 2.1) on shared-embedding weights computed on the fly (Section 4.1): only the
    two arcs leaving every state (t,u) of the intersected lattice are evaluated.  f [B,T,H], e [C,H],
    W [H,V+1] as bfloat16 bit patterns.  Returns the dict of `numerator` plus df, de, dW (float64):
    the chain of the intersected lattice's arc marginals through the weight function."""
    f, e, W = _u16(f), _u16(e), _u16(W)
    B, T, H = f.shape
    C = e.shape[0]
    V = W.shape[1] - 1
    assert num_states(V, order) == C and e.shape[1] == H and W.shape[0] == H
    lengths, refs, ref_lengths = _i32(lengths), _i32(refs), _i32(ref_lengths)
    Umax = refs.shape[1]
    U1 = Umax + 1
    ctx = np.empty((B, U1), dtype=np.int32)
    a = np.empty((B, T + 1, U1), dtype=np.float64)
    bb = np.empty((B, T + 1, U1), dtype=np.float64)
    N = np.empty((B,), dtype=np.float64)
    pb = np.empty((B, T, U1), dtype=np.float64)
    pl = np.empty((B, T, U1), dtype=np.float64)
    df = np.empty((B, T, H), dtype=np.float64) if grads else None
    de = np.empty((C, H), dtype=np.float64) if grads else None
    dW = np.empty((H, V + 1), dtype=np.float64) if grads else None
    rc = _load().lo_fused_numerator(_p(f, ctypes.c_uint16), _p(e, ctypes.c_uint16), _p(W, ctypes.c_uint16),
                                    _p(lengths, ctypes.c_int32), _p(refs, ctypes.c_int32),
                                    _p(ref_lengths, ctypes.c_int32), B, T, V, order, H, Umax,
                                    int(bool(round_h)), _p(ctx, ctypes.c_int32), _p(a, ctypes.c_double),
                                    _p(bb, ctypes.c_double), _p(N, ctypes.c_double), _p(pb, ctypes.c_double),
                                    _p(pl, ctypes.c_double), _p(df, ctypes.c_double), _p(de, ctypes.c_double),
                                    _p(dW, ctypes.c_double))
    assert rc == 0
    return dict(N=N, ctx=ctx, a=a, b=bb, pb=pb, pl=pl, df=df, de=de, dW=dW)
