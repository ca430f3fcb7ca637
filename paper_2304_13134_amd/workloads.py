"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU oracle.

This module holds none of the method's arithmetic: it only draws random
arrays with the shapes and value distributions of the benchmark configurations
(complete recognition lattices with dense or on-the-fly arc weights, reference
label strings, per-item lengths).  Both the HIP path and the oracle consume
exactly these arrays; neither side generates inputs on its own.

Recipe: ``rng = numpy.random.default_rng(2304_13134 * 10 + k)`` for
configuration ``k``; draws are made in the order lengths, weights (or f, e, W),
reference lengths, references.  The second parameter of every normal
distribution is a standard deviation.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 2304_13134 * 10


def num_states(V: int, order: int) -> int:
    return 1 + V if order == 1 else 1 + V + V * V


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) >> 16
    return u.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def random_table(C, V, seed=0):
    """A random deterministic automaton over V labels that accepts every string: table [C, V]
    int32, table[q, y-1] = state after label y.  Every state is made reachable from state 0."""
    rng = np.random.default_rng(seed)
    table = rng.integers(0, C, size=(C, V)).astype(np.int32)
    used = set()
    for q in range(1, C):          # a spanning tree of label arcs keeps every state reachable
        slot = (int(rng.integers(0, q)), int(rng.integers(0, V)))
        if slot in used:           # state q-1 has given away no arc yet
            slot = (q - 1, slot[1])
        used.add(slot)
        table[slot] = q
    return table


def dense(B, T, V, order=1, sigma=1.0, len_lo=None, len_hi=None, seed=0, pad_nan=False, C=None):
    """Dense weights [B,T,C,V+1] ~ sigma*N(0,1) with per-item lengths (C given: table contexts)."""
    rng = np.random.default_rng(seed)
    if C is None:
        C = num_states(V, order)
    if len_lo is None:
        lengths = np.full((B,), T, dtype=np.int32)
    else:
        lengths = rng.integers(len_lo, len_hi + 1, size=B).astype(np.int32)
    w = rng.standard_normal((B, T, C, V + 1), dtype=np.float32)
    if sigma != 1.0:
        w *= np.float32(sigma)
    if pad_nan:
        for b in range(B):
            w[b, lengths[b]:] = np.nan
    return dict(w=w, lengths=lengths, B=B, T=T, V=V, C=C, order=order)


def references(rng, B, V, Umax, u_lo, u_hi):
    ulen = rng.integers(u_lo, u_hi + 1, size=B).astype(np.int32)
    refs = rng.integers(1, V + 1, size=(B, Umax)).astype(np.int32)
    return refs, ulen


def config(k: int, **over):
    """The five benchmark configurations (0-indexed) and, as number 5, the paper's Table 2 shape.  Keyword overrides shrink
    a configuration for parity tests while keeping its structure."""
    seed = SEED_BASE + k
    if k == 0:
        p = dict(B=1, T=8, V=3, order=1, sigma=1.0)
        p.update(over)
        return dense(seed=seed, **p)
    if k == 1:
        p = dict(B=8, T=200, V=32, order=1, sigma=1.0, len_lo=150, len_hi=200)
        p.update(over)
        return dense(seed=seed, **p)
    if k == 2:
        p = dict(B=16, T=500, V=256, order=1, sigma=2.0)
        p.update(over)
        return dense(seed=seed, **p)
    if k == 3:
        p = dict(B=16, T=500, V=256, order=1, sigma=2.0)
        u = dict(Umax=150, u_lo=50, u_hi=150)
        for key in list(over):
            if key in u:
                u[key] = over.pop(key)
        p.update(over)
        d = dense(seed=seed, **p)
        rng = np.random.default_rng(seed + 1000)
        d["refs"], d["ref_lengths"] = references(rng, p["B"], p["V"], **u)
        d["Umax"] = u["Umax"]
        return d
    if k == 4:
        p = dict(B=4, T=1000, V=64, order=2, H=512)
        p.update(over)
        return shared_emb(seed=seed, **p)
    if k == 5:
        # the shape of the paper's own benchmark (Table 2): 32 labels, context size 2 (1057 states),
        # 512 hidden units, batch 16, 1024 frames, 256 output labels; inputs as in configuration 4
        p = dict(B=16, T=1024, V=32, order=2, H=512)
        U = over.pop("U", 256)
        p.update(over)
        d = shared_emb(seed=seed, **p)
        rng = np.random.default_rng(seed + 1000)
        d["refs"], d["ref_lengths"] = references(rng, p["B"], p["V"], U, U, U)
        d["Umax"] = U
        return d
    raise ValueError("unknown configuration %r" % (k,))


def shared_emb(B, T, V, order=2, H=512, seed=0, len_lo=None, len_hi=None):
    """Inputs of the on-the-fly weight function: frames f ~ N(0,1), context
    embeddings e ~ 0.5*N(0,1), projection W ~ N(0,1)/sqrt(H), all rounded to
    bfloat16 and returned as uint16 bit patterns."""
    rng = np.random.default_rng(seed)
    C = num_states(V, order)
    if len_lo is None:
        lengths = np.full((B,), T, dtype=np.int32)
    else:
        lengths = rng.integers(len_lo, len_hi + 1, size=B).astype(np.int32)
    f = rng.standard_normal((B, T, H), dtype=np.float32)
    e = rng.standard_normal((C, H), dtype=np.float32) * np.float32(0.5)
    W = rng.standard_normal((H, V + 1), dtype=np.float32) / np.float32(np.sqrt(H))
    return dict(f=to_bf16_bits(f), e=to_bf16_bits(e), W=to_bf16_bits(W), lengths=lengths,
                B=B, T=T, V=V, C=C, order=order, H=H)
