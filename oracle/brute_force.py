"""TEST INFRASTRUCTURE -- not part of the product path.

The definitions of Section 2.3 of arXiv 2304.13134 written out literally for
tiny lattices: enumerate every accepting path of the recognition lattice,
(+)-sum the path weights for the shortest distance D, apply Eq. 1 path by path
for the arc marginals, take the arg max for the shortest path.

The context state is tracked as the tuple of the last n labels (what "the
states encode the output history" means, Section 3) and only then mapped to
an index, so this module checks the closed-form next-state arithmetic used
elsewhere rather than repeating it.  Because the context dependency is
deterministic and accepts every string, each label sequence in
{0..V}^T (0 = empty label) is exactly one accepting path of the frame
dependent lattice (Figure 1b: one arc per frame).
"""
from __future__ import annotations

import itertools

import numpy as np


def history_index(h: tuple, V: int) -> int:
    """Index of the context state whose history is the tuple ``h``."""
    if len(h) == 0:
        return 0
    if len(h) == 1:
        return h[0]
    a, b = h
    return 1 + V + (a - 1) * V + (b - 1)


def enumerate_paths(w_item: np.ndarray, order: int):
    """All accepting paths of one item's lattice.

    w_item: [T, C, V+1].  Returns (labels [P,T], states [P,T+1], scores [P])
    in float64, P = (V+1)^T."""
    T, C, V1 = w_item.shape
    V = V1 - 1
    w = w_item.astype(np.float64)
    labels, states, scores = [], [], []
    for seq in itertools.product(range(V1), repeat=T):
        h = ()
        st = [0]
        s = 0.0
        for t, y in enumerate(seq):
            q = history_index(h, V)
            s += w[t, q, y]
            if y != 0:
                h = (h + (y,))[-order:]
            st.append(history_index(h, V))
        labels.append(seq)
        states.append(st)
        scores.append(s)
    return (np.array(labels, dtype=np.int64).reshape(-1, T),
            np.array(states, dtype=np.int64).reshape(-1, T + 1),
            np.array(scores, dtype=np.float64))


def history_table(V: int, order: int):
    """The full n-gram context dependency of any order as an explicit automaton (Section 3): the
    states are the label histories of length < order ... = order in order of length, then
    lexicographically; returns (table [C, V] with table[q, y-1] = state after label y, histories)."""
    hist = [()]
    for n in range(1, order + 1):
        hist += list(itertools.product(range(1, V + 1), repeat=n))
    index = {h: i for i, h in enumerate(hist)}
    table = np.zeros((len(hist), V), dtype=np.int32)
    for h, i in index.items():
        for y in range(1, V + 1):
            table[i, y - 1] = index[(h + (y,))[-order:]]
    return table, hist


def enumerate_paths_table(w_item: np.ndarray, table: np.ndarray):
    """All accepting paths when the context dependency is an explicit automaton: table[q, y-1] is
    the state after label y in state q, label 0 (empty) keeps the state."""
    T, C, V1 = w_item.shape
    w = w_item.astype(np.float64)
    labels, states, scores = [], [], []
    for seq in itertools.product(range(V1), repeat=T):
        q = 0
        st = [0]
        s = 0.0
        for t, y in enumerate(seq):
            s += w[t, q, y]
            if y != 0:
                q = int(table[q, y - 1])
            st.append(q)
        labels.append(seq)
        states.append(st)
        scores.append(s)
    return (np.array(labels, dtype=np.int64).reshape(-1, T),
            np.array(states, dtype=np.int64).reshape(-1, T + 1),
            np.array(scores, dtype=np.float64))


def log_sum(scores: np.ndarray) -> float:
    if scores.size == 0:
        return -np.inf
    m = scores.max()
    if np.isneginf(m):
        return -np.inf
    return float(m + np.log(np.sum(np.exp(scores - m))))


def arc_marginals(labels, states, scores, shape):
    """Eq. 1: for each arc, the sum over the paths through it of exp(w(path) - D)."""
    T, C, V1 = shape
    D = log_sum(scores)
    g = np.zeros(shape, dtype=np.float64)
    p = np.exp(scores - D)
    for t in range(T):
        np.add.at(g[t], (states[:, t], labels[:, t]), p)
    return D, g


def best_path(labels, states, scores):
    i = int(np.argmax(scores))
    return labels[i], states[i], float(scores[i])


def output_string(seq) -> tuple:
    return tuple(int(y) for y in seq if y != 0)


def restrict_to_reference(labels, states, scores, ref):
    """Paths of the intersection with the reference string ``ref`` (labels 1..V)."""
    ref = tuple(int(r) for r in ref)
    keep = np.array([output_string(s) == ref for s in labels], dtype=bool)
    return labels[keep], states[keep], scores[keep]
