"""CPU oracle of chunk generation by weighted label propagation (Section 4.1 of the paper).

TEST INFRASTRUCTURE ONLY: plain Python loops over NumPy arrays, integer arithmetic.  Nothing in
the product path may import this module.

The super-graph: one vertex x = t*N + i per (snapshot t, vertex i); the spatial edges of every
snapshot (self-loops of the CSR dropped) with weight w_s; a virtual temporal edge between (t, i)
and (t+1, i) for every t with weight w_t.  The weights stand for the traffic an edge causes in the
DGNN at hand (e.g. 2 and 1 for two structure layers and one time layer); they are integers here
so that sums do not depend on their order.

The paper fixes: the initial labels (all different, c(v_{i,t}) = sum of the earlier snapshots' sizes
+ i), the score of a label at a vertex (total weight of the edges to the neighbours that carry
it), the update (the label with the largest score), the end (no label changes) and a size limit
that holds labels back when they are attached to too many vertices.  It does not fix how the
updates of one iteration interleave, how ties are broken, nor how the limit is applied; decided
here, so that the procedure is deterministic, parallel and certain to end:
  * an iteration reads only the labels of the iteration before;
  * the candidate of a vertex is the admissible neighbour label with the largest score, ties to
    the label that fewer vertices carried when the iteration started, then to the smaller label
    (at the start all scores tie; preferring the smaller chunk keeps one label from spreading over
    a single edge into a region that has not formed its own chunks yet); a label is admissible if
    fewer than `cap` vertices carried it when the iteration started (the limit is soft: several
    vertices may take the same label in one iteration);
  * a vertex wants to change only if its candidate scores strictly more than its own label does;
  * of two adjacent vertices that both want to change, only the one that comes first in the
    iteration's order does (so no two neighbours change in the same iteration, every change raises
    the total weight of the edges inside chunks, and the procedure ends); the order of iteration r
    (0-based) is by h(x xor (r * 0x9E3779B9 mod 2^32)), then by x, with h a fixed 32-bit mixing
    function - an order by index alone makes long chains of vertices that wait for each other;
  * it stops when nobody wants to change, or after `max_iters` iterations.
"""
from __future__ import annotations

import numpy as np


def initial_labels(T: int, N: int) -> np.ndarray:
    """c(v_{i,t}) with every snapshot holding the same N vertices, 0-based."""
    return (np.arange(T, dtype=np.int64)[:, None] * N + np.arange(N, dtype=np.int64)[None, :]).reshape(-1)


def neighbours(graph, x: int, w_s: int, w_t: int) -> list:
    """[(neighbour, weight)] of super-vertex x."""
    N, T = graph.N, graph.T
    t, i = divmod(x, N)
    sn = graph.snaps[t]
    out = [(t * N + int(j), w_s) for j in sn.col[sn.rowptr[i]:sn.rowptr[i + 1]] if j != i]
    if t > 0:
        out.append(((t - 1) * N + i, w_t))
    if t + 1 < T:
        out.append(((t + 1) * N + i, w_t))
    return out


def _h(v: int) -> int:
    """32-bit mixing function (xor-shift-multiply), a bijection."""
    v &= 0xFFFFFFFF
    v ^= v >> 16
    v = (v * 0x7FEB352D) & 0xFFFFFFFF
    v ^= v >> 15
    v = (v * 0x846CA68B) & 0xFFFFFFFF
    v ^= v >> 16
    return v


def order_key(x: int, r: int) -> tuple:
    """Position of vertex x in the order of iteration r."""
    return (_h(x ^ ((r * 0x9E3779B9) & 0xFFFFFFFF)), x)


def _scores(graph, labels, x, w_s, w_t) -> dict:
    sc = {}
    for u, w in neighbours(graph, x, w_s, w_t):
        if w > 0:
            sc[int(labels[u])] = sc.get(int(labels[u]), 0) + w
    return sc


def iteration(graph, labels: np.ndarray, w_s: int, w_t: int, cap: int, r: int = 0):
    """Iteration r.  Returns (new labels, number of vertices that changed)."""
    n = labels.size
    size = np.bincount(labels, minlength=n)
    want = np.full(n, -1, np.int64)
    for x in range(n):
        sc = _scores(graph, labels, x, w_s, w_t)
        own = sc.get(int(labels[x]), 0)
        best = None
        for c, s in sc.items():
            if c == labels[x] or size[c] >= cap:
                continue
            key = (s, -int(size[c]), -c)
            if best is None or key > best:
                best = key
        if best is not None and best[0] > own:
            want[x] = -best[2]
    new = labels.copy()
    changed = 0
    for x in range(n):
        if want[x] < 0:
            continue
        if all(not (want[u] >= 0 and order_key(u, r) < order_key(x, r)) for u, w in neighbours(graph, x, w_s, w_t)):
            new[x] = want[x]
            changed += 1
    return new, changed


def propagate(graph, w_s: int, w_t: int, cap: int, max_iters: int) -> dict:
    """Labels after label propagation.  Returns labels int64 [T*N], iterations run, converged."""
    labels = initial_labels(graph.T, graph.N)
    it = 0
    converged = False
    while it < max_iters:
        labels, changed = iteration(graph, labels, w_s, w_t, cap, it)
        it += 1
        if changed == 0:
            converged = True
            break
    return {"labels": labels, "iterations": it, "converged": converged}


def inside_weight(graph, labels: np.ndarray, w_s: int, w_t: int) -> int:
    """Total weight of the edges whose two ends carry the same label (each edge once): the
    quantity the paper maximises in place of minimising the weight between chunks."""
    tot = 0
    for x in range(labels.size):
        for u, w in neighbours(graph, x, w_s, w_t):
            if u > x and labels[u] == labels[x]:
                tot += w
    return tot


def total_weight(graph, w_s: int, w_t: int) -> int:
    n = graph.T * graph.N
    return sum(w for x in range(n) for u, w in neighbours(graph, x, w_s, w_t) if u > x)
