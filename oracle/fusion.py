"""CPU oracle of spatial-fusion selection (Section 5.1.1 of the paper) and of the chunk assignment
algorithm (Section 4.2, Algorithm 1).

TEST INFRASTRUCTURE ONLY: Python sets and loops, exact integer / float64 arithmetic.  Nothing in
the product path may import this module.

Definitions (the paper describes both in a paragraph each; the points it leaves open are decided
here and listed with the function they belong to):

  load(a)     the (snapshot, vertex) rows chunk a has to have on the GPU: its own rows and, per
              snapshot of its window, every neighbour of one of its rows outside its vertex range.
  shared(a,b) |load(a) & load(b)|: rows that are loaded twice if a and b are processed one after
              the other and once if they are fused -- the paper's "redundant data loading",
              counted in rows (the bytes are this times the row size, the same for all pairs).
"""
from __future__ import annotations

import numpy as np


def load_sets(graph, chunks) -> list:
    """load(a) for every chunk, as Python sets of (t, v)."""
    out = []
    for v_lo, v_hi, t_lo, t_hi in np.asarray(chunks, np.int64).reshape(-1, 4).tolist():
        rows = set()
        for t in range(t_lo, t_hi):
            sn = graph.snaps[t]
            for v in range(v_lo, v_hi):
                rows.add((t, v))
                for j in sn.col[sn.rowptr[v]:sn.rowptr[v + 1]].tolist():
                    rows.add((t, j))
        out.append(rows)
    return out


def shared_rows(graph, chunks) -> np.ndarray:
    """int64 [n, n], symmetric, zero diagonal."""
    sets = load_sets(graph, chunks)
    n = len(sets)
    S = np.zeros((n, n), np.int64)
    for a in range(n):
        for b in range(a + 1, n):
            S[a, b] = S[b, a] = len(sets[a] & sets[b])
    return S


def select_fusion(shared: np.ndarray, mem: np.ndarray, cap: int) -> np.ndarray:
    """Greedy fusion under a memory cap.  Every chunk starts as its own group.  Repeatedly: among
    all pairs of groups whose memories add up to at most `cap`, take the pair with the largest
    shared amount and fuse it; stop when no pair fits.  Returns group[a] for every chunk, groups
    numbered by their smallest member in ascending order (0, 1, ...).

    Decided here: the shared amount of two groups is the sum of the pairwise figures of their
    members (the estimate is made once, before fusing starts); a group's memory is the sum of its
    members' measured memories; ties go to the pair with the smallest (first, second) group where a
    group is named by its smallest member; pairs that share nothing are still fused while they fit
    (fused chunks also run together, which is the section's second purpose)."""
    shared = np.asarray(shared, np.int64)
    n = shared.shape[0]
    groups = {a: [a] for a in range(n)}          # keyed by smallest member
    gmem = {a: int(mem[a]) for a in range(n)}
    while True:
        best = None
        keys = sorted(groups)
        for i, ga in enumerate(keys):
            for gb in keys[i + 1:]:
                if gmem[ga] + gmem[gb] > cap:
                    continue
                s = int(sum(shared[x, y] for x in groups[ga] for y in groups[gb]))
                if best is None or s > best[0]:
                    best = (s, ga, gb)
        if best is None:
            break
        _, ga, gb = best
        groups[ga] += groups.pop(gb)
        gmem[ga] += gmem.pop(gb)
    out = np.zeros(n, np.int32)
    for gid, key in enumerate(sorted(groups)):
        out[groups[key]] = gid
    return out


def assign_chunks(g: np.ndarray, h: np.ndarray, n_gpus: int) -> np.ndarray:
    """Algorithm 1: chunks in decreasing order of predicted workload g (ties: smaller index first);
    chunk a goes to the GPU m with the largest score
        s_m = (g_bar - sum_{a' in Q_m} g_a') * sum_{a' in Q_m} h(a, a'),
    g_bar = sum(g) / n_gpus (the average load of a GPU), Q_m = chunks already on m.
    Decided here: equal scores (in particular the zeros of empty GPUs and of chunks without
    communication) go to the GPU with the smaller assigned load, then the smaller index.
    Returns x[a] int32."""
    g = np.asarray(g, np.float64)
    h = np.asarray(h, np.float64)
    n = g.size
    g_bar = float(g.sum()) / n_gpus
    Q = [[] for _ in range(n_gpus)]
    load = [0.0] * n_gpus
    x = np.full(n, -1, np.int32)
    for a in sorted(range(n), key=lambda i: (-g[i], i)):
        best = None
        for m in range(n_gpus):
            comm = 0.0
            for b in Q[m]:
                comm += h[a, b]
            key = ((g_bar - load[m]) * comm, -load[m], -m)
            if best is None or key > best[0]:
                best = (key, m)
        m = best[1]
        x[a] = m
        Q[m].append(a)
        load[m] += g[a]
    return x
