"""Data selection for comparisons at sizes where the CPU oracle can only compute a sample:
which rows of the (device-resident) tensors a sampled computation reads, copied back into
HostMirror arrays, and small stand-in problems in which a sampled vertex sees exactly the rows
it sees in the full problem.  Index plumbing only: no arithmetic of the method, all of which
stays in the oracle that is handed these arrays.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np

from . import synth


def _row(s: synth.Snapshot, i: int) -> np.ndarray:
    return s.col[s.rowptr[i]:s.rowptr[i + 1]].astype(np.int64)


def rows_read_two_layers(hg: synth.DynamicGraph, chunk: Sequence[int], subset: np.ndarray):
    """For a two-layer structure encoder evaluated for the vertices `subset` of one chunk: per
    snapshot t of the chunk's window, (first-layer rows evaluated, cache rows of the first layer's
    input read, cache rows of the second layer's input read) as ascending global vertex ids.  The
    first-layer input rows read inside the chunk range are not listed: callers copy the whole range."""
    v_lo, v_hi, t_lo, t_hi = (int(x) for x in chunk)
    out = []
    for t in range(t_lo, t_hi):
        s = hg.snaps[t]
        nb = [_row(s, int(v)) for v in subset]
        allnb = np.unique(np.concatenate(nb)) if nb else np.zeros(0, np.int64)
        inside = (allnb >= v_lo) & (allnb < v_hi)
        eval1 = np.union1d(allnb[inside], np.asarray(subset, np.int64))
        c1_rows = allnb[~inside]
        cols = np.concatenate([_row(s, int(j)) for j in eval1]) if eval1.size else np.zeros(0, np.int64)
        cols = np.unique(cols)
        c_rows = cols[(cols < v_lo) | (cols >= v_hi)]
        out.append((eval1, c_rows, c1_rows))
    return out


def fill_two_layer_mirrors(hg, chunk, subset, mx, mc, mc1) -> None:
    """Copy into the mirrors every row the oracle reads when it evaluates `subset` of `chunk`
    (two structure layers): the chunk's own input rows, the cache rows its evaluated first-layer
    rows read, the second-layer cache rows the subset's rows read."""
    v_lo, v_hi, t_lo, t_hi = (int(x) for x in chunk)
    for t, (_, c_rows, c1_rows) in zip(range(t_lo, t_hi), rows_read_two_layers(hg, chunk, subset)):
        mx.fill_range(t, v_lo, v_hi)
        mc.fill_rows(t, c_rows)
        if mc1 is not None:
            mc1.fill_rows(t, c1_rows)


def pick_chunks(hg, chunks: np.ndarray, n_random: int, rng) -> List[int]:
    """Chunk sample for a bounded comparison: the first and the last chunk (lowest and highest
    addresses), the chunk holding the densest (chunk, snapshot) segment, the chunk holding the
    highest-degree vertex, and n_random more."""
    ids = {0, len(chunks) - 1}
    best_seg, best_deg = (-1, -1), (-1, -1)
    for k, (v_lo, v_hi, t_lo, t_hi) in enumerate(chunks.tolist()):
        for t in range(t_lo, t_hi):
            rp = hg.snaps[t].rowptr
            seg = int(rp[v_hi] - rp[v_lo])
            deg = int(np.diff(rp[v_lo:v_hi + 1]).max())
            best_seg = max(best_seg, (seg, k))
            best_deg = max(best_deg, (deg, k))
    ids |= {best_seg[1], best_deg[1]}
    rest = [k for k in range(len(chunks)) if k not in ids]
    if rest and n_random > 0:
        ids |= set(rng.choice(rest, size=min(n_random, len(rest)), replace=False).tolist())
    return sorted(ids)


def pick_vertices(hg, chunk, n_random: int, rng, with_hub: bool = True) -> np.ndarray:
    """Vertices of a chunk to compare: its first and last vertex (tile edges), n_random seeded ones
    and, if asked, the vertex with the most neighbours in the chunk's first snapshot."""
    v_lo, v_hi, t_lo, _ = (int(x) for x in chunk)
    pick = {v_lo, v_hi - 1} | set((rng.choice(v_hi - v_lo, size=min(n_random, v_hi - v_lo), replace=False) + v_lo).tolist())
    if with_hub:
        pick.add(v_lo + int(np.argmax(np.diff(hg.snaps[t_lo].rowptr[v_lo:v_hi + 1]))))
    return np.array(sorted(pick), np.int64)


def bounded_neighbours(hg, v: int, ch, max_deg: int) -> bool:
    """All of v's neighbours inside the chunk's vertex range have at most max_deg stored non-zeros in
    every snapshot of the chunk's window (keeps the two-hop stand-in problem small)."""
    for t in range(ch[2], ch[3]):
        s = hg.snaps[t]
        nb = s.col[s.rowptr[v]:s.rowptr[v + 1]].astype(np.int64)
        nb = nb[(nb >= ch[0]) & (nb < ch[1])]
        if int((s.rowptr[nb + 1] - s.rowptr[nb]).max()) > max_deg:
            return False
    return True


def bounded_pick(hg, ch, rng, max_deg: int, tries: int = 2000) -> int:
    """A seeded random vertex of the chunk with bounded_neighbours."""
    for _ in range(tries):
        v = int(rng.integers(ch[0], ch[1]))
        if bounded_neighbours(hg, v, ch, max_deg):
            return v
    raise ValueError("no vertex with bounded neighbours found")


# --------------------------------------------------------------------------- stand-in problems


def one_hop_problem(g, picks, X, C, F: int):
    """One small problem in which local vertex i, a chunk of its own, computes exactly what the
    sampled vertex picks[i] = (v, chunk) does.  The other local vertices are copies of the sampled
    vertices' neighbours, one per (sampled vertex, snapshot, neighbour): each lies outside every
    one-vertex chunk, so the oracle reads it from the cache handed over here, which holds the row
    the neighbour is really read from (X inside the real chunk's vertex range, the cache
    outside), and its row length is the neighbour's real degree, which the normalisation uses.
    X, C: anything indexable as [t, ids] -> rows (host arrays, or RowFetcher over device tensors).
    Data selection only; all arithmetic stays in the oracle."""
    T, m = g.T, len(picks)
    rows = [[None] * m for _ in range(T)]
    copies = np.zeros(T, np.int64)
    for t in range(T):
        s = g.snaps[t]
        for i, (v, ch) in enumerate(picks):
            if ch[2] <= t < ch[3]:
                rows[t][i] = s.col[s.rowptr[v]:s.rowptr[v + 1]].astype(np.int64)
                copies[t] += int((rows[t][i] != v).sum())
    n_loc = m + int(copies.max())
    Xs = np.zeros((T, n_loc, F), np.float32)
    Cs = np.zeros((T, n_loc, F), np.float32)
    snaps = []
    for t in range(T):
        deg = np.diff(g.snaps[t].rowptr)
        row_len = np.zeros(n_loc, np.int64)
        cols, nxt = [], m
        for i, (v, ch) in enumerate(picks):
            c = rows[t][i]
            if c is None:
                continue
            other = c != v
            nb = c[other]
            loc = np.full(len(c), i, np.int32)
            loc[other] = nxt + np.arange(len(nb), dtype=np.int32)
            inside = (nb >= ch[0]) & (nb < ch[1])
            Xs[t, i] = X[t, v]
            Cs[t, nxt:nxt + len(nb)] = np.where(inside[:, None], X[t, nb], C[t, nb])
            row_len[i] = len(c)
            row_len[nxt:nxt + len(nb)] = deg[nb]
            cols.append(loc)
            nxt += len(nb)
        rowptr = np.concatenate([[0], np.cumsum(row_len)]).astype(np.int64)
        col = np.zeros(int(rowptr[-1]), np.int32)          # the copies' own rows are never walked
        if cols:
            head = np.concatenate(cols)
            col[:len(head)] = head
        snaps.append(synth.Snapshot(rowptr, col))
    chunks = np.array([[i, i + 1, ch[2], ch[3]] for i, (_, ch) in enumerate(picks)], np.int64)
    return synth.DynamicGraph(n_loc, snaps), chunks, Xs, Cs



def one_vertex_problem(graph, v, chunk, X, C, F: int, params: dict):
    """The problem (for the attention layer, whose time encoder sees the whole window of one vertex)
    whose only covered vertex computes exactly what vertex v of `chunk` does: local vertex 0 is v, the
    other local vertices are its neighbours of one snapshot each, all outside the one-vertex chunk, so
    the oracle reads them from the cache handed over here, which holds the row each neighbour is really
    read from (X inside the chunk's vertex range, the cache outside).  The window becomes snapshots
    0..w-1 and the position table is cut to it.  X, C: indexable as [t, ids] -> fp32 rows."""
    v_lo, v_hi, t_lo, t_hi = chunk
    per_t = []
    for t in range(t_lo, t_hi):
        s = graph.snaps[t]
        per_t.append(s.col[s.rowptr[v]:s.rowptr[v + 1]].astype(np.int64))
    n_loc = 1 + max(int((c != v).sum()) for c in per_t)
    w = t_hi - t_lo
    Xs = np.zeros((w, n_loc, F), np.float32)
    Cs = np.zeros((w, n_loc, F), np.float32)
    snaps = []
    for k, cols in enumerate(per_t):
        t = t_lo + k
        Xs[k, 0] = X[t, v]
        loc = np.zeros(len(cols), np.int32)
        others = cols != v
        loc[others] = 1 + np.arange(int(others.sum()), dtype=np.int32)
        nb = cols[others]
        inside = (nb >= v_lo) & (nb < v_hi)
        if len(nb):
            Cs[k, 1:1 + len(nb)] = np.where(inside[:, None], X[t, nb], C[t, nb])
        rowptr = np.full(n_loc + 1, len(cols), np.int64)
        rowptr[0] = 0
        snaps.append(synth.Snapshot(rowptr, loc))
    p = dict(params)
    p["attn.pos"] = params["attn.pos"][t_lo:t_hi]
    return synth.DynamicGraph(n_loc, snaps), np.array([[0, 1, 0, w]], np.int64), p, Xs, Cs


def two_hop_problem(hg, picks, fetch_x, fetch_c, fetch_tgt, F: int):
    """One small problem for a single-layer structure encoder with an input gradient: local chunk
    i holds the sampled vertex picks[i] = (v, chunk) and, per snapshot, slots for v's neighbours
    inside the real chunk's vertex range, each with its real stored row, so that both v's output
    and the gradient that v's input row receives from those neighbours are what they are in the
    full problem.  Every other vertex a stored row names is a copy placed outside all local chunks:
    it carries the row that is really read (the input row if it lies in the real chunk's range, the
    cache row otherwise) and, as row length, its real degree.  Slots and copies are reused from
    snapshot to snapshot (the structure encoder does not couple snapshots); a slot without a
    neighbour in some snapshot is an isolated vertex with a zero input row and a zero target.
    fetch_x / fetch_c / fetch_tgt (t, ids) -> [len(ids), F] rows of the input, the cache and the
    targets.  Returns (graph, chunks, X, C, target, where, members) with where[i] = local id of
    picks[i] and members[i] = [(t, local id, real vertex)] of every real row local chunk i holds."""
    T = hg.T
    slots = []
    for v, ch in picks:
        n = 0
        for t in range(ch[2], ch[3]):
            nb = _row(hg.snaps[t], v)
            n = max(n, int(((nb >= ch[0]) & (nb < ch[1]) & (nb != v)).sum()))
        slots.append(n)
    base = np.concatenate([[0], np.cumsum([1 + n for n in slots])]).astype(np.int64)
    n_in = int(base[-1])
    per_t, n_copies = [], 0
    held = [[] for _ in picks]
    for t in range(T):
        s = hg.snaps[t]
        deg = np.diff(s.rowptr)
        rows, copy_id, copy_fresh = [], [], []
        for i, (v, ch) in enumerate(picks):
            if not (ch[2] <= t < ch[3]):
                continue
            nb_v = _row(s, v)
            members = np.concatenate([[v], nb_v[(nb_v >= ch[0]) & (nb_v < ch[1]) & (nb_v != v)]])
            for pos, j in enumerate(members.tolist()):
                cols = _row(s, j)
                loc = np.full(len(cols), -1, np.int64)
                loc[cols == v] = base[i]
                loc[cols == j] = base[i] + pos
                if pos == 0:                      # the sampled vertex's row names its slots
                    order = np.argsort(members[1:])
                    hit = np.isin(cols, members[1:])
                    loc[hit] = base[i] + 1 + order[np.searchsorted(members[1:], cols[hit], sorter=order)]
                other = np.flatnonzero(loc < 0)
                loc[other] = n_in + len(copy_id) + np.arange(len(other))
                copy_id += cols[other].tolist()
                copy_fresh += ((cols[other] >= ch[0]) & (cols[other] < ch[1])).tolist()
                rows.append((int(base[i] + pos), j, loc))
                held[i].append((t, int(base[i] + pos), j))
        per_t.append((rows, np.asarray(copy_id, np.int64), np.asarray(copy_fresh, bool), deg))
        n_copies = max(n_copies, len(copy_id))
    n_loc = n_in + n_copies
    X = np.zeros((T, n_loc, F), np.float32)
    C = np.zeros((T, n_loc, F), np.float32)
    tgt = np.zeros((T, n_loc, F), np.float32)
    snaps = []
    for t, (rows, cid, fresh, deg) in enumerate(per_t):
        row_len = np.ones(n_loc, np.int64)
        for loc_id, _, loc in rows:
            row_len[loc_id] = len(loc)
        row_len[n_in:n_in + len(cid)] = deg[cid]
        rowptr = np.concatenate([[0], np.cumsum(row_len)]).astype(np.int64)
        col = np.zeros(int(rowptr[-1]), np.int32)          # the copies' own rows are never walked
        col[rowptr[:n_in]] = np.arange(n_in)               # slots without a row: a self-loop only
        for loc_id, _, loc in rows:
            col[rowptr[loc_id]:rowptr[loc_id + 1]] = loc
        if rows:
            ids = np.asarray([r[0] for r in rows], np.int64)
            real = np.asarray([r[1] for r in rows], np.int64)
            X[t, ids] = fetch_x(t, real)
            tgt[t, ids] = fetch_tgt(t, real)
        if len(cid):
            got = np.empty((len(cid), F), np.float32)
            if fresh.any():
                got[fresh] = fetch_x(t, cid[fresh])
            if (~fresh).any():
                got[~fresh] = fetch_c(t, cid[~fresh])
            C[t, n_in:n_in + len(cid)] = got
        snaps.append(synth.Snapshot(rowptr, col))
    chunks = np.array([[base[i], base[i + 1], ch[2], ch[3]] for i, (_, ch) in enumerate(picks)], np.int64)
    return synth.DynamicGraph(n_loc, snaps), chunks, X, C, tgt, base[:-1].copy(), held
