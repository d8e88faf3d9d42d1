"""Pins of the fusion-selection / chunk-assignment oracle (oracle/fusion.py): the paper's drawn
example, a dense-matrix formulation of the same sets, worked examples of both greedy procedures,
their stopping conditions and the special cases that reduce to textbook procedures."""
import heapq
import os

import numpy as np
import pytest

from oracle import fusion
from workloads import synth

CHUNKS = [[0, 70, 0, 8], [70, 201, 0, 5], [70, 201, 5, 8], [201, 260, 2, 8]]


def test_paper_drawn_example():
    spec = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "spatial_fusion_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, *v = line.split()
                spec[k] = v
    u, v = zip(*[map(int, e.split("-")) for e in spec["edges"]])
    g = synth.DynamicGraph(N=6, snaps=[synth.csr_from_undirected(6, np.array(u), np.array(v))])
    ci, cj = [int(x) for x in spec["chunk_i"]], [int(x) for x in spec["chunk_j"]]
    chunks = [[ci[0], ci[-1] + 1, 0, 1], [cj[0], cj[-1] + 1, 0, 1]]
    sets = fusion.load_sets(g, chunks)
    assert sorted(v for _, v in sets[0] & sets[1]) == [int(x) for x in spec["loaded_twice"]]
    S = fusion.shared_rows(g, chunks)
    assert S.tolist() == [[0, int(spec["shared"][0])], [int(spec["shared"][0]), 0]]


def _dense_shared(graph, chunks):
    """The same quantity from dense adjacency matrices and boolean masks."""
    T, N = graph.T, graph.N
    loads = []
    for v_lo, v_hi, t_lo, t_hi in chunks:
        m = np.zeros((T, N), bool)
        for t in range(t_lo, t_hi):
            sn = graph.snaps[t]
            A = np.zeros((N, N), bool)
            A[np.repeat(np.arange(N), np.diff(sn.rowptr)), sn.col] = True
            m[t] = A[v_lo:v_hi].any(axis=0)
            m[t, v_lo:v_hi] = True
        loads.append(m)
    n = len(chunks)
    return np.array([[0 if a == b else int((loads[a] & loads[b]).sum()) for b in range(n)] for a in range(n)])


def test_shared_rows_against_dense_masks():
    wl = synth.random_small(5, 8, 260, 8, 32, 32, 4.0, CHUNKS, "gru", hub=True)
    S = fusion.shared_rows(wl.graph, wl.chunks)
    np.testing.assert_array_equal(S, _dense_shared(wl.graph, CHUNKS))
    assert (S == S.T).all() and (np.diag(S) == 0).all()
    assert S[1, 2] == 0                       # same vertices, disjoint windows: nothing in common
    assert S[0, 1] > 0 and S[2, 3] > 0
    sizes = [len(s) for s in fusion.load_sets(wl.graph, wl.chunks)]
    assert all(S[a, b] <= min(sizes[a], sizes[b]) for a in range(4) for b in range(4))


def test_no_cross_edges_share_nothing():
    # two cliques, one per chunk
    u = [0, 0, 1, 3, 3, 4]
    v = [1, 2, 2, 4, 5, 5]
    g = synth.DynamicGraph(N=6, snaps=[synth.csr_from_undirected(6, np.array(u), np.array(v))] * 2)
    assert fusion.shared_rows(g, [[0, 3, 0, 2], [3, 6, 0, 2]]).sum() == 0


SH4 = np.array([[0, 5, 1, 0], [5, 0, 2, 0], [1, 2, 0, 4], [0, 0, 4, 0]])


@pytest.mark.parametrize("cap,want", [
    (5, [0, 1, 2, 3]),      # no two chunks fit together
    (6, [0, 0, 1, 1]),      # (0,1) shares 5, then (2,3) shares 4; the two groups (12) do not fit
    (9, [0, 0, 1, 1]),      # after (0,1): {0,1}+2 shares 3 and fits, but (2,3) shares 4 and goes first
    (12, [0, 0, 0, 0]),     # everything fits in the end
])
def test_select_fusion_worked_example(cap, want):
    assert fusion.select_fusion(SH4, np.array([3, 3, 3, 3]), cap).tolist() == want


def test_select_fusion_prefers_the_pair_that_fits():
    # the largest pair (0,1) does not fit; the next one does
    sh = np.array([[0, 9, 2], [9, 0, 3], [2, 3, 0]])
    assert fusion.select_fusion(sh, np.array([6, 6, 2]), 10).tolist() == [0, 1, 1]


def _matrix_greedy(shared, mem, cap):
    """Same procedure kept as a contracted matrix: rows / columns of fused groups are added."""
    S = np.array(shared, np.int64)
    np.fill_diagonal(S, -1)
    mem = [int(m) for m in mem]
    members = [[i] for i in range(len(mem))]
    alive = [True] * len(mem)
    while True:
        best = None
        for a in range(len(mem)):
            for b in range(a + 1, len(mem)):
                if alive[a] and alive[b] and mem[a] + mem[b] <= cap and (best is None or S[a, b] > best[0]):
                    best = (S[a, b], a, b)
        if best is None:
            break
        _, a, b = best
        S[a, :] += S[b, :]
        S[:, a] += S[:, b]
        S[a, a] = -1
        mem[a] += mem[b]
        members[a] += members[b]
        alive[b] = False
    out = np.zeros(len(mem), np.int32)
    for gid, a in enumerate(i for i in range(len(mem)) if alive[i]):
        out[members[a]] = gid
    return out


@pytest.mark.parametrize("seed", range(6))
def test_select_fusion_random_instances(seed):
    rng = np.random.default_rng(seed)
    n = 14
    sh = rng.integers(0, 50, (n, n))
    sh = np.triu(sh, 1) + np.triu(sh, 1).T
    sh[rng.random((n, n)) < 0.3] = 0
    sh = np.minimum(sh, sh.T)
    mem = rng.integers(1, 20, n)
    cap = int(rng.integers(15, 60))
    grp = fusion.select_fusion(sh, mem, cap)
    np.testing.assert_array_equal(grp, _matrix_greedy(sh, mem, cap))
    gm = np.bincount(grp, weights=mem)
    assert all(gm[k] <= cap or (grp == k).sum() == 1 for k in range(gm.size))       # the cap holds
    assert all(gm[a] + gm[b] > cap for a in range(gm.size) for b in range(a + 1, gm.size))  # nothing left to fuse
    assert sorted(np.unique(grp)) == list(range(gm.size))
    first = [np.flatnonzero(grp == k)[0] for k in range(gm.size)]
    assert first == sorted(first)                                                   # numbered by smallest member


def test_assign_worked_example():
    # g_bar = 14 / 2 = 7.  Order 0, 1, 2, 3.
    # a=0: all scores 0, equal loads -> GPU 0.            a=1: s0 = (7-5)*h(1,0) = 2*3 = 6 > s1 = 0 -> GPU 0.
    # a=2: s0 = (7-9)*(1+1) = -4 < s1 = 0 -> GPU 1.        a=3: s0 = (7-9)*(0+2) = -4, s1 = (7-3)*1 = 4 -> GPU 1.
    g = np.array([5.0, 4.0, 3.0, 2.0])
    h = np.array([[0, 3, 1, 0], [3, 0, 1, 2], [1, 1, 0, 1], [0, 2, 1, 0]], float)
    assert fusion.assign_chunks(g, h, 2).tolist() == [0, 0, 1, 1]
    assert fusion.assign_chunks(g, h, 1).tolist() == [0, 0, 0, 0]
    # the score multiplies balance and communication: with a much stronger tie to GPU 1's chunk,
    # chunk 3 still goes where the product is largest
    h2 = h.copy()
    h2[3, 2] = h2[2, 3] = 0.0
    assert fusion.assign_chunks(g, h2, 2).tolist() == [0, 0, 1, 1]      # s1 = 0 > s0 = -4


def test_assign_without_communication_is_longest_processing_time_first():
    rng = np.random.default_rng(3)
    for n_gpus in (2, 3, 5):
        g = rng.integers(1, 100, 40).astype(float)
        x = fusion.assign_chunks(g, np.zeros((40, 40)), n_gpus)
        heap = [(0.0, m) for m in range(n_gpus)]
        want = np.zeros(40, np.int32)
        for a in sorted(range(40), key=lambda i: (-g[i], i)):
            load, m = heapq.heappop(heap)
            want[a] = m
            heapq.heappush(heap, (load + g[a], m))
        np.testing.assert_array_equal(x, want)
        loads = np.bincount(x, weights=g, minlength=n_gpus)
        assert loads.max() - loads.min() <= g.max()
