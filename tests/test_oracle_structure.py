"""Pins for the oracle's structure encoder (aggregation + dense transform) and packing.
CPU only.  Each check is something other than the oracle's own formula: dense matmul from
an edge list, the hand-worked fixture, invariants of the normalised adjacency."""
import os
import re

import numpy as np
import pytest

import oracle
from workloads import synth
from refs import brute_pack, dense_aggregate, dense_norm_adj, edges_of

GOLD = os.path.join(os.path.dirname(__file__), "golden", "hand_example.txt")


def _graph_from_edges(N, edge_lists):
    snaps = []
    for edges in edge_lists:
        u = np.array([e[0] for e in edges], np.int64)
        v = np.array([e[1] for e in edges], np.int64)
        snaps.append(synth.csr_from_undirected(N, u, v))
    return synth.DynamicGraph(N, snaps)


def _random_edge_lists(rng, T, N, p):
    out = []
    for _ in range(T):
        out.append([(i, j) for i in range(N) for j in range(i + 1, N) if rng.random() < p])
    return out


# ------------------------------------------------------------------ hand example


def _read_gold():
    g = {}
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, val = line.split(":", 1)
        g[key.strip()] = val.strip()
    return g


def _hand_graph(g):
    edge_lists = []
    for t in range(3):
        edge_lists.append([tuple(int(x) for x in e.split("-")) for e in g[f"edges {t}"].split()])
    return _graph_from_edges(4, edge_lists)


def _expr(s):
    s6, s8 = np.sqrt(6.0), np.sqrt(8.0)  # noqa: F841  (used by eval)
    return [eval(e, {"s6": s6, "s8": s8}) for e in s.split("|")]


HAND_CHUNKS = np.array([[0, 2, 0, 3], [2, 4, 0, 3]], np.int64)


def test_hand_example_fixture_is_self_consistent():
    g = _read_gold()
    for kind in ("M_unchunked", "M_chunked"):
        for t in range(3):
            vals = [float(x) for x in g[f"{kind}_val {t}"].split()]
            assert np.allclose(_expr(g[f"{kind} {t}"]), vals, atol=5e-10)


def test_hand_example_aggregation_and_gru():
    g = _read_gold()
    graph = _hand_graph(g)
    for t in range(3):
        assert np.diff(graph.snaps[t].rowptr).tolist() == [int(x) for x in g[f"deg {t}"].split()]
    X = np.tile(np.array([1, 2, 3, 4], np.float32)[None, :, None], (3, 1, 1))
    C = np.tile(np.array([10, 20, 30, 40], np.float32)[None, :, None], (3, 1, 1))
    want_un = np.array([[float(x) for x in g[f"M_unchunked_val {t}"].split()] for t in range(3)])
    want_ch = np.array([[float(x) for x in g[f"M_chunked_val {t}"].split()] for t in range(3)])
    got_ch = np.concatenate([oracle.aggregate_chunk(graph, c, X, C)[:, :, 0] for c in HAND_CHUNKS], axis=1)
    got_un = np.concatenate([oracle.aggregate_chunk(graph, c, X, X)[:, :, 0] for c in HAND_CHUNKS], axis=1)
    whole = oracle.aggregate_chunk(graph, [0, 4, 0, 3], X, C)[:, :, 0]
    assert np.abs(got_ch - want_ch).max() < 1e-9
    assert np.abs(got_un - want_un).max() < 1e-9
    assert np.abs(whole - want_un).max() < 1e-9  # one chunk covering everything never reads C
    # GRU: r = z = 1/2, n = tanh(M + h/2)
    params = {"gcn0.weight": np.ones((1, 1), np.float32), "gcn0.bias": np.zeros(1, np.float32),
              "rnn.weight_ih": np.array([[0], [0], [1]], np.float32),
              "rnn.weight_hh": np.array([[0], [0], [1]], np.float32),
              "rnn.bias_ih": np.zeros(3, np.float32), "rnn.bias_hh": np.zeros(3, np.float32)}
    for cache, kind in ((C, "h_chunked"), (X, "h_unchunked")):
        Y = oracle.forward(graph, HAND_CHUNKS, params, X, cache, time_kind="gru")
        want = np.array([[float(x) for x in g[f"{kind} {t}"].split()] for t in range(3)])
        assert np.abs(Y[:, :, 0] - want).max() < 2e-7  # Y is stored as fp32


def test_hand_example_packing():
    g = _read_gold()
    graph = _hand_graph(g)
    p = oracle.pack(graph, HAND_CHUNKS)
    for key in ("seg_row_off", "seg_nnz_off", "halo_ptr", "halo_idx"):
        assert p[key].tolist() == [int(x) for x in g[key].split()], key
    assert p["col_local"].tolist() == [int(x) for x in g["col_local"].replace("|", " ").split()]


# ------------------------------------------------------------------ dense brute force


@pytest.mark.parametrize("seed", range(6))
def test_aggregation_equals_dense_matmul(seed):
    rng = np.random.default_rng(seed)
    T, N, F = 3, int(rng.integers(5, 40)), int(rng.integers(1, 7))
    edge_lists = _random_edge_lists(rng, T, N, float(rng.uniform(0.02, 0.5)))
    hub = int(rng.integers(0, N))
    edge_lists[1] += [(hub, j) for j in range(N) if j != hub]  # a hub adjacent to all
    edge_lists[2] = []                                          # isolated but self-looped
    graph = _graph_from_edges(N, edge_lists)
    X = rng.standard_normal((T, N, F)).astype(np.float32)
    C = rng.standard_normal((T, N, F)).astype(np.float32)
    cuts = sorted({0, N, *rng.integers(1, N, size=3).tolist()})
    for v_lo, v_hi in zip(cuts[:-1], cuts[1:]):
        M = oracle.aggregate_chunk(graph, [v_lo, v_hi, 0, T], X, C)
        for t in range(T):
            Ahat = dense_norm_adj(N, edge_lists[t])
            want = dense_aggregate(Ahat, X[t], C[t], v_lo, v_hi)
            assert np.abs(M[t] - want).max() < 1e-12


def test_every_edge_cut_and_no_edge_cut():
    N, F = 8, 3
    rng = np.random.default_rng(3)
    X = rng.standard_normal((1, N, F)).astype(np.float32)
    C = rng.standard_normal((1, N, F)).astype(np.float32)
    # bipartite between {0..3} and {4..7}: chunks [0,4),[4,8) cut every edge
    cut_all = [(i, j) for i in range(4) for j in range(4, 8) if (i + j) % 2]
    # two cliques: chunks cut no edge
    cut_none = [(i, j) for i in range(4) for j in range(i + 1, 4)] + \
               [(i, j) for i in range(4, 8) for j in range(i + 1, 8)]
    for edges, depends_on_cache in ((cut_all, True), (cut_none, False)):
        graph = _graph_from_edges(N, [edges])
        Ahat = dense_norm_adj(N, edges)
        for v_lo, v_hi in ((0, 4), (4, 8)):
            M = oracle.aggregate_chunk(graph, [v_lo, v_hi, 0, 1], X, C)[0]
            assert np.abs(M - dense_aggregate(Ahat, X[0], C[0], v_lo, v_hi)).max() < 1e-12
            M2 = oracle.aggregate_chunk(graph, [v_lo, v_hi, 0, 1], X, C + 1.0)[0]
            assert (np.abs(M2 - M).max() > 1e-3) == depends_on_cache


@pytest.mark.parametrize("seed", range(3))
def test_sqrt_degree_vector_is_fixed(seed):
    """x_i = c*sqrt(d_i) is an eigenvector of the normalised adjacency with eigenvalue 1; it
    survives chunking iff the cache equals the input."""
    rng = np.random.default_rng(100 + seed)
    N = 30
    graph = _graph_from_edges(N, _random_edge_lists(rng, 2, N, 0.2))
    X = np.zeros((2, N, 2), np.float32)
    for t in range(2):
        d = np.diff(graph.snaps[t].rowptr).astype(np.float64)
        X[t, :, 0] = 3.0 * np.sqrt(d)
        X[t, :, 1] = -0.5 * np.sqrt(d)
    for v_lo, v_hi in ((0, 11), (11, 30)):
        M = oracle.aggregate_chunk(graph, [v_lo, v_hi, 0, 2], X, X)
        # X holds sqrt(d) rounded to fp32, so the fixed point holds to that rounding
        assert np.abs(M - X[:, v_lo:v_hi].astype(np.float64)).max() < 2e-6
    # d-regular graph (a ring): the constant vector maps to itself
    ring = _graph_from_edges(N, [[(i, (i + 1) % N) for i in range(N)]])
    ones = np.ones((1, N, 1), np.float32)
    assert np.abs(oracle.aggregate_chunk(ring, [0, N, 0, 1], ones, ones) - 1.0).max() < 1e-15


def test_zero_in_gives_activation_of_bias():
    wl = synth.random_small(5, T=3, N=20, F=4, S=5, H=5, avg_deg=3.0, chunks=[[0, 9, 0, 3], [9, 20, 0, 3]],
                            time_kind="none")
    Z = np.zeros_like(wl.X)
    Y = oracle.forward(wl.graph, wl.chunks, wl.params, Z, Z, time_kind="none", act_out="relu")
    want = np.maximum(wl.params["gcn0.bias"], 0.0)
    assert np.abs(Y - want[None, None, :]).max() == 0.0
    Y = oracle.forward(wl.graph, wl.chunks, wl.params, Z, Z, time_kind="none", act_out="none")
    assert np.abs(Y - wl.params["gcn0.bias"][None, None, :]).max() == 0.0


@pytest.mark.parametrize("layers", [1, 2])
def test_gcn_layers_equal_dense(layers):
    """One and two stacked GCN layers against dense float64 matmuls; the second layer reads
    the first layer's output for in-chunk neighbours and its own cache outside."""
    rng = np.random.default_rng(11)
    T, N, F, S = 2, 17, 5, 4
    chunks = np.array([[0, 6, 0, 2], [6, 17, 0, 1], [6, 17, 1, 2]], np.int64)
    wl = synth.random_small(11, T, N, F, S, S, 4.0, chunks, "none", layers, hub=True)
    p = wl.params
    Y = oracle.forward(wl.graph, chunks, p, wl.X, wl.C, time_kind="none", n_struct_layers=layers,
                       act_hidden="relu", act_out="none", C1=wl.C1)
    for v_lo, v_hi, t_lo, t_hi in chunks.tolist():
        for t in range(t_lo, t_hi):
            Ahat = dense_norm_adj(N, edges_of(wl.graph.snaps[t]))
            z = dense_aggregate(Ahat, wl.X[t], wl.C[t], v_lo, v_hi) @ p["gcn0.weight"].astype(np.float64).T \
                + p["gcn0.bias"]
            if layers == 2:
                z1_all = wl.C1[t].astype(np.float64).copy()
                z1_all[v_lo:v_hi] = np.maximum(z, 0.0)
                z = Ahat[v_lo:v_hi] @ z1_all @ p["gcn1.weight"].astype(np.float64).T + p["gcn1.bias"]
            assert np.abs(Y[t, v_lo:v_hi] - z).max() < 1e-5 * max(1.0, np.abs(z).max())
    del rng


# ------------------------------------------------------------------ packing


@pytest.mark.parametrize("seed", range(5))
def test_packing_equals_brute_force(seed):
    rng = np.random.default_rng(200 + seed)
    T, N = 4, int(rng.integers(6, 50))
    graph = _graph_from_edges(N, _random_edge_lists(rng, T, N, float(rng.uniform(0.05, 0.4))))
    cuts = sorted({0, N, *rng.integers(1, N, size=3).tolist()})
    chunks = []
    for v_lo, v_hi in zip(cuts[:-1], cuts[1:]):
        t_cut = int(rng.integers(1, T))
        chunks += [[v_lo, v_hi, 0, t_cut], [v_lo, v_hi, t_cut, T]]
    order = rng.permutation(len(chunks))
    chunks = np.array(chunks, np.int64)[order]
    got, want = oracle.pack(graph, chunks), brute_pack(graph, chunks)
    for k in want:
        assert np.array_equal(got[k], want[k]), k
    # properties: halo sorted-unique and outside the range; col_local inverts to the column
    s = 0
    for v_lo, v_hi, t_lo, t_hi in chunks.tolist():
        for t in range(t_lo, t_hi):
            halo = got["halo_idx"][got["halo_ptr"][s]:got["halo_ptr"][s + 1]]
            assert np.all(np.diff(halo) > 0)
            assert np.all((halo < v_lo) | (halo >= v_hi))
            snap = graph.snaps[t]
            cols = snap.col[snap.rowptr[v_lo]:snap.rowptr[v_hi]]
            loc = got["col_local"][got["seg_nnz_off"][s]:got["seg_nnz_off"][s + 1]]
            back = np.where(loc < v_hi - v_lo, loc + v_lo, halo[np.maximum(loc - (v_hi - v_lo), 0)] if len(halo)
                            else loc + v_lo)
            assert np.array_equal(back, cols)
            s += 1


def test_worklist_rule():
    rng = np.random.default_rng(7)
    N, T = 40, 2
    edge_lists = _random_edge_lists(rng, T, N, 0.1)
    edge_lists[0] += [(3, j) for j in range(N) if j != 3] + [(30, j) for j in range(0, N, 2) if j != 30]
    graph = _graph_from_edges(N, edge_lists)
    chunks = np.array([[0, 17, 0, 2], [17, 40, 0, 1]], np.int64)
    R, L, P = 4, 12, 5
    got = oracle.worklist(graph, chunks, R, L, P)
    short, long_ = [], []
    seg_of = {}
    s = 0
    for k, (v_lo, v_hi, t_lo, t_hi) in enumerate(chunks.tolist()):
        for t in range(t_lo, t_hi):
            seg_of[(k, t)] = s
            deg = np.diff(graph.snaps[t].rowptr)
            for i in range(v_lo, v_hi):
                if deg[i] > L:
                    parts = -(-int(deg[i]) // P)
                    long_ += [(s, i - v_lo, p, parts) for p in range(parts)]
            s += 1
    for t in range(T):  # short list: snapshot by snapshot
        for k, (v_lo, v_hi, t_lo, t_hi) in enumerate(chunks.tolist()):
            if t_lo <= t < t_hi:
                for r in range(0, v_hi - v_lo, R):
                    short.append((seg_of[(k, t)], r, min(R, v_hi - v_lo - r)))
    assert got["work_short"].tolist() == [list(x) for x in short]
    assert got["work_long"].tolist() == [list(x) for x in long_]
    assert len(long_) > 0
