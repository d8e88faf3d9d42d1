"""Pins for the oracle of the layer over generated (labelled) chunks.  CPU only."""
import numpy as np
import pytest

import oracle
from oracle import labelled
from workloads import synth
from refs import dense_norm_adj, edges_of

T, N, F, S = 5, 31, 6, 8
RECT = np.array([[0, 12, 0, 5], [12, 31, 0, 2], [12, 31, 2, 5]], np.int64)


def _hc_from_h0(wl, kind):
    """A state cache whose rows at the window starts of the rectangular chunks are the chunks'
    H0 rows and everything else NaN (must not be read)."""
    V = T * N
    n_state = 2 if kind == "lstm" else 1
    Hc = np.full((n_state * V, wl.H), np.nan)
    tot = int((RECT[:, 1] - RECT[:, 0]).sum())
    off = 0
    for v_lo, v_hi, t_lo, _ in RECT.tolist():
        nv = v_hi - v_lo
        for part in range(n_state):
            Hc[part * V + t_lo * N + v_lo: part * V + t_lo * N + v_hi] = wl.H0[part * tot + off: part * tot + off + nv]
        off += nv
    return Hc


@pytest.mark.parametrize("kind,layers", [("gru", 1), ("lstm", 2), ("none", 2)])
def test_rectangular_labels_reproduce_the_rectangular_layer(kind, layers):
    """Labels that happen to be vertex ranges x windows: the same result as the layer defined over
    rectangular chunks (pinned elsewhere), states included; cache rows nobody may read are NaN."""
    wl = synth.random_small(11, T, N, F, S, S, 3.0, RECT, kind, n_struct_layers=layers, hub=True)
    lab = labelled.labels_of_chunks(RECT, T, N)
    Hc = _hc_from_h0(wl, kind) if kind != "none" else None
    Y, HN = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind=kind, n_struct_layers=layers, C1=wl.C1, Hc=Hc)
    want = oracle.forward(wl.graph, RECT, wl.params, wl.X, wl.C, time_kind=kind, n_struct_layers=layers, C1=wl.C1,
                          H0=wl.H0, return_state=kind != "none")
    want_Y, want_HN = want if kind != "none" else (want, None)
    assert np.abs(Y - want_Y).max() < 2e-6
    if kind != "none":
        V = T * N
        tot = int((RECT[:, 1] - RECT[:, 0]).sum())
        off = 0
        seen = np.zeros(HN.shape[0], bool)
        for v_lo, v_hi, _, t_hi in RECT.tolist():
            nv = v_hi - v_lo
            for part in range(HN.shape[0] // V):
                rows = slice(part * V + (t_hi - 1) * N + v_lo, part * V + (t_hi - 1) * N + v_hi)
                assert np.abs(HN[rows] - want_HN[part * tot + off: part * tot + off + nv]).max() < 2e-6
                seen[rows] = True
            off += nv
        assert np.isnan(HN[~seen]).all()          # nothing else leaves a chunk


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_one_label_is_the_unchunked_layer(kind):
    """Everything in one chunk: no cache row is read (they are NaN here), only Hc at t = 0."""
    wl = synth.random_small(12, T, N, F, S, S, 3.0, [[0, N, 0, T]], kind, n_struct_layers=2)
    V = T * N
    n_state = 2 if kind == "lstm" else 1
    Hc = np.full((n_state * V, S), np.nan)
    for part in range(n_state):
        Hc[part * V: part * V + N] = wl.H0[part * N:(part + 1) * N]
    nanC = np.full_like(wl.X, np.nan)
    Y, HN = labelled.forward(wl.graph, np.full((T, N), 7), wl.params, wl.X, nanC, time_kind=kind, n_struct_layers=2,
                             C1=np.full_like(wl.C1, np.nan), Hc=Hc)
    want, want_HN = oracle.forward(wl.graph, [[0, N, 0, T]], wl.params, wl.X, wl.X, time_kind=kind, n_struct_layers=2,
                                   C1=wl.C1, H0=wl.H0, return_state=True)
    assert np.abs(Y - want).max() < 2e-6
    assert np.abs(HN[(T - 1) * N: T * N] - want_HN[:N]).max() < 2e-6


def test_all_labels_different_reads_only_stale_neighbours():
    """Every (snapshot, vertex) its own chunk: the aggregation is the off-diagonal part of the
    normalised adjacency times the cache plus the diagonal times X (dense matrices), and every
    step of the time encoder starts from the state cache."""
    wl = synth.random_small(13, T, N, F, S, S, 3.0, [[0, N, 0, T]], "gru", hub=True)
    lab = np.arange(T * N).reshape(T, N)
    Hc = 0.3 * np.random.default_rng(5).standard_normal((T * N, S))
    Y, HN = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="gru", Hc=Hc)
    P = {k: v.astype(np.float64) for k, v in wl.params.items()}
    for t in range(T):
        A = dense_norm_adj(N, edges_of(wl.graph.snaps[t]))
        D = np.diag(np.diag(A))
        Z = (D @ wl.X[t] + (A - D) @ wl.C[t]) @ P["gcn0.weight"].T + P["gcn0.bias"]
        want = labelled.gru_step(P, Z, Hc[t * N:(t + 1) * N])
        assert np.abs(Y[t] - want).max() < 1e-12
        assert np.abs(HN[t * N:(t + 1) * N] - want).max() < 1e-12     # every state leaves its chunk


def test_label_of_the_right_snapshot_decides():
    """A vertex that changes chunk between two snapshots: its neighbours in the snapshot before
    see it as fresh, in the snapshot after as stale (a mistake that looks the label up in another
    snapshot fails here)."""
    wl = synth.random_small(14, 3, 9, 4, 8, 8, 8.0, [[0, 9, 0, 3]], "none")     # complete graph
    lab = np.zeros((3, 9), np.int64)
    lab[1:, 4] = 1                                   # vertex 4 leaves the chunk after snapshot 0
    X, C = wl.X.astype(np.float64), wl.C.astype(np.float64)
    M = labelled.aggregate(wl.graph, lab, X, C)
    for t in range(3):
        A = dense_norm_adj(9, edges_of(wl.graph.snaps[t]))
        mix = X[t].copy()
        if t >= 1:
            mix[4] = C[t, 4]
        want = A @ mix
        rows = [i for i in range(9) if i != 4]
        assert np.abs(M[t][rows] - want[rows]).max() < 1e-12
        # vertex 4 itself: alone in its chunk from snapshot 1 on
        if t >= 1:
            own = np.diag(np.diag(A)) @ X[t] + (A - np.diag(np.diag(A))) @ C[t]
            assert np.abs(M[t][4] - own[4]).max() < 1e-12


def test_vertex_subset_equals_full():
    wl = synth.random_small(15, T, N, F, S, S, 3.0, [[0, N, 0, T]], "gru")
    rng = np.random.default_rng(2)
    lab = rng.integers(0, 4, (T, N))
    Hc = rng.standard_normal((T * N, S))
    full, _ = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="gru", Hc=Hc)
    sub, hn = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="gru", Hc=Hc, vertices=[3, 17, 30])
    assert hn is None
    np.testing.assert_array_equal(sub, full[:, [3, 17, 30]])
