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


# ---- temporal fusion on top of generated chunks (presence) ------------------------------------

def test_presence_all_ones_changes_nothing():
    wl = synth.random_small(16, T, N, F, S, S, 3.0, [[0, N, 0, T]], "lstm", n_struct_layers=2)
    rng = np.random.default_rng(3)
    lab = rng.integers(0, 3, (T, N))
    Hc = rng.standard_normal((2 * T * N, S))
    a, hn_a = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="lstm", n_struct_layers=2, C1=wl.C1, Hc=Hc)
    b, hn_b = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="lstm", n_struct_layers=2, C1=wl.C1, Hc=Hc,
                               present=np.ones((T, N), np.uint8))
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(hn_a, hn_b)


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_presence_with_one_label_is_temporal_fusion_of_one_chunk(kind):
    """One chunk covering everything: the sequences, the lanes and the outputs are those of the
    temporal-fusion oracle for the rectangle [0,N) x [0,T) (pinned by the paper's drawn example and
    the library recurrences), with the state rows re-indexed: a sequence starts from the cache row of
    its first instance and leaves its state in the row of its last one."""
    from oracle import tfusion
    wl = synth.random_small(17, T, N, F, S, S, 3.0, [[0, N, 0, T]], kind)
    present = synth.presence(4, T, N)
    lab = np.full((T, N), 5)
    rect = [[0, N, 0, T]]
    n_state = 2 if kind == "lstm" else 1
    H0 = 0.3 * np.random.default_rng(6).standard_normal((n_state * N, S))
    V = T * N
    Hc = np.full((n_state * V, S), np.nan)
    first = {i: int(np.flatnonzero(present[:, i])[0]) for i in range(N) if present[:, i].any()}
    last = {i: int(np.flatnonzero(present[:, i])[-1]) for i in first}
    for i, t in first.items():
        for part in range(n_state):
            Hc[part * V + t * N + i] = H0[part * N + i]
    Y, HN = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind=kind, Hc=Hc, present=present)
    Z, _ = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="none")
    want, want_HN = tfusion.run_separate(Z, present, rect, wl.params, kind, H0=H0, return_state=True)
    assert np.array_equal(np.isnan(Y), np.isnan(want))
    assert np.nanmax(np.abs(Y - want)) < 1e-12
    seen = np.zeros(HN.shape[0], bool)
    for i, t in last.items():
        for part in range(n_state):
            assert np.abs(HN[part * V + t * N + i] - want_HN[part * N + i]).max() < 1e-12
            seen[part * V + t * N + i] = True
    assert np.isnan(HN[~seen]).all()
    p, q = labelled.pack(lab, present), tfusion.pack(present, rect)
    np.testing.assert_array_equal(p["slot_row"], q["slot_row"])
    np.testing.assert_array_equal(p["slot_reset"], q["slot_reset"])


def test_presence_sequences_against_the_library_recurrence():
    """Random labels and presence: every run of present instances with one label, compressed and run
    through torch.nn.GRU from its cache row, gives the oracle's rows; the label of an absent
    instance plays no part (scrambling those labels changes nothing)."""
    import torch
    wl = synth.random_small(18, 7, 23, F, S, S, 3.0, [[0, 23, 0, 7]], "gru")
    Tn, Nn = 7, 23
    rng = np.random.default_rng(8)
    lab = rng.integers(0, 2, (Tn, Nn))
    present = synth.presence(9, Tn, Nn)
    Hc = rng.standard_normal((Tn * Nn, S))
    Y, HN = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="gru", Hc=Hc, present=present)
    lab2 = np.where(present.astype(bool), lab, rng.integers(5, 9, (Tn, Nn)))
    Y2, HN2 = labelled.forward(wl.graph, lab2, wl.params, wl.X, wl.C, time_kind="gru", Hc=Hc, present=present)
    # spatial neighbours that are absent keep their real label's role: compare only the time encoder's part,
    # i.e. feed both from the same structure output
    Z, _ = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind="none")
    gru = torch.nn.GRU(S, S, batch_first=True).double()
    with torch.no_grad():
        gru.weight_ih_l0.copy_(torch.from_numpy(wl.params["rnn.weight_ih"].astype(np.float64)))
        gru.weight_hh_l0.copy_(torch.from_numpy(wl.params["rnn.weight_hh"].astype(np.float64)))
        gru.bias_ih_l0.copy_(torch.from_numpy(wl.params["rnn.bias_ih"].astype(np.float64)))
        gru.bias_hh_l0.copy_(torch.from_numpy(wl.params["rnn.bias_hh"].astype(np.float64)))
    seqs = labelled.sequences(lab, present)
    assert sum(len(ts) for _, ts in seqs) == int(present.sum())
    n_multi = 0
    for i, ts in seqs:
        assert all(present[t, i] for t in ts) and len({int(lab[t, i]) for t in ts}) == 1
        n_multi += len(ts) > 1 and ts[-1] - ts[0] + 1 > len(ts)          # a sequence with a gap inside
        x = torch.from_numpy(Z[ts, i][None])
        h0 = torch.from_numpy(Hc[ts[0] * Nn + i][None, None])
        with torch.no_grad():
            out, hn = gru(x, h0)
        assert np.abs(out[0].numpy() - Y[ts, i]).max() < 1e-12
        assert np.abs(hn[0, 0].numpy() - HN[ts[-1] * Nn + i]).max() < 1e-12
    assert n_multi > 0
    assert np.isnan(Y[~present.astype(bool)]).all()
    assert int((~np.isnan(HN[:, 0])).sum()) == len(seqs)
    # labels of absent instances do not matter for where sequences start and end
    assert [(i, ts) for i, ts in labelled.sequences(lab2, present)] == seqs
    assert np.array_equal(np.isnan(HN2), np.isnan(HN))


def test_presence_packing_hand_example_and_properties():
    """T = 4, three vertices.  Vertex 0: present 1111, labels aabb -> sequences [0,1], [2,3];
    vertex 1: present 1011, labels aaab -> [0,2] (gap carried), [3]; vertex 2: present 0100 -> [1].
    Order (length desc, vertex, first snapshot): (0,[0,1]) (0,[2,3]) (1,[0,2]) (1,[3]) (2,[1]);
    first fit into lanes of 4: lane 0 = (0,[0,1]) + (0,[2,3]); lane 1 = (1,[0,2]) + (1,[3]) + (2,[1])."""
    lab = np.array([[0, 0, 0], [0, 0, 0], [1, 0, 0], [1, 1, 0]])
    present = np.array([[1, 1, 0], [1, 0, 1], [1, 1, 0], [1, 1, 0]], np.uint8)
    p = labelled.pack(lab, present)
    assert p["n_lanes"] == 2
    np.testing.assert_array_equal(p["slot_row"], np.array([[0, 1], [3, 7], [6, 10], [9, 5]]))
    np.testing.assert_array_equal(p["slot_reset"], np.array([[1, 1], [0, 0], [1, 1], [0, 1]]))
    rng = np.random.default_rng(12)
    Tn, Nn = 9, 40
    lab = rng.integers(0, 3, (Tn, Nn))
    present = synth.presence(13, Tn, Nn)
    p = labelled.pack(lab, present)
    rows = p["slot_row"][p["slot_row"] >= 0]
    assert sorted(rows.tolist()) == sorted(np.flatnonzero(present.reshape(-1)).tolist())     # every instance once
    assert -(-int(present.sum()) // Tn) <= p["n_lanes"] <= len(labelled.sequences(lab, present))
    for lane in range(p["n_lanes"]):
        col, rst = p["slot_row"][:, lane], p["slot_reset"][:, lane]
        n = int((col >= 0).sum())
        assert (col[:n] >= 0).all() and rst[0] == 1 and (rst[n:] == 0).all()
        for s in range(1, n):
            same = col[s] % Nn == col[s - 1] % Nn and col[s] > col[s - 1] and \
                lab.reshape(-1)[col[s]] == lab.reshape(-1)[col[s - 1]] and \
                not present[col[s - 1] // Nn + 1: col[s] // Nn, col[s] % Nn].any()
            assert bool(rst[s]) == (not same)


# ---- stacked time encoder (two recurrent layers) over sequences ---------------------------------

@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_stacked_encoder_over_sequences(kind):
    """(i) every instance present, rectangular chunks: the temporal-fusion oracle with two recurrent
    layers is the rectangular layer with two recurrent layers (pinned against the library's
    two-layer unit elsewhere), states of both layers included; (ii) rectangular labels give the
    same through the labelled oracle; (iii) with a presence matrix, every sequence compressed and run
    through torch.nn.GRU / LSTM with num_layers = 2 from its own state rows."""
    import torch
    from oracle import tfusion
    wl = synth.random_small(61, T, N, F, S, S, 3.0, RECT, kind, hub=True)
    wl.params = synth.layer_params(61, F, S, S, kind, 1, random_bias=True, n_time_layers=2)
    n_state = 2 if kind == "lstm" else 1
    tot = int((RECT[:, 1] - RECT[:, 0]).sum())
    rng = np.random.default_rng(62)
    H0 = (0.5 * rng.standard_normal((2 * n_state * tot, S))).astype(np.float32)
    want, want_HN = oracle.forward(wl.graph, RECT, wl.params, wl.X, wl.C, time_kind=kind, H0=H0, return_state=True,
                                   n_time_layers=2)
    Z = oracle.forward(wl.graph, RECT, wl.params, wl.X, wl.C, time_kind="none").astype(np.float64)
    ones = np.ones((T, N), np.uint8)
    Y, HN = tfusion.run_separate(Z, ones, RECT, wl.params, kind, H0=H0, return_state=True, n_time_layers=2)
    assert np.abs(Y - want).max() < 2e-6 and np.abs(HN - want_HN).max() < 2e-6
    # (ii) labelled oracle, state cache rows at the window starts of the rectangles, both layers
    V = T * N
    Hc = np.full((2 * n_state * V, S), np.nan)
    off = 0
    for v_lo, v_hi, t_lo, _ in RECT.tolist():
        nv = v_hi - v_lo
        for blk in range(2 * n_state):
            Hc[blk * V + t_lo * N + v_lo: blk * V + t_lo * N + v_hi] = H0[blk * tot + off: blk * tot + off + nv]
        off += nv
    lab = labelled.labels_of_chunks(RECT, T, N)
    Yl, HNl = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind=kind, Hc=Hc, n_time_layers=2)
    assert np.abs(Yl - want).max() < 2e-6
    off = 0
    for v_lo, v_hi, _, t_hi in RECT.tolist():
        nv = v_hi - v_lo
        for blk in range(2 * n_state):
            rows = slice(blk * V + (t_hi - 1) * N + v_lo, blk * V + (t_hi - 1) * N + v_hi)
            assert np.abs(HNl[rows] - want_HN[blk * tot + off: blk * tot + off + nv]).max() < 2e-6
        off += nv
    # (iii) presence: the library's two-layer unit on the compressed sequences
    present = synth.presence(63, T, N)
    Yp, HNp = tfusion.run_separate(Z, present, RECT, wl.params, kind, H0=H0, return_state=True, n_time_layers=2)
    rnn = (torch.nn.GRU if kind == "gru" else torch.nn.LSTM)(S, S, num_layers=2, batch_first=True).double()
    with torch.no_grad():
        for l, pre in ((0, "rnn"), (1, "rnn1")):
            for nm in ("weight_ih", "weight_hh", "bias_ih", "bias_hh"):
                getattr(rnn, f"{nm}_l{l}").copy_(torch.from_numpy(wl.params[f"{pre}.{nm}"]).double())
    offs = tfusion.state_rows(RECT)
    n_checked = 0
    for k, seqs in enumerate(tfusion.sequences(present, RECT)):
        for i, ts in seqs:
            row = int(offs[k] + i - RECT[k, 0])
            x = torch.from_numpy(Z[ts, i][None])
            h0 = torch.from_numpy(np.stack([H0[row], H0[n_state * tot + row]]).astype(np.float64))[:, None]
            with torch.no_grad():
                if kind == "gru":
                    out, hn = rnn(x, h0)
                else:
                    c0 = torch.from_numpy(np.stack([H0[tot + row], H0[3 * tot + row]]).astype(np.float64))[:, None]
                    out, (hn, cn) = rnn(x, (h0, c0))
                    for l in range(2):
                        assert np.abs(HNp[(2 * l + 1) * tot + row] - cn[l, 0].numpy()).max() < 1e-12
            assert np.abs(out[0].numpy() - Yp[ts, i]).max() < 1e-12
            for l in range(2):
                assert np.abs(HNp[l * n_state * tot + row] - hn[l, 0].numpy()).max() < 1e-12
            n_checked += 1
    assert n_checked > 30
    # and the labelled oracle with presence and one label per rectangle agrees with it
    Ylp, _ = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind=kind, Hc=_hc_first_instances(Hc, H0, present, n_state, tot),
                              present=present, n_time_layers=2)
    # (Yp was fed the C oracle's structure output, rounded to float32 on return: hence 1e-7, not 1e-12)
    assert np.array_equal(np.isnan(Ylp), np.isnan(Yp)) and np.nanmax(np.abs(Ylp - Yp)) < 1e-7


def _hc_first_instances(Hc, H0, present, n_state, tot):
    """State cache for the labelled oracle under a presence matrix: the H0 row of (chunk, vertex) sits at
    the vertex's first present instance of the chunk's window."""
    V = T * N
    out = np.full_like(Hc, np.nan)
    off = 0
    for v_lo, v_hi, t_lo, t_hi in RECT.tolist():
        for i in range(v_lo, v_hi):
            ts = [t for t in range(t_lo, t_hi) if present[t, i]]
            if ts:
                for blk in range(2 * n_state):
                    out[blk * V + ts[0] * N + i] = H0[blk * tot + off + i - v_lo]
        off += v_hi - v_lo
    return out


# ---- EvolveGCN-O over generated chunks --------------------------------------------------------

def test_evolving_weights_over_rectangular_labels_equal_the_rectangular_oracle():
    """Labels that are rectangles: outputs, loss, all ten parameter gradients and the input gradient of
    the labelled definition (torch autograd, dense matrices) against the C oracle's (loops, hand-written
    back-propagation; itself pinned by autograd from edge lists and finite differences).  And labels
    matter: moving one vertex to another chunk changes its neighbours' rows."""
    Fe = 6
    wl = synth.random_small(71, T, N, Fe, 32, 32, 3.0, RECT, "none", hub=True)
    params = synth.evolve_params(8, Fe, Fe, random_bias=True)
    target = synth.stream(8, "target").standard_normal((T, N, Fe)).astype(np.float32)
    want = oracle.evolve(wl.graph, RECT, params, wl.X, wl.C, target, want_grads=True, want_dx=True)
    lab = labelled.labels_of_chunks(RECT, T, N)
    got = labelled.evolve(wl.graph, lab, params, wl.X, wl.C, target, want_dx=True)
    assert np.abs(got["Y"] - want["Y"]).max() < 1e-5                  # the C oracle returns float32
    assert abs(got["loss"] - want["loss"]) < 1e-10 * max(1.0, want["loss"])
    for k in oracle.EVOLVE_PARAMS:
        assert np.abs(got["grads"][k] - want["grads"][k]).max() < 1e-10 * max(1.0, np.abs(want["grads"][k]).max()), k
    assert np.abs(got["dX"] - want["dX"]).max() < 1e-12 * max(1.0, np.abs(want["dX"]).max())
    lab2 = lab.copy()
    lab2[2, 3] = 99
    moved = labelled.evolve(wl.graph, lab2, params, wl.X, wl.C)["Y"]
    sn = wl.graph.snaps[2]
    nb = [int(j) for j in sn.col[sn.rowptr[3]:sn.rowptr[4]] if j != 3 and lab[2, j] == lab[2, 3]]
    changed = np.flatnonzero(np.abs(moved[2] - got["Y"][2]).max(axis=1) > 0)
    assert set(changed.tolist()) <= set(nb + [3]) and (not nb or len(changed) > 0)
    assert np.array_equal(moved[[0, 1, 3, 4]], got["Y"][[0, 1, 3, 4]])
