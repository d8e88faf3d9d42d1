"""Pins for the oracle's time encoder and for the chunking invariants.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth
from refs import dense_aggregate, dense_norm_adj, edges_of


def _torch_rnn(kind, params, S, H):
    rnn = (torch.nn.GRU if kind == "gru" else torch.nn.LSTM)(S, H, num_layers=1, batch_first=False).double()
    with torch.no_grad():
        rnn.weight_ih_l0.copy_(torch.from_numpy(params["rnn.weight_ih"]).double())
        rnn.weight_hh_l0.copy_(torch.from_numpy(params["rnn.weight_hh"]).double())
        rnn.bias_ih_l0.copy_(torch.from_numpy(params["rnn.bias_ih"]).double())
        rnn.bias_hh_l0.copy_(torch.from_numpy(params["rnn.bias_hh"]).double())
    return rnn


def _dense_struct(wl, t, v_lo, v_hi, cache):
    Ahat = dense_norm_adj(wl.graph.N, edges_of(wl.graph.snaps[t]))
    m = dense_aggregate(Ahat, wl.X[t], cache[t], v_lo, v_hi)
    return m @ wl.params["gcn0.weight"].astype(np.float64).T + wl.params["gcn0.bias"]


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_layer_equals_dense_gcn_plus_torch_rnn(kind):
    """Special case -> library routine: the per-vertex recurrence over a window is
    torch.nn.GRU / torch.nn.LSTM (float64) with batch = the chunk's vertices."""
    T, N, F, S, H = 5, 23, 6, 7, 5
    chunks = np.array([[0, 10, 0, 5], [10, 23, 0, 2], [10, 23, 2, 5]], np.int64)
    wl = synth.random_small(21, T, N, F, S, H, 3.0, chunks, kind, hub=True)
    Y, hN = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, H0=wl.H0,
                           return_state=True)
    rnn = _torch_rnn(kind, wl.params, S, H)
    tot = int((chunks[:, 1] - chunks[:, 0]).sum())
    off = 0
    for v_lo, v_hi, t_lo, t_hi in chunks.tolist():
        z = np.stack([_dense_struct(wl, t, v_lo, v_hi, wl.C) for t in range(t_lo, t_hi)])  # [w,nv,S]
        nv = v_hi - v_lo
        h0 = torch.from_numpy(wl.H0[off:off + nv]).double()[None]
        with torch.no_grad():
            if kind == "gru":
                out, hn = rnn(torch.from_numpy(z), h0)
            else:
                c0 = torch.from_numpy(wl.H0[tot + off:tot + off + nv]).double()[None]
                out, (hn, cn) = rnn(torch.from_numpy(z), (h0, c0))
                assert np.abs(hN[tot + off:tot + off + nv] - cn[0].numpy()).max() < 2e-6
        assert np.abs(Y[t_lo:t_hi, v_lo:v_hi] - out.numpy()).max() < 2e-6
        assert np.abs(hN[off:off + nv] - hn[0].numpy()).max() < 2e-6
        off += nv


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_concatenated_sequences_with_mask_equal_separate_runs(kind):
    """Section 5.1.2: in the concatenated sequence (B1,B2,C1,C2) the mask at C1 must stop
    B2's state; the result then equals running (B1,B2) and (C1,C2) separately."""
    T, N, F, S, H = 4, 12, 3, 4, 6
    wl = synth.random_small(33, T, N, F, S, H, 2.5, [[0, N, 0, T]], kind)
    mask = np.zeros((T, N), np.uint8)
    mask[2, :] = 1
    Y_cat = oracle.forward(wl.graph, [[0, N, 0, 4]], wl.params, wl.X, wl.C, time_kind=kind, reset_mask=mask)
    Y_sep = oracle.forward(wl.graph, [[0, N, 0, 2], [0, N, 2, 4]], wl.params, wl.X, wl.C, time_kind=kind)
    assert np.array_equal(Y_cat, Y_sep)
    # without the mask the second half does receive the first half's state
    Y_leak = oracle.forward(wl.graph, [[0, N, 0, 4]], wl.params, wl.X, wl.C, time_kind=kind)
    assert np.array_equal(Y_leak[:2], Y_sep[:2]) and np.abs(Y_leak[2:] - Y_sep[2:]).max() > 1e-3
    # per-vertex masks: only the masked vertices change
    mask2 = np.zeros((T, N), np.uint8)
    mask2[2, ::3] = 1
    Y_part = oracle.forward(wl.graph, [[0, N, 0, 4]], wl.params, wl.X, wl.C, time_kind=kind, reset_mask=mask2)
    assert np.array_equal(Y_part[:, ::3], Y_sep[:, ::3])
    assert np.array_equal(Y_part[:, 1::3], Y_leak[:, 1::3])


@pytest.mark.parametrize("kind,layers", [("gru", 1), ("lstm", 2), ("none", 2)])
def test_cache_equal_to_input_makes_chunking_invisible(kind, layers):
    """Partitioning does not change the training algorithm (Section 7.6): with the cache
    holding the current values and window-start states chained, the chunked layer equals
    the whole-graph layer."""
    T, N, F, S, H = 6, 31, 5, 6, 6 if kind != "none" else 6
    wl = synth.random_small(44, T, N, F, S, H, 3.5, [[0, N, 0, T]], kind, layers, hub=True)
    kw = dict(time_kind=kind, n_struct_layers=layers, act_hidden="relu")
    # whole graph as one chunk: the cache is never read
    C1_exact = None
    if layers == 2:
        p1 = {"gcn0.weight": wl.params["gcn0.weight"], "gcn0.bias": wl.params["gcn0.bias"]}
        C1_exact = oracle.forward(wl.graph, [[0, N, 0, T]], p1, wl.X, wl.X, time_kind="none", act_out="relu")
    whole = oracle.forward(wl.graph, [[0, N, 0, T]], wl.params, wl.X, wl.X, C1=C1_exact, **kw)
    garbage = np.full_like(wl.X, 1e6)
    whole2 = oracle.forward(wl.graph, [[0, N, 0, T]], wl.params, wl.X, garbage,
                            C1=None if C1_exact is None else np.full_like(C1_exact, -1e6), **kw)
    assert np.array_equal(whole, whole2)
    # 3 vertex ranges x 2 windows, windows chained through the returned state
    bounds = [0, 9, 20, N]
    Y = np.full_like(whole, np.nan)
    state = None
    for t_lo, t_hi in ((0, 3), (3, 6)):
        chunks = [[bounds[r], bounds[r + 1], t_lo, t_hi] for r in range(3)]
        if kind == "none":
            oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.X, C1=C1_exact, Y=Y, **kw)
        else:
            _, state = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.X, C1=C1_exact, H0=state, Y=Y,
                                      return_state=True, **kw)
    # hN is stored as fp32 between windows: equality up to that rounding
    assert np.abs(Y - whole).max() < 5e-6


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_fused_equals_one_chunk_at_a_time(kind):
    T, N, F, S, H = 4, 26, 4, 5, 3
    chunks = np.array([[0, 7, 0, 4], [7, 19, 0, 2], [7, 19, 2, 4], [19, 26, 1, 4]], np.int64)
    wl = synth.random_small(55, T, N, F, S, H, 3.0, chunks, kind)
    fused = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, H0=wl.H0)
    tot = int((chunks[:, 1] - chunks[:, 0]).sum())
    Y = np.full_like(fused, np.nan)
    off = np.concatenate([[0], np.cumsum(chunks[:, 1] - chunks[:, 0])])
    for k in (2, 0, 3, 1):  # any order
        sl = slice(off[k], off[k + 1])
        h0 = wl.H0[sl] if kind == "gru" else np.concatenate([wl.H0[sl], wl.H0[tot + off[k]:tot + off[k + 1]]])
        oracle.forward(wl.graph, chunks[k:k + 1], wl.params, wl.X, wl.C, time_kind=kind, H0=h0, Y=Y)
    assert np.array_equal(np.isnan(Y), np.isnan(fused))
    assert np.array_equal(np.nan_to_num(Y), np.nan_to_num(fused))  # bit-equal
    assert np.isnan(fused[0, 19:26]).all()  # rows outside every chunk are not written


def test_subset_evaluation_equals_full():
    """A subset evaluates only the first-layer rows its vertices read; what it returns for them is
    bit for bit what the evaluation of every row returns (one and two structure layers, the time
    encoder reading the last layer or both)."""
    T, N, F, S, H = 4, 30, 4, 5, 5
    chunks = np.array([[0, 13, 0, 4], [13, 30, 0, 4]], np.int64)
    for kind, layers, cat in (("gru", 1, False), ("lstm", 2, False), ("lstm", 2, True), ("none", 2, False)):
        wl = synth.random_small(66, T, N, F, S, H, 3.0, chunks, kind, layers, input_concat=cat)
        full = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, H0=wl.H0,
                              n_struct_layers=layers, C1=wl.C1, input_concat=cat)
        subset = [[1, 5, 12], [13, 29]]
        part = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, H0=wl.H0,
                              n_struct_layers=layers, C1=wl.C1, subset=subset, input_concat=cat)
        rows = [1, 5, 12, 13, 29]
        assert np.array_equal(part[:, rows], full[:, rows])
        others = [i for i in range(N) if i not in rows]
        assert np.isnan(part[:, others]).all()


def test_identity_structure_reduces_to_plain_rnn():
    """Self-loops only (normalised adjacency = I) and W0 = I: the layer is torch.nn.GRU on X."""
    T, N, D = 5, 9, 4
    graph = synth.DynamicGraph(N, [synth.csr_from_undirected(N, np.zeros(0, np.int64), np.zeros(0, np.int64))
                                   for _ in range(T)])
    params = synth.layer_params(3, D, D, D, "gru", 1, random_bias=True)
    params["gcn0.weight"] = np.eye(D, dtype=np.float32)
    params["gcn0.bias"] = np.zeros(D, np.float32)
    X = synth.stream(3, "feat").standard_normal((T, N, D)).astype(np.float32)
    Y = oracle.forward(graph, [[0, N, 0, T]], params, X, X, time_kind="gru")
    with torch.no_grad():
        out, _ = _torch_rnn("gru", params, D, D)(torch.from_numpy(X).double())
    assert np.abs(Y - out.numpy()).max() < 2e-6


@pytest.mark.parametrize("kind", ["lstm", "gru"])
def test_concatenated_structure_outputs_feed_the_time_encoder(kind):
    """Section 6 (MPNN-LSTM): the time encoder reads both structure layers' outputs side by
    side.  Built here from dense matrices and the library recurrence with a 2S-wide input; the
    two halves of the input weights are scaled differently so that swapped halves fail."""
    T, N, F, S, H = 4, 19, 5, 6, 7
    chunks = np.array([[0, 8, 0, 4], [8, 19, 0, 3], [8, 19, 3, 4]], np.int64)
    wl = synth.random_small(33, T, N, F, S, H, 3.0, chunks, kind, n_struct_layers=2, hub=True, input_concat=True)
    assert wl.params["rnn.weight_ih"].shape[1] == 2 * S
    wl.params["rnn.weight_ih"][:, :S] *= 1.7
    Y, hN = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, n_struct_layers=2, C1=wl.C1,
                           H0=wl.H0, return_state=True, input_concat=True)
    rnn = _torch_rnn(kind, wl.params, 2 * S, H)
    P = {k: v.astype(np.float64) for k, v in wl.params.items()}
    tot = int((chunks[:, 1] - chunks[:, 0]).sum())
    off = 0
    for v_lo, v_hi, t_lo, t_hi in chunks.tolist():
        xs = []
        for t in range(t_lo, t_hi):
            Ahat = dense_norm_adj(N, edges_of(wl.graph.snaps[t]))
            z1 = np.maximum(dense_aggregate(Ahat, wl.X[t], wl.C[t], v_lo, v_hi) @ P["gcn0.weight"].T + P["gcn0.bias"], 0)
            full = np.zeros((N, S))
            full[v_lo:v_hi] = z1
            z2 = dense_aggregate(Ahat, full, wl.C1[t], v_lo, v_hi) @ P["gcn1.weight"].T + P["gcn1.bias"]
            xs.append(np.concatenate([z1, z2], axis=1))
        nv = v_hi - v_lo
        h0 = torch.from_numpy(wl.H0[off:off + nv]).double()[None]
        with torch.no_grad():
            if kind == "gru":
                out, hn = rnn(torch.from_numpy(np.stack(xs)), h0)
            else:
                c0 = torch.from_numpy(wl.H0[tot + off:tot + off + nv]).double()[None]
                out, (hn, cn) = rnn(torch.from_numpy(np.stack(xs)), (h0, c0))
                assert np.abs(hN[tot + off:tot + off + nv] - cn[0].numpy()).max() < 2e-6
        assert np.abs(Y[t_lo:t_hi, v_lo:v_hi] - out.numpy()).max() < 2e-6
        assert np.abs(hN[off:off + nv] - hn[0].numpy()).max() < 2e-6
        off += nv
    # without the flag the same call refuses the wide weights
    with pytest.raises(AssertionError):
        oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, n_struct_layers=2, C1=wl.C1)


@pytest.mark.parametrize("kind", ["lstm", "gru"])
def test_stacked_time_encoder_equals_the_two_layer_library_unit(kind):
    """Section 6 (MPNN-LSTM: two stacked LSTM layers).  Special case -> library routine: structure
    encoder as dense matrices, then torch.nn.LSTM / GRU with num_layers = 2 (float64), initial and
    final states of both layers included; the second layer's weights must matter; a reset mask on
    the stacked layer equals separate runs."""
    T, N, F, S, H = 5, 19, 6, 7, 5
    chunks = np.array([[0, 8, 0, 5], [8, 19, 0, 2], [8, 19, 2, 5]], np.int64)
    wl = synth.random_small(52, T, N, F, S, H, 3.0, chunks, kind, hub=True)
    wl.params = synth.layer_params(52, F, S, H, kind, 1, random_bias=True, n_time_layers=2)
    tot = int((chunks[:, 1] - chunks[:, 0]).sum())
    n_state = 2 if kind == "lstm" else 1
    H0 = (0.5 * synth.stream(52, "h0-stacked").standard_normal((2 * n_state * tot, H))).astype(np.float32)
    Y, hN = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, H0=H0, return_state=True,
                           n_time_layers=2)
    rnn = (torch.nn.GRU if kind == "gru" else torch.nn.LSTM)(S, H, num_layers=2).double()
    with torch.no_grad():
        for l, pre in ((0, "rnn"), (1, "rnn1")):
            for nm in ("weight_ih", "weight_hh", "bias_ih", "bias_hh"):
                getattr(rnn, f"{nm}_l{l}").copy_(torch.from_numpy(wl.params[f"{pre}.{nm}"]).double())
    blk = lambda b, a, n: torch.from_numpy(H0[b * tot + a:b * tot + a + n]).double()
    off = 0
    for v_lo, v_hi, t_lo, t_hi in chunks.tolist():
        nv = v_hi - v_lo
        z = torch.from_numpy(np.stack([_dense_struct(wl, t, v_lo, v_hi, wl.C) for t in range(t_lo, t_hi)]))
        h0 = torch.stack([blk(0, off, nv), blk(n_state, off, nv)])
        with torch.no_grad():
            if kind == "gru":
                out, hn = rnn(z, h0)
            else:
                c0 = torch.stack([blk(1, off, nv), blk(3, off, nv)])
                out, (hn, cn) = rnn(z, (h0, c0))
                for l in range(2):
                    assert np.abs(hN[(l * 2 + 1) * tot + off:(l * 2 + 1) * tot + off + nv] - cn[l].numpy()).max() < 2e-6
        assert np.abs(Y[t_lo:t_hi, v_lo:v_hi] - out.numpy()).max() < 2e-6
        for l in range(2):
            assert np.abs(hN[l * n_state * tot + off:l * n_state * tot + off + nv] - hn[l].numpy()).max() < 2e-6
        off += nv
    one = oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=kind, H0=H0[:n_state * tot])
    assert np.nanmax(np.abs(one - Y)) > 1e-2          # the second layer is not a pass-through
    # reset mask: the stacked encoder over the concatenated sequence = separate runs (Section 5.1.2)
    wl2 = synth.random_small(53, 4, 12, 3, 4, 6, 2.5, [[0, 12, 0, 4]], kind)
    wl2.params = synth.layer_params(53, 3, 4, 6, kind, 1, random_bias=True, n_time_layers=2)
    mask = np.zeros((4, 12), np.uint8)
    mask[2] = 1
    whole = oracle.forward(wl2.graph, wl2.chunks, wl2.params, wl2.X, wl2.C, time_kind=kind, reset_mask=mask, n_time_layers=2)
    parts = np.full_like(whole, np.nan)
    for t0, t1 in ((0, 2), (2, 4)):
        oracle.forward(wl2.graph, [[0, 12, t0, t1]], wl2.params, wl2.X, wl2.C, time_kind=kind, Y=parts, n_time_layers=2)
    assert np.array_equal(whole, parts)
