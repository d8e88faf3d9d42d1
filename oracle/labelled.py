"""CPU oracle of the layer over GENERATED chunks (Sections 4.1 and 5.2 of the paper): a chunk is
whatever set of (snapshot, vertex) pairs carries one label, not a vertex range times a window.

TEST INFRASTRUCTURE ONLY: plain NumPy / Python loops, float64.  Nothing in the product path may
import this module.

What the paper fixes: a chunk owns the vertices with its label; a spatial neighbour in another
chunk contributes its stale copy (the embedding cache) instead of its current embedding, and so
does a temporal neighbour (the same vertex one snapshot earlier) for the time encoder.  Written
out for label[t, i] (any integers):
  * structure encoder, row (t, i): the normalised sum over the stored row of snapshot t, taking
    X[t, j] if label[t, j] == label[t, i] and the cache row C[t, j] otherwise (the self-loop always
    reads X); degrees are those of the full snapshot.  With two layers the second one reads the
    first layer's output Z1[t, j] for neighbours with the same label and C1[t, j] otherwise.
  * time encoder, vertex i, t ascending: the state entering step t is the vertex's own state
    after step t-1 if label[t-1, i] == label[t, i], else (also at t = 0) the stale copy
    Hc[t, i] of it - Hc holds one row per (t, i), "the state entering step t" (zero if no Hc is
    given; for the LSTM the cell rows follow all hidden rows).
  * states that leave a chunk: HN[t, i] = state after step t wherever the next step belongs to
    another chunk (t = T-1 or label[t+1, i] != label[t, i]); other rows of HN are NaN.

Temporal fusion on top (Section 5.1.2 together with Section 4.1; `present[t, i]`): a vertex that
does not exist in a snapshot has no instance in the super-graph, so its label there means
nothing.  The temporal neighbour of an instance (t, i) is the vertex's previous PRESENT instance
(t', i); the state is carried from t' to t (over the gap) if the two carry the same label and is
taken from the stale copy Hc[t, i] otherwise or if there is no earlier instance.  A vertex's
sequences are thus its maximal runs of present instances with one label; nothing is computed or
written for an absent row (its rows of Y stay NaN); an absent vertex still counts as a spatial
neighbour where the adjacency stores the edge.  HN[t, i] = state after the last instance of a
sequence.  Packing rule for the lanes (this build's own, the rule of the rectangular case with
one more key): all sequences ordered by (length descending, vertex ascending, first snapshot
ascending) go first-fit into lanes of T slots.
"""
from __future__ import annotations

import numpy as np

from .tfusion import gru_step, lstm_step


def aggregate_row(graph, labels: np.ndarray, fresh: np.ndarray, stale: np.ndarray, t: int, i: int) -> np.ndarray:
    """Row (t, i): sum_j (d_i d_j)^-1/2 * (fresh[t,j] if same label else stale[t,j]), float64."""
    sn = graph.snaps[t]
    d_i = float(sn.rowptr[i + 1] - sn.rowptr[i])
    acc = np.zeros(fresh.shape[2])
    for j in sn.col[sn.rowptr[i]:sn.rowptr[i + 1]]:
        d_j = float(sn.rowptr[j + 1] - sn.rowptr[j])
        src = fresh[t, j] if labels[t, j] == labels[t, i] else stale[t, j]
        acc += src.astype(np.float64) / np.sqrt(d_i * d_j)
    return acc


def aggregate(graph, labels: np.ndarray, fresh: np.ndarray, stale: np.ndarray) -> np.ndarray:
    """All rows, [T,N,F] float64."""
    T, N = labels.shape
    out = np.zeros((T, N, fresh.shape[2]))
    for t in range(T):
        for i in range(N):
            out[t, i] = aggregate_row(graph, labels, fresh, stale, t, i)
    return out


def sequences(labels, present) -> list:
    """(vertex, [snapshots]) for every maximal run of present instances of a vertex that carry one
    label, ordered by vertex, then first snapshot."""
    labels = np.asarray(labels)
    T, N = labels.shape
    out = []
    for i in range(N):
        ts = []
        for t in range(T):
            if not present[t, i]:
                continue
            if ts and labels[ts[-1], i] != labels[t, i]:
                out.append((i, ts))
                ts = []
            ts.append(t)
        if ts:
            out.append((i, ts))
    return out


def pack(labels, present) -> dict:
    """Lanes of T slots by the packing rule.  Returns n_lanes, slot_row int64 [T, n_lanes] (t*N + i of
    the instance in that slot, -1 = empty) and slot_reset uint8 [T, n_lanes] (1 on the first slot
    of every sequence)."""
    labels = np.asarray(labels)
    T, N = labels.shape
    lanes = []          # [free slots, [sequences]]
    for i, ts in sorted(sequences(labels, present), key=lambda s: (-len(s[1]), s[0], s[1][0])):
        for lane in lanes:
            if lane[0] >= len(ts):
                lane[0] -= len(ts)
                lane[1].append((i, ts))
                break
        else:
            lanes.append([T - len(ts), [(i, ts)]])
    slot_row = np.full((T, len(lanes)), -1, np.int64)
    slot_reset = np.zeros((T, len(lanes)), np.uint8)
    for lane, (_, seqs) in enumerate(lanes):
        s = 0
        for i, ts in seqs:
            slot_reset[s, lane] = 1
            for t in ts:
                slot_row[s, lane] = t * N + i
                s += 1
    return {"n_lanes": len(lanes), "slot_row": slot_row, "slot_reset": slot_reset}


def forward(graph, labels, params: dict, X, C, *, time_kind: str = "gru", n_struct_layers: int = 1,
            C1=None, Hc=None, act_hidden: str = "relu", act_out: str = "none", vertices=None, present=None,
            n_time_layers: int = 1):
    """Returns Y [T,N,out] float64 and HN [n_state*T*N, H] (NaN where no state leaves a chunk;
    None without a time encoder).  vertices (one structure layer only): evaluate just these
    vertices, all snapshots; Y is then [T, len(vertices), out] and HN is not returned.
    present [T,N] (needs a time encoder): rows of absent instances are NaN in Y.
    n_time_layers = 2: a second recurrent layer ("rnn1.*") on the first one's outputs; a temporal
    neighbour in another chunk is stale for it too, so its state enters and leaves at the same
    instances, through its own blocks of Hc / HN (after the first layer's); Y is its output."""
    labels = np.asarray(labels).reshape(graph.T, graph.N)
    T, N = labels.shape
    if present is not None:
        assert time_kind != "none"
        present = np.asarray(present).reshape(T, N).astype(bool)
    P = {k: np.asarray(v, np.float64) for k, v in params.items()}
    idx = list(range(N)) if vertices is None else [int(v) for v in vertices]

    def act(a, kind):
        return np.maximum(a, 0.0) if kind == "relu" else a

    def rows(fresh, stale):
        M = np.zeros((T, len(idx), fresh.shape[2]))
        for k, i in enumerate(idx):
            for t in range(T):
                M[t, k] = aggregate_row(graph, labels, fresh, stale, t, i)
        return M

    M = rows(np.asarray(X), np.asarray(C))
    if n_struct_layers == 2:
        assert vertices is None      # the second layer needs the first one's output of every neighbour
        Z1 = act(M @ P["gcn0.weight"].T + P["gcn0.bias"], act_hidden)
        M = rows(Z1, np.asarray(C1))
        Z = act(M @ P["gcn1.weight"].T + P["gcn1.bias"], act_out)
    else:
        Z = act(M @ P["gcn0.weight"].T + P["gcn0.bias"], act_out)
    if time_kind == "none":
        return Z, None
    H = P["rnn.weight_hh"].shape[1]
    lstm = time_kind == "lstm"
    V = T * N
    Y = np.zeros((T, len(idx), H))
    n_state = 2 if lstm else 1
    HN = np.full((n_time_layers * n_state * V, H), np.nan) if vertices is None else None
    if present is not None:
        Y[:] = np.nan
    for k, i in enumerate(idx):
        ts = [t for t in range(T) if present is None or present[t, i]]      # the vertex's instances
        x = {t: Z[t, k][None] for t in ts}
        for layer in range(n_time_layers):
            base = layer * n_state * V
            rnn = "rnn" if layer == 0 else "rnn1"
            h = c = None
            out = {}
            for n, t in enumerate(ts):
                if n == 0 or labels[ts[n - 1], i] != labels[t, i]:      # the temporal neighbour is in another chunk
                    h = np.zeros((1, H)) if Hc is None else np.asarray(Hc[base + t * N + i], np.float64)[None]
                    c = np.zeros((1, H)) if (Hc is None or not lstm) else np.asarray(Hc[base + V + t * N + i], np.float64)[None]
                if lstm:
                    h, c = lstm_step(P, x[t], h, c, rnn)
                else:
                    h = gru_step(P, x[t], h, rnn)
                out[t] = h
                if HN is not None and (n == len(ts) - 1 or labels[ts[n + 1], i] != labels[t, i]):
                    HN[base + t * N + i] = h[0]
                    if lstm:
                        HN[base + V + t * N + i] = c[0]
            x = out
        for t in ts:
            Y[t, k] = x[t][0]
    return Y, HN


def labels_of_chunks(chunks, T: int, N: int) -> np.ndarray:
    """label[t, i] = index of the rectangular chunk that covers (t, i); every pair must be covered."""
    lab = np.full((T, N), -1, np.int64)
    for k, (v_lo, v_hi, t_lo, t_hi) in enumerate(np.asarray(chunks, np.int64).reshape(-1, 4).tolist()):
        lab[t_lo:t_hi, v_lo:v_hi] = k
    assert (lab >= 0).all()
    return lab


def evolve(graph, labels, params: dict, X, C, target=None, want_dx: bool = False) -> dict:
    """EvolveGCN-O (the paper's Section 1 names it; weight W_t = matGRU(W_{t-1}), Y_t = relu(M_t W_t),
    mean-squared-error loss over all T*N*S outputs) over GENERATED chunks: M_t is the aggregation by
    labels of this module (row (t, i) reads X[t, j] from neighbours with its own label, the cache row
    otherwise; the cache is a constant).  Written with torch CPU float64 operations on dense per-snapshot
    matrices, gradients by autograd: the plain definition, for small cases.
    Returns dict(Y [T,N,S], loss, grads {name: array} and dX [T,N,F] if a target is given)."""
    import torch
    labels = np.asarray(labels).reshape(graph.T, graph.N)
    T, N = labels.shape
    P = {k: torch.tensor(np.asarray(v, np.float64), requires_grad=target is not None) for k, v in params.items()}
    Xt = torch.tensor(np.asarray(X, np.float64), requires_grad=want_dx and target is not None)
    Ct = torch.tensor(np.asarray(C, np.float64))
    W = P["evolve.W_init"]
    Ys = []
    for t in range(T):
        Zg = torch.sigmoid(P["evolve.U_z"] @ W + P["evolve.V_z"] @ W + P["evolve.B_z"])
        Rg = torch.sigmoid(P["evolve.U_r"] @ W + P["evolve.V_r"] @ W + P["evolve.B_r"])
        Wc = torch.tanh(P["evolve.U_h"] @ W + P["evolve.V_h"] @ (Rg * W) + P["evolve.B_h"])
        W = (1 - Zg) * W + Zg * Wc
        sn = graph.snaps[t]
        deg = np.diff(sn.rowptr).astype(np.float64)
        fresh = np.zeros((N, N))
        stale = np.zeros((N, N))
        for i in range(N):
            for j in sn.col[sn.rowptr[i]:sn.rowptr[i + 1]]:
                (fresh if labels[t, j] == labels[t, i] else stale)[i, j] = 1.0 / np.sqrt(deg[i] * deg[j])
        M = torch.from_numpy(fresh) @ Xt[t] + torch.from_numpy(stale) @ Ct[t]
        Ys.append(torch.relu(M @ W))
    Y = torch.stack(Ys)
    out = {"Y": Y.detach().numpy()}
    if target is not None:
        loss = ((Y - torch.tensor(np.asarray(target, np.float64))) ** 2).mean()
        loss.backward()
        out["loss"] = float(loss.item())
        out["grads"] = {k: P[k].grad.numpy() for k in params}
        if want_dx:
            out["dX"] = Xt.grad.numpy()
    return out
