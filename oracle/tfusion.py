"""CPU oracle of temporal fusion (Section 5.1.2 of the paper): vertex sequences of different
lengths are concatenated into fixed-length lanes instead of being padded with zeros, and a mask
keeps the hidden state of one sequence from reaching the next one.

TEST INFRASTRUCTURE ONLY: plain NumPy / Python loops, float64.  Nothing in the product path may
import this module.

Definitions used here (the paper gives the idea and the mask equation, not a packing rule):
  * `present[t, i]` says whether vertex i exists in snapshot t.  The sequence of vertex i in a
    chunk (vertex range x window) is the ascending list of the window's snapshots in which it is
    present; the time encoder steps through exactly those (its state is carried over the gaps).
  * Packing rule (this build's own, first-fit decreasing): per chunk, the non-empty sequences
    are ordered by (length descending, vertex ascending); each goes into the first lane, in order
    of creation, that still has room for all of it, else into a new lane; lanes are as long as
    the chunk's window; a sequence occupies consecutive slots.  Lanes are numbered chunk after
    chunk in order of creation.
  * The first slot of every sequence carries a reset flag: the state entering that step is zero
    (the mask of the paper's update-gate equation, applied wherever the incoming state appears),
    or, if initial states are given, the state row of that (chunk, vertex): H0 / HN hold one row per
    (chunk, vertex) in chunk order (for an LSTM the cell rows follow all hidden rows), as without
    fusion.  HN receives the state after the vertex's last present snapshot of the window; a vertex
    that is absent throughout keeps its state (HN row = H0 row).  Chained windows then equal one
    long window.
"""
from __future__ import annotations

import numpy as np


def sequences(present: np.ndarray, chunks) -> list:
    """Per chunk: list of (vertex, [snapshots]) for the vertices with a non-empty sequence."""
    out = []
    for v_lo, v_hi, t_lo, t_hi in np.asarray(chunks, np.int64).reshape(-1, 4).tolist():
        seqs = []
        for i in range(v_lo, v_hi):
            ts = [t for t in range(t_lo, t_hi) if present[t, i]]
            if ts:
                seqs.append((i, ts))
        out.append(seqs)
    return out


def pack(present: np.ndarray, chunks) -> dict:
    """Lanes by the packing rule.  Returns lane_ptr int64[n_chunks+1] (first lane of each chunk),
    slot_row int64[Lmax, n_lanes] (t*N + i of the row in that slot, -1 = empty) and slot_reset
    uint8[Lmax, n_lanes] (1 on the first slot of every sequence)."""
    T, N = present.shape
    ch = np.asarray(chunks, np.int64).reshape(-1, 4)
    Lmax = int((ch[:, 3] - ch[:, 2]).max())
    lanes = []           # list of (chunk, [(vertex, [snapshots]), ...])
    lane_ptr = [0]
    for k, seqs in enumerate(sequences(present, ch)):
        L = int(ch[k, 3] - ch[k, 2])
        mine = []        # [free slots, [sequences]] per lane of this chunk
        for i, ts in sorted(seqs, key=lambda s: (-len(s[1]), s[0])):
            for lane in mine:
                if lane[0] >= len(ts):
                    lane[0] -= len(ts)
                    lane[1].append((i, ts))
                    break
            else:
                mine.append([L - len(ts), [(i, ts)]])
        lanes += [m[1] for m in mine]
        lane_ptr.append(len(lanes))
    slot_row = np.full((Lmax, len(lanes)), -1, np.int64)
    slot_reset = np.zeros((Lmax, len(lanes)), np.uint8)
    for lane, seqs in enumerate(lanes):
        s = 0
        for i, ts in seqs:
            slot_reset[s, lane] = 1
            for t in ts:
                slot_row[s, lane] = t * N + i
                s += 1
    return {"lane_ptr": np.asarray(lane_ptr, np.int64), "slot_row": slot_row, "slot_reset": slot_reset}


def _sig(x):
    return 1.0 / (1.0 + np.exp(-x))


def gru_step(P, x, h, rnn: str = "rnn"):
    """One step of the GRU the paper's time encoders use (Section 6), rows = sequences.  rnn: the
    parameter prefix ("rnn", or "rnn1" for a stacked second layer)."""
    H = h.shape[1]
    gi = x @ P[rnn + ".weight_ih"].T.astype(np.float64) + P[rnn + ".bias_ih"]
    gh = h @ P[rnn + ".weight_hh"].T.astype(np.float64) + P[rnn + ".bias_hh"]
    r = _sig(gi[:, :H] + gh[:, :H])
    z = _sig(gi[:, H:2 * H] + gh[:, H:2 * H])
    n = np.tanh(gi[:, 2 * H:] + r * gh[:, 2 * H:])
    return (1.0 - z) * n + z * h


def lstm_step(P, x, h, c, rnn: str = "rnn"):
    H = h.shape[1]
    g = (x @ P[rnn + ".weight_ih"].T.astype(np.float64) + P[rnn + ".bias_ih"] +
         h @ P[rnn + ".weight_hh"].T.astype(np.float64) + P[rnn + ".bias_hh"])
    i, f, gg, o = _sig(g[:, :H]), _sig(g[:, H:2 * H]), np.tanh(g[:, 2 * H:3 * H]), _sig(g[:, 3 * H:])
    c = f * c + i * gg
    return o * np.tanh(c), c


def state_rows(chunks) -> np.ndarray:
    """First state row of every chunk (rows are (chunk, vertex) in chunk order) and the total."""
    ch = np.asarray(chunks, np.int64).reshape(-1, 4)
    return np.concatenate([[0], np.cumsum(ch[:, 1] - ch[:, 0])])


def run_separate(Z: np.ndarray, present: np.ndarray, chunks, params: dict, time_kind: str, H0=None,
                 return_state: bool = False, n_time_layers: int = 1):
    """Time encoder over every vertex's own sequence, one chunk and one vertex at a time.
    Z [T,N,S] float64: structure-encoder output.  Returns Y [T,N,H], NaN where nothing is computed
    (and, with return_state, HN laid out like H0).  n_time_layers = 2 (Section 6: the two LSTM
    layers of MPNN-LSTM): a second recurrent layer ("rnn1.*") steps through the same sequence on the
    first one's outputs; its state blocks follow the first layer's in H0 / HN; Y is its output."""
    T, N, _ = Z.shape
    H = params["rnn.weight_hh"].shape[1]
    Y = np.full((T, N, H), np.nan)
    ch = np.asarray(chunks, np.int64).reshape(-1, 4)
    off = state_rows(ch)
    V = int(off[-1])
    n_state = 2 if time_kind == "lstm" else 1
    HN = np.zeros((n_time_layers * n_state * V, H)) if H0 is None else np.array(H0, np.float64, copy=True)
    for k, seqs in enumerate(sequences(present, ch)):
        for i, ts in seqs:
            row = int(off[k] + i - ch[k, 0])
            x = [Z[t, i][None] for t in ts]
            for layer in range(n_time_layers):
                base = layer * n_state * V
                rnn = "rnn" if layer == 0 else "rnn1"
                h = HN[base + row][None].copy()
                c = HN[base + V + row][None].copy() if time_kind == "lstm" else np.zeros((1, H))
                out = []
                for xt in x:
                    if time_kind == "gru":
                        h = gru_step(params, xt, h, rnn)
                    else:
                        h, c = lstm_step(params, xt, h, c, rnn)
                    out.append(h)
                HN[base + row] = h[0]
                if time_kind == "lstm":
                    HN[base + V + row] = c[0]
                x = out
            for t, y in zip(ts, x):
                Y[t, i] = y[0]
    return (Y, HN) if return_state else Y


def run_lanes(Z: np.ndarray, packing: dict, params: dict, time_kind: str, chunks=None, H0=None,
              return_state: bool = False):
    """The same over the packed lanes: all lanes step together, slot by slot; on a reset flag the
    incoming state is replaced (the paper's mask) by zero or, with H0, by the state row of the
    sequence that starts there (needs `chunks` to find it).  Results are scattered back to [T,N,H]."""
    T, N, S = Z.shape
    H = params["rnn.weight_hh"].shape[1]
    slot_row, slot_reset = packing["slot_row"], packing["slot_reset"]
    L, n_lanes = slot_row.shape
    Zf = Z.reshape(T * N, S)
    Y = np.full((T * N, H), np.nan)
    h = np.zeros((n_lanes, H))
    c = np.zeros((n_lanes, H))
    srow = None
    if chunks is not None:     # state row of the sequence that occupies each slot
        ch = np.asarray(chunks, np.int64).reshape(-1, 4)
        off = state_rows(ch)
        V = int(off[-1])
        lane_chunk = np.searchsorted(packing["lane_ptr"], np.arange(n_lanes), side="right") - 1
        srow = np.full((L, n_lanes), -1, np.int64)
        for lane in range(n_lanes):
            k = lane_chunk[lane]
            for s in range(L):
                if slot_row[s, lane] >= 0:
                    srow[s, lane] = off[k] + slot_row[s, lane] % N - ch[k, 0]
        n_state = 2 if time_kind == "lstm" else 1
        HN = np.zeros((n_state * V, H)) if H0 is None else np.array(H0, np.float64, copy=True)
    for s in range(L):
        live = slot_row[s] >= 0
        start = slot_reset[s].astype(bool)
        if srow is not None and H0 is not None:
            h[start] = np.asarray(H0, np.float64)[srow[s][start]]
            if time_kind == "lstm":
                c[start] = np.asarray(H0, np.float64)[V + srow[s][start]]
        else:
            h[start] = 0.0
            c[start] = 0.0
        x = np.where(live[:, None], Zf[np.maximum(slot_row[s], 0)], 0.0)
        if time_kind == "gru":
            h = gru_step(params, x, h)
        else:
            h, c = lstm_step(params, x, h, c)
        Y[slot_row[s][live]] = h[live]
        if srow is not None:   # the latest state of every sequence; the last write is its final state
            HN[srow[s][live]] = h[live]
            if time_kind == "lstm":
                HN[V + srow[s][live]] = c[live]
    Y = Y.reshape(T, N, H)
    return (Y, HN) if (return_state and srow is not None) else Y
