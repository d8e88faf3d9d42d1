"""Oracle values for samples of the full-size, device-resident configurations.

TEST INFRASTRUCTURE ONLY (tests/ and bench.py's cpu_baseline leg).  Orchestration: which chunks and
vertices are sampled, copies of the rows the oracle reads (workloads.sampling, workloads.device_gen),
then the unchanged oracle on those copies.  No arithmetic of the method lives here.
"""
from __future__ import annotations

import time

import numpy as np

import oracle
from workloads import sampling
from workloads.device_gen import HostMirror, RowFetcher


def two_layer_reference(data, hg, chunk_ids, subsets, *, input_concat: bool = False, n_time_layers: int = 1):
    """The two-layer GCN + LSTM layer (config 3) for the vertices subsets[i] of chunk chunk_ids[i]:
    returns (want [n, window, H] float32, where [n, 2] = (chunk id, vertex), seconds of oracle time).
    The oracle reads host mirrors that hold exactly the rows it needs, copied from the device."""
    F, S, H = data.F, data.S, data.H
    mx, mc, mc1 = HostMirror(data.X, F), HostMirror(data.C, F), HostMirror(data.C1, S)
    for k, sub in zip(chunk_ids, subsets):
        sampling.fill_two_layer_mirrors(hg, data.chunks[k], sub, mx, mc, mc1)
    sel = np.ascontiguousarray(data.chunks[chunk_ids])
    widths = (data.chunks[:, 1] - data.chunks[:, 0]).astype(np.int64)
    off = np.concatenate([[0], np.cumsum(widths)])
    tot = int(off[-1])
    H0 = None
    if data.H0 is not None:                    # blocks of tot rows: hidden, cell (then the second layer's), packed per chunk
        blocks = int(data.H0.shape[0]) // tot
        H0 = np.ascontiguousarray(np.concatenate(
            [data.H0[b * tot + off[k]:b * tot + off[k + 1]].cpu().numpy() for b in range(blocks) for k in chunk_ids]))
    Y = np.zeros((data.T, data.N, H), np.float32)          # untouched pages stay unallocated
    t0 = time.perf_counter()
    oracle.forward(hg, sel, data.params, mx.host, mc.host, time_kind="lstm", n_struct_layers=2, C1=mc1.host,
                   H0=H0, subset=[np.asarray(s, np.int64) for s in subsets], Y=Y, act_hidden="relu", act_out="none",
                   input_concat=input_concat, n_time_layers=n_time_layers)
    dt = time.perf_counter() - t0
    want, where = [], []
    for k, sub in zip(chunk_ids, subsets):
        t_lo, t_hi = int(data.chunks[k, 2]), int(data.chunks[k, 3])
        for v in np.asarray(sub).tolist():
            want.append(Y[t_lo:t_hi, v].copy())
            where.append((k, v))
    return np.stack(want), np.asarray(where, np.int64), dt


def device_rows(Y_dev, chunks, where, width: int):
    """Rows [n, window, width] of a device tensor [T, N, ld] for the (chunk id, vertex) pairs."""
    out = []
    for k, v in where.tolist():
        out.append(Y_dev[int(chunks[k, 2]):int(chunks[k, 3]), v, :width].cpu().numpy())
    return np.stack(out)


def evolve_forward_reference(data, hg, picks, params):
    """EvolveGCN-O outputs of the sampled (vertex, chunk) pairs, each as a one-vertex chunk of a
    stand-in problem whose copies carry the rows really read.  Returns (want [n][window, S], seconds)."""
    g1, c1, X1, C1 = sampling.one_hop_problem(hg, picks, RowFetcher(data.X, data.F), RowFetcher(data.C, data.F), data.F)
    t0 = time.perf_counter()
    Y = oracle.evolve(g1, c1, params, X1, C1)["Y"]
    dt = time.perf_counter() - t0
    return [Y[ch[2]:ch[3], i] for i, (_, ch) in enumerate(picks)], dt


def evolve_input_gradient_reference(data, hg, picks, params, target_dev, n_real_rows: int):
    """Outputs and input-row gradients (mean-squared-error loss over all n_real_rows covered rows of
    the real problem) of the sampled pairs through the two-hop stand-in problem.  The stand-in's loss
    averages over its own covered rows, so its gradient is rescaled by the ratio of the two counts
    (the mean's denominator is the only thing the sampled rows see of the rest of the problem).
    Returns (ys, dxs, held, seconds): held[i] = [(t, real vertex, oracle output row)] of every row whose
    ReLU gate enters pick i's gradient (the caller compares the gates with the device's)."""
    fx, fc, ft = RowFetcher(data.X, data.F), RowFetcher(data.C, data.F), RowFetcher(target_dev, data.S)
    g1, c1, X1, C1, T1, where, members = sampling.two_hop_problem(
        hg, picks, lambda t, ids: fx[t, ids], lambda t, ids: fc[t, ids], lambda t, ids: ft[t, ids], data.F)
    t0 = time.perf_counter()
    o = oracle.evolve(g1, c1, params, X1, C1, T1, want_dx=True)
    dt = time.perf_counter() - t0
    n_part = int(((c1[:, 1] - c1[:, 0]) * (c1[:, 3] - c1[:, 2])).sum())
    ys = [o["Y"][ch[2]:ch[3], loc] for (_, ch), loc in zip(picks, where.tolist())]
    dxs = [o["dX"][ch[2]:ch[3], loc] * (n_part / n_real_rows) for (_, ch), loc in zip(picks, where.tolist())]
    held = [[(t, j, o["Y"][t, loc]) for t, loc, j in m] for m in members]
    return ys, dxs, held, dt
