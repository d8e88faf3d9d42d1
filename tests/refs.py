"""Independent references used to pin the oracle: dense-adjacency matmuls built from edge
lists (not from the CSR arrays), brute-force packing with Python sets, torch.nn recurrences.
Nothing here is imported by the oracle or by the HIP path."""
from __future__ import annotations

import numpy as np


def dense_norm_adj(N: int, edges) -> np.ndarray:
    """D^-1/2 (A + I) D^-1/2 as a dense float64 matrix from an undirected edge list."""
    A = np.zeros((N, N), np.float64)
    for u, v in edges:
        if u != v:
            A[u, v] = 1.0
            A[v, u] = 1.0
    A += np.eye(N)
    d = A.sum(1)
    return A / np.sqrt(np.outer(d, d))


def edges_of(snapshot) -> list:
    """Undirected edge list of a CSR snapshot (used only to feed dense_norm_adj for graphs
    that come from the generators)."""
    out = []
    rp, cj = snapshot.rowptr, snapshot.col
    for i in range(len(rp) - 1):
        for j in cj[rp[i]:rp[i + 1]]:
            if i < j:
                out.append((i, int(j)))
    return out


def dense_aggregate(Ahat: np.ndarray, x_t: np.ndarray, c_t: np.ndarray, v_lo: int, v_hi: int) -> np.ndarray:
    """Rows v_lo..v_hi of Ahat @ (x inside the range, c outside)."""
    mix = c_t.astype(np.float64).copy()
    mix[v_lo:v_hi] = x_t[v_lo:v_hi]
    return Ahat[v_lo:v_hi] @ mix


def brute_pack(graph, chunks) -> dict:
    """Packing by its definition, with Python sets and lists."""
    row_off, nnz_off, halo_ptr = [0], [0], [0]
    halo_idx, col_local = [], []
    for v_lo, v_hi, t_lo, t_hi in np.asarray(chunks).reshape(-1, 4).tolist():
        for t in range(t_lo, t_hi):
            s = graph.snaps[t]
            cols = [int(j) for i in range(v_lo, v_hi) for j in s.col[s.rowptr[i]:s.rowptr[i + 1]]]
            halo = sorted({j for j in cols if not (v_lo <= j < v_hi)})
            where = {j: k for k, j in enumerate(halo)}
            col_local += [j - v_lo if v_lo <= j < v_hi else (v_hi - v_lo) + where[j] for j in cols]
            halo_idx += halo
            row_off.append(row_off[-1] + v_hi - v_lo)
            nnz_off.append(nnz_off[-1] + len(cols))
            halo_ptr.append(halo_ptr[-1] + len(halo))
    return {"seg_row_off": np.array(row_off, np.int64), "seg_nnz_off": np.array(nnz_off, np.int64),
            "halo_ptr": np.array(halo_ptr, np.int64), "halo_idx": np.array(halo_idx, np.int32),
            "col_local": np.array(col_local, np.int32)}


def parity(got: np.ndarray, want: np.ndarray) -> dict:
    """The error figures every comparison reports: the floored relative error at tau = 1e-2 RMS
    and at tau = 1e-1 RMS (max |got - want| / max(|want|, tau)), the plain largest absolute error
    in units of RMS(want), and the 99.9th percentile of the unfloored relative error."""
    got = np.asarray(got, np.float64).ravel()
    want = np.asarray(want, np.float64).ravel()
    if not want.size:
        return {"floor_1e-2": 0.0, "floor_1e-1": 0.0, "max_abs_over_rms": 0.0, "p999_rel": 0.0}
    rms = max(float(np.sqrt(np.mean(want * want))), 1e-300)
    d = np.abs(got - want)
    a = np.abs(want)
    nz = a > 0
    return {"floor_1e-2": float(np.max(d / np.maximum(a, 1e-2 * rms))),
            "floor_1e-1": float(np.max(d / np.maximum(a, 1e-1 * rms))),
            "max_abs_over_rms": float(d.max() / rms),
            "p999_rel": float(np.quantile(d[nz] / a[nz], 0.999)) if nz.any() else 0.0}


def parity_str(got: np.ndarray, want: np.ndarray) -> str:
    p = parity(got, want)
    return (f"rel err floored at 1e-2 RMS {p['floor_1e-2']:.2e}, at 1e-1 RMS {p['floor_1e-1']:.2e}; "
            f"max abs / RMS {p['max_abs_over_rms']:.2e}; p99.9 unfloored rel {p['p999_rel']:.2e}")


def rel_err(got: np.ndarray, want: np.ndarray, floor: float = 1e-1) -> float:
    """max |got - want| / max(|want|, tau), tau = floor * RMS(want): the elementwise relative
    error with a floor, since a plain relative error is unbounded near zero.  floor = 0.1 for
    fp32 paths; 1.0 for bf16 paths, whose stored intermediates carry an absolute error of a few
    2^-9 * RMS whatever the size of the element they end up in."""
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    tau = floor * float(np.sqrt(np.mean(want * want))) if want.size else 0.0
    den = np.maximum(np.abs(want), max(tau, 1e-300))
    return float(np.max(np.abs(got - want) / den)) if want.size else 0.0
