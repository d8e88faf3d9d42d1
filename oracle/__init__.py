"""Python face of the CPU oracle (oracle/dgc_oracle.c).

TEST INFRASTRUCTURE ONLY.  Imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py; never by the product package.  It marshals NumPy arrays into
the C functions and holds no arithmetic of its own.
"""
from __future__ import annotations

import ctypes as ct
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dgc_oracle.c")
_LIB = os.path.join(_HERE, "_build", "libdgc_oracle.so")

TIME_KIND = {"none": 0, "gru": 1, "lstm": 2}
ACT = {"none": 0, "relu": 1}


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP over rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        os.makedirs(os.path.dirname(_LIB), exist_ok=True)
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ct.CDLL:
    global _lib
    if _lib is None:
        _lib = ct.CDLL(build())
        _lib.dgc_oracle_num_segments.restype = ct.c_int64
    return _lib


def threads() -> int:
    return int(lib().dgc_oracle_threads())


def set_threads(n: int) -> None:
    """Number of OpenMP threads the oracle's row loops use from now on (bench.py times it on one
    core and on all of them); the arithmetic does not depend on it."""
    lib()
    ct.CDLL("libgomp.so.1").omp_set_num_threads(ct.c_int(int(n)))


def _p(a: Optional[np.ndarray], ctype):
    if a is None:
        return ct.cast(None, ct.POINTER(ctype))
    assert a.flags["C_CONTIGUOUS"], "oracle arguments must be C-contiguous"
    return a.ctypes.data_as(ct.POINTER(ctype))


class _Csr:
    """Arrays of per-snapshot pointers; keeps the NumPy arrays alive."""

    def __init__(self, graph):
        self.T = graph.T
        self.N = graph.N
        self.keep = [(np.ascontiguousarray(s.rowptr, np.int64), np.ascontiguousarray(s.col, np.int32))
                     for s in graph.snaps]
        self.rowptr = (ct.POINTER(ct.c_int64) * self.T)(*[_p(r, ct.c_int64) for r, _ in self.keep])
        self.col = (ct.POINTER(ct.c_int32) * self.T)(*[_p(c, ct.c_int32) for _, c in self.keep])


def _chunks(chunks) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(chunks, np.int64).reshape(-1, 4))


def pack(graph, chunks) -> dict:
    """Segment offsets, halo lists and local column ids of the fused batch."""
    g = _Csr(graph)
    ch = _chunks(chunks)
    nseg = int(lib().dgc_oracle_num_segments(_p(ch, ct.c_int64), ct.c_int32(len(ch))))
    row_off = np.zeros(nseg + 1, np.int64)
    nnz_off = np.zeros(nseg + 1, np.int64)
    halo_ptr = np.zeros(nseg + 1, np.int64)

    def call(halo_idx, col_local):
        rc = lib().dgc_oracle_pack(ct.c_int32(g.T), ct.c_int64(g.N), g.rowptr, g.col,
                                   _p(ch, ct.c_int64), ct.c_int32(len(ch)), _p(row_off, ct.c_int64),
                                   _p(nnz_off, ct.c_int64), _p(halo_ptr, ct.c_int64),
                                   _p(halo_idx, ct.c_int32), _p(col_local, ct.c_int32))
        if rc:
            raise ValueError(f"dgc_oracle_pack failed: {rc}")

    call(None, None)
    halo_idx = np.zeros(int(halo_ptr[-1]), np.int32)
    col_local = np.zeros(int(nnz_off[-1]), np.int32)
    call(halo_idx, col_local)
    return {"seg_row_off": row_off, "seg_nnz_off": nnz_off, "halo_ptr": halo_ptr,
            "halo_idx": halo_idx, "col_local": col_local}


def worklist(graph, chunks, rows_per_group: int, long_nnz: int, part_nnz: int) -> dict:
    g = _Csr(graph)
    ch = _chunks(chunks)
    ns, nl = ct.c_int64(0), ct.c_int64(0)

    def call(sl, ll):
        rc = lib().dgc_oracle_worklist(ct.c_int32(g.T), ct.c_int64(g.N), g.rowptr, _p(ch, ct.c_int64),
                                       ct.c_int32(len(ch)), ct.c_int32(rows_per_group),
                                       ct.c_int32(long_nnz), ct.c_int32(part_nnz),
                                       _p(sl, ct.c_int32), ct.byref(ns), _p(ll, ct.c_int32), ct.byref(nl))
        if rc:
            raise ValueError(f"dgc_oracle_worklist failed: {rc}")

    call(None, None)
    sl = np.zeros((ns.value, 3), np.int32)
    ll = np.zeros((nl.value, 4), np.int32)
    call(sl, ll)
    return {"work_short": sl, "work_long": ll}


def aggregate_chunk(graph, chunk, X: np.ndarray, C: np.ndarray) -> np.ndarray:
    """Normalised neighbour aggregation for one chunk: float64 [w, nv, F]."""
    g = _Csr(graph)
    ch = _chunks(chunk)
    assert len(ch) == 1
    v_lo, v_hi, t_lo, t_hi = (int(x) for x in ch[0])
    F = X.shape[-1]
    M = np.zeros((t_hi - t_lo, v_hi - v_lo, F), np.float64)
    rc = lib().dgc_oracle_aggregate_chunk(ct.c_int32(g.T), ct.c_int64(g.N), g.rowptr, g.col,
                                          _p(ch, ct.c_int64), _p(X, ct.c_float), ct.c_int64(X.strides[1] // 4),
                                          _p(C, ct.c_float), ct.c_int64(C.strides[1] // 4), ct.c_int32(F),
                                          _p(M, ct.c_double))
    if rc:
        raise ValueError(f"dgc_oracle_aggregate_chunk failed: {rc}")
    return M


def forward(graph, chunks, params: dict, X: np.ndarray, C: np.ndarray, *, time_kind: str = "gru",
            n_struct_layers: int = 1, act_hidden: str = "relu", act_out: str = "none",
            C1: Optional[np.ndarray] = None, H0: Optional[np.ndarray] = None,
            reset_mask: Optional[np.ndarray] = None, subset: Optional[list] = None,
            Y: Optional[np.ndarray] = None, return_state: bool = False, input_concat: bool = False,
            n_time_layers: int = 1):
    """The whole layer over the listed chunks.  Returns Y float32 [T,N,out_dim] (rows not
    covered by a chunk, or outside `subset`, keep the value they had in the `Y` passed in,
    NaN if none was passed) and optionally the final recurrent states packed like H0.
    input_concat (two structure layers): the time encoder reads both layers' outputs side by
    side, first layer first (Section 6, MPNN-LSTM); rnn.weight_ih is then [gH, 2S].
    n_time_layers = 2: a second recurrent layer ("rnn1.*", input width H) reads the first one's
    output; Y is its output, and H0 / the returned states hold the first layer's blocks followed
    by the second layer's."""
    g = _Csr(graph)
    ch = _chunks(chunks)
    T, N = g.T, g.N
    W0 = np.ascontiguousarray(params["gcn0.weight"], np.float32)
    b0 = np.ascontiguousarray(params["gcn0.bias"], np.float32)
    S, F = W0.shape
    assert X.shape == (T, N, F) and C.shape == (T, N, F)
    W1 = b1 = None
    if n_struct_layers == 2:
        W1 = np.ascontiguousarray(params["gcn1.weight"], np.float32)
        b1 = np.ascontiguousarray(params["gcn1.bias"], np.float32)
        assert C1 is not None and C1.shape == (T, N, S)
    Wih = Whh = bih = bhh = None
    H = S
    if time_kind != "none":
        Wih = np.ascontiguousarray(params["rnn.weight_ih"], np.float32)
        Whh = np.ascontiguousarray(params["rnn.weight_hh"], np.float32)
        bih = np.ascontiguousarray(params["rnn.bias_ih"], np.float32)
        bhh = np.ascontiguousarray(params["rnn.bias_hh"], np.float32)
        H = Whh.shape[1]
        gH = {"gru": 3, "lstm": 4}[time_kind] * H
        assert Wih.shape == (gH, 2 * S if input_concat else S) and Whh.shape == (gH, H)
    assert not input_concat or (n_struct_layers == 2 and time_kind != "none")
    out_dim = H if time_kind != "none" else S
    if Y is None:
        Y = np.full((T, N, out_dim), np.nan, np.float32)
    assert Y.shape == (T, N, out_dim) and Y.dtype == np.float32
    tot_v = int((ch[:, 1] - ch[:, 0]).sum())
    n_state = (2 if time_kind == "lstm" else 1) * n_time_layers
    W2 = None
    if n_time_layers == 2:
        assert time_kind != "none"
        W2 = [np.ascontiguousarray(params[k], np.float32)
              for k in ("rnn1.weight_ih", "rnn1.weight_hh", "rnn1.bias_ih", "rnn1.bias_hh")]
        assert W2[0].shape == (gH, H) and W2[1].shape == (gH, H)
    if H0 is not None:
        H0 = np.ascontiguousarray(H0, np.float32)
        assert H0.shape == (n_state * tot_v, H)
    if reset_mask is not None:
        reset_mask = np.ascontiguousarray(reset_mask, np.uint8)
        assert reset_mask.shape == (T, N)
    sub_ptr = sub_idx = None
    if subset is not None:
        assert len(subset) == len(ch)
        sub_ptr = np.zeros(len(ch) + 1, np.int64)
        sub_ptr[1:] = np.cumsum([len(s) for s in subset])
        sub_idx = np.ascontiguousarray(np.concatenate([np.asarray(s, np.int64) for s in subset])
                                       if sub_ptr[-1] else np.zeros(0, np.int64))
    hN = np.zeros((n_state * tot_v, H), np.float32) if (return_state and time_kind != "none") else None
    args_tail = [ct.c_int32(int(input_concat))]
    fn = lib().dgc_oracle_forward
    if n_time_layers == 2:
        fn = lib().dgc_oracle_forward_stacked
        args_tail += [_p(a, ct.c_float) for a in W2]
    rc = fn(
        ct.c_int32(T), ct.c_int64(N), g.rowptr, g.col, _p(ch, ct.c_int64), ct.c_int32(len(ch)),
        ct.c_int32(n_struct_layers), ct.c_int32(TIME_KIND[time_kind]), ct.c_int32(ACT[act_hidden]),
        ct.c_int32(ACT[act_out]), ct.c_int32(F), ct.c_int32(S), ct.c_int32(H),
        _p(X, ct.c_float), ct.c_int64(X.strides[1] // 4), _p(C, ct.c_float), ct.c_int64(C.strides[1] // 4),
        _p(C1, ct.c_float), ct.c_int64(C1.strides[1] // 4 if C1 is not None else 0),
        _p(W0, ct.c_float), _p(b0, ct.c_float), _p(W1, ct.c_float), _p(b1, ct.c_float),
        _p(Wih, ct.c_float), _p(Whh, ct.c_float), _p(bih, ct.c_float), _p(bhh, ct.c_float),
        _p(H0, ct.c_float), _p(reset_mask, ct.c_uint8), _p(sub_ptr, ct.c_int64), _p(sub_idx, ct.c_int64),
        _p(Y, ct.c_float), ct.c_int64(Y.strides[1] // 4), _p(hN, ct.c_float), *args_tail)
    if rc:
        raise ValueError(f"dgc_oracle_forward failed: {rc}")
    return (Y, hN) if return_state else Y


EVOLVE_PARAMS = ["evolve.W_init", "evolve.U_z", "evolve.V_z", "evolve.B_z", "evolve.U_r", "evolve.V_r",
                 "evolve.B_r", "evolve.U_h", "evolve.V_h", "evolve.B_h"]


def evolve(graph, chunks, params: dict, X: np.ndarray, C: np.ndarray, target: Optional[np.ndarray] = None,
           want_grads: bool = False, Y: Optional[np.ndarray] = None, want_dx: bool = False):
    """EvolveGCN-O layer: weights evolved by a matrix GRU, Y = relu(M W_t), mean-squared-error loss.
    Returns dict(Y, loss, grads {name: float64 array}, Wt [T,F,S], dX [T,N,F] float64 if want_dx)."""
    g = _Csr(graph)
    ch = _chunks(chunks)
    T, N = g.T, g.N
    P = [np.ascontiguousarray(params[k], np.float64) for k in EVOLVE_PARAMS]
    F, S = P[0].shape
    assert X.shape == (T, N, F) and C.shape == (T, N, F)
    parr = (ct.POINTER(ct.c_double) * 10)(*[_p(a, ct.c_double) for a in P])
    if Y is None:
        Y = np.full((T, N, S), np.nan, np.float32)
    grads = [np.zeros_like(a) for a in P] if want_grads else None
    garr = (ct.POINTER(ct.c_double) * 10)(*[_p(a, ct.c_double) for a in grads]) if want_grads else None
    Wt = np.zeros((T, F, S), np.float64)
    dX = np.zeros((T, N, F), np.float64) if want_dx else None
    loss = ct.c_double(0.0)
    if target is not None:
        target = np.ascontiguousarray(target, np.float32)
        assert target.shape == (T, N, S)
    rc = lib().dgc_oracle_evolve(
        ct.c_int32(T), ct.c_int64(N), g.rowptr, g.col, _p(ch, ct.c_int64), ct.c_int32(len(ch)), ct.c_int32(F),
        ct.c_int32(S), _p(X, ct.c_float), ct.c_int64(X.strides[1] // 4), _p(C, ct.c_float),
        ct.c_int64(C.strides[1] // 4), parr, _p(target, ct.c_float),
        ct.c_int64(target.strides[1] // 4 if target is not None else 0), _p(Y, ct.c_float),
        ct.c_int64(Y.strides[1] // 4), ct.byref(loss), garr, _p(Wt, ct.c_double), _p(dX, ct.c_double))
    if rc:
        raise ValueError(f"dgc_oracle_evolve failed: {rc}")
    return {"Y": Y, "loss": loss.value, "Wt": Wt, "dX": dX,
            "grads": dict(zip(EVOLVE_PARAMS, grads)) if want_grads else None}
