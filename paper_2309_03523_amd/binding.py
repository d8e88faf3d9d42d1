"""Thin ctypes binding of libdgc (include/dgc.h): argument marshalling only.

Every step of the path runs inside the HIP library.  PyTorch supplies device memory and the
stream.  There is no CPU fallback: if the library has not been built, or no GPU is present,
the calls raise.
"""
from __future__ import annotations

import ctypes as ct
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdgc.so")

TIME_KIND = {"none": 0, "gru": 1, "lstm": 2, "self_attn": 3}
ACT = {"none": 0, "relu": 1}
GATHER = {"in_place": 0, "staged": 1}
DENSE = {"auto": 0, "tile": 1, "wave": 2}
AGG = {"table": 0, "walk": 1}
STRUCT = {"gcn": 0, "evolve_gcn_o": 1, "gat": 2}
DTYPE = {"f32": 0, "bf16": 1}

STATUS = {0: "DGC_OK", 1: "DGC_ERR_INVALID_ARG", 2: "DGC_ERR_BAD_GRAPH", 3: "DGC_ERR_BAD_CHUNK",
          4: "DGC_ERR_UNSUPPORTED", 5: "DGC_ERR_OOM", 6: "DGC_ERR_DEVICE", 7: "DGC_ERR_STATE"}

EXPORTS = ["dgc_layer_create", "dgc_layer_destroy", "dgc_layer_set_param", "dgc_layer_get_param",
           "dgc_layer_forward", "dgc_layer_backward", "dgc_layer_aggregate", "dgc_layer_gather",
           "dgc_layer_packing", "dgc_layer_set_presence", "dgc_layer_set_labels", "dgc_layer_set_profiling", "dgc_layer_stage_times", "dgc_last_error",
           "dgc_version", "dgc_stale_theta_factor", "dgc_stale_workspace_bytes", "dgc_stale_filter",
           "dgc_stale_static_max_candidates", "dgc_stale_filter_static",
           "dgc_layer_shared_rows", "dgc_fusion_select", "dgc_chunk_assign", "dgc_chunk_generate"]
THETA_VARIANT = {"printed": 0, "sigmoid": 1}
N_STAGES = 13


class DgcError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{STATUS.get(code, code)}: {text}")
        self.code = code


class ChunkT(ct.Structure):
    _fields_ = [("v_lo", ct.c_int64), ("v_hi", ct.c_int64), ("t_lo", ct.c_int32), ("t_hi", ct.c_int32)]


class GraphT(ct.Structure):
    _fields_ = [("T", ct.c_int32), ("N", ct.c_int64),
                ("rowptr", ct.POINTER(ct.c_void_p)), ("colidx", ct.POINTER(ct.c_void_p))]


class DescT(ct.Structure):
    _fields_ = [(n, ct.c_int32) for n in
                ("struct_kind", "n_struct_layers", "time_kind", "dtype", "F", "S", "H", "act_hidden",
                 "act_out", "gather_mode", "validate_level", "rows_per_group", "long_nnz", "part_nnz",
                 "dense_kernel", "heads", "lstm_input_concat", "agg_kernel", "n_time_layers")]


_lib = None


def load() -> ct.CDLL:
    """Load libdgc.so (built in-tree by __graft_entry__.build()).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = ct.CDLL(LIB_PATH)
    vp, i32, i64 = ct.c_void_p, ct.c_int32, ct.c_int64
    lib.dgc_layer_create.argtypes = [ct.POINTER(DescT), ct.POINTER(GraphT), ct.POINTER(ChunkT), i32, vp,
                                     ct.POINTER(vp)]
    lib.dgc_layer_destroy.argtypes = [vp]
    lib.dgc_layer_set_param.argtypes = [vp, ct.c_char_p, vp, i64]
    lib.dgc_layer_get_param.argtypes = [vp, ct.c_char_p, vp, i64]
    lib.dgc_layer_forward.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp, vp, vp, i64, vp, vp]
    lib.dgc_layer_backward.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp, vp, i64, vp]
    lib.dgc_layer_aggregate.argtypes = [vp, vp, i64, vp, i64, vp, i64, vp]
    lib.dgc_layer_gather.argtypes = [vp, vp, i64, vp, i64, vp]
    lib.dgc_layer_packing.argtypes = [vp, ct.c_char_p, vp, i64, ct.POINTER(i64)]
    lib.dgc_layer_set_presence.argtypes = [vp, vp, vp]
    lib.dgc_layer_set_labels.argtypes = [vp, vp, vp]
    lib.dgc_layer_set_profiling.argtypes = [vp, i32]
    lib.dgc_layer_stage_times.argtypes = [vp, vp]
    lib.dgc_last_error.argtypes = [vp]
    lib.dgc_last_error.restype = ct.c_char_p
    lib.dgc_version.restype = ct.c_char_p
    lib.dgc_chunk_generate.argtypes = [ct.POINTER(GraphT), i32, i32, i64, i32, vp, ct.POINTER(i32), ct.POINTER(i32), vp]
    lib.dgc_layer_shared_rows.argtypes = [vp, vp, vp]
    lib.dgc_fusion_select.argtypes = [i32, vp, vp, i64, vp]
    lib.dgc_chunk_assign.argtypes = [i32, vp, vp, i32, vp]
    lib.dgc_stale_theta_factor.argtypes = [ct.c_double, ct.c_double, i32]
    lib.dgc_stale_theta_factor.restype = ct.c_double
    lib.dgc_stale_workspace_bytes.argtypes = [i64]
    lib.dgc_stale_workspace_bytes.restype = i64
    lib.dgc_stale_filter.argtypes = [vp, i64, vp, i64, i64, i32, i32, vp, i64, ct.c_double, ct.c_double, vp, vp, vp, i64,
                                     vp, vp, i64, vp]
    lib.dgc_stale_filter_static.argtypes = [vp, i64, vp, i64, i64, i32, i32, vp, i64, ct.c_double, ct.c_double, vp, vp, vp,
                                            i64, vp, vp]
    lib.dgc_stale_static_max_candidates.argtypes = []
    lib.dgc_stale_static_max_candidates.restype = i64
    for name in EXPORTS:
        if name not in ("dgc_last_error", "dgc_version", "dgc_stale_theta_factor", "dgc_stale_workspace_bytes",
                        "dgc_stale_static_max_candidates"):
            getattr(lib, name).restype = ct.c_int
    _lib = lib
    return lib


def version() -> str:
    return load().dgc_version().decode()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ct.c_void_p(stream.cuda_stream)


def _dev(t, name: str):
    """Device pointer of a contiguous-in-the-last-dim CUDA tensor (or None)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    return ct.c_void_p(t.data_ptr())


def _ld(t, name: str) -> int:
    if t is None:
        return 0
    if t.dim() != 3 or t.stride(2) != 1 or t.stride(0) != t.shape[1] * t.stride(1):
        raise ValueError(f"{name} must be [T,N,ld] row-major (last dim contiguous, no gap between snapshots)")
    return int(t.stride(1))


_PACK_DTYPES = {"seg_row_off": np.int64, "seg_nnz_off": np.int64, "halo_ptr": np.int64,
                "halo_idx": np.int32, "col_local": np.int32, "work_short": np.int32,
                "work_long": np.int32, "deg_inv_sqrt": np.float32, "lane_ptr": np.int64, "slot_row": np.int64,
                "slot_reset": np.uint8}


class DgcLayer:
    """dgc_layer_create / forward / backward / destroy with torch tensors as arguments.

    rowptr, colidx: lists of T device tensors (int64 [N+1], int32 [nnz_t]).
    chunks: array-like [n,4] of (v_lo, v_hi, t_lo, t_hi).
    """

    def __init__(self, rowptr, colidx, N: int, chunks, *, F: int, S: int, H: int, time_kind: str = "gru",
                 n_struct_layers: int = 1, act_hidden: str = "relu", act_out: str = "none",
                 gather_mode: str = "in_place", validate_level: int = 0, rows_per_group: int = 0,
                 long_nnz: int = 0, part_nnz: int = 0, dense_kernel: str = "auto", struct_kind: str = "gcn",
                 dtype: str = "f32", heads: int = 0, lstm_input_concat: bool = False, agg_kernel: str = "table",
                 n_time_layers: int = 1, stream=None):
        import torch
        lib = load()
        self._lib = lib
        self._h = ct.c_void_p(None)
        T = len(rowptr)
        for r, c in zip(rowptr, colidx):
            if r.dtype != torch.int64 or c.dtype != torch.int32 or not r.is_cuda or not c.is_cuda:
                raise ValueError("rowptr must be int64 and colidx int32 device tensors")
            if not r.is_contiguous() or not c.is_contiguous():
                raise ValueError("CSR arrays must be contiguous")
        self._keep = (list(rowptr), list(colidx))  # the layer borrows the CSR arrays for its life
        rp = (ct.c_void_p * T)(*[r.data_ptr() for r in rowptr])
        cj = (ct.c_void_p * T)(*[c.data_ptr() for c in colidx])
        graph = GraphT(T, N, rp, cj)
        ch = np.asarray(chunks, np.int64).reshape(-1, 4)
        carr = (ChunkT * len(ch))(*[ChunkT(int(a), int(b), int(c), int(d)) for a, b, c, d in ch])
        desc = DescT(STRUCT[struct_kind], n_struct_layers, TIME_KIND[time_kind], DTYPE[dtype], F, S, H, ACT[act_hidden],
                     ACT[act_out],
                     GATHER[gather_mode], validate_level, rows_per_group, long_nnz, part_nnz, DENSE[dense_kernel],
                     heads, int(lstm_input_concat), AGG[agg_kernel], int(n_time_layers))
        rc = lib.dgc_layer_create(ct.byref(desc), ct.byref(graph), carr, len(ch), _stream_ptr(stream),
                                  ct.byref(self._h))
        if rc:
            raise DgcError(rc, lib.dgc_last_error(None).decode())
        self.T, self.N, self.F, self.S, self.H = T, N, F, S, H
        self.time_kind, self.n_struct_layers, self.n_time_layers = time_kind, n_struct_layers, n_time_layers
        self.chunks = ch
        self.out_dim = H if time_kind in ("gru", "lstm") else S

    # -- lifetime
    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.dgc_layer_destroy(self._h)
            self._h = ct.c_void_p(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc:
            raise DgcError(rc, self._lib.dgc_last_error(self._h).decode())

    # -- parameters
    def set_param(self, name: str, value: np.ndarray):
        v = np.ascontiguousarray(value, np.float32)
        self._check(self._lib.dgc_layer_set_param(self._h, name.encode(), v.ctypes.data_as(ct.c_void_p), v.size))

    def set_params(self, params: dict):
        for k, v in params.items():
            self.set_param(k, v)

    def get_param(self, name: str, shape) -> np.ndarray:
        out = np.zeros(shape, np.float32)
        self._check(self._lib.dgc_layer_get_param(self._h, name.encode(), out.ctypes.data_as(ct.c_void_p), out.size))
        return out

    # -- the path
    def forward(self, X, C, Y, *, C1=None, H0=None, reset_mask=None, HN=None, stream=None):
        self._check(self._lib.dgc_layer_forward(
            self._h, _dev(X, "X"), _ld(X, "X"), _dev(C, "C"), _ld(C, "C"), _dev(C1, "C1"), _ld(C1, "C1"),
            _dev(H0, "H0"), _dev(reset_mask, "reset_mask"), _dev(Y, "Y"), _ld(Y, "Y"), _dev(HN, "HN"),
            _stream_ptr(stream)))
        return Y

    def backward(self, Y, *, dY=None, target=None, loss_out=None, dX=None, stream=None):
        self._check(self._lib.dgc_layer_backward(
            self._h, _dev(Y, "Y"), _ld(Y, "Y"), _dev(dY, "dY"), _ld(dY, "dY"), _dev(target, "target"),
            _ld(target, "target"), _dev(loss_out, "loss_out"), _dev(dX, "dX"), _ld(dX, "dX"), _stream_ptr(stream)))

    def set_presence(self, present, stream=None):
        """present: uint8 device tensor [T,N]; switches the layer to temporal fusion (on a layer that has
        labels: over the runs of present instances with one label; labels are set first)."""
        if not present.is_cuda or present.dtype.itemsize != 1 or not present.is_contiguous():
            raise ValueError("present must be a contiguous uint8 device tensor [T,N]")
        self._check(self._lib.dgc_layer_set_presence(self._h, _dev(present, "present"), _stream_ptr(stream)))

    def set_labels(self, labels, stream=None):
        """labels: int32 device tensor [T*N] (or [T,N]), e.g. chunk_generate's output; the layer then
        runs over the generated chunks."""
        import torch
        if not labels.is_cuda or labels.dtype != torch.int32 or not labels.is_contiguous() or labels.numel() != self.T * self.N:
            raise ValueError("labels must be a contiguous int32 device tensor with T*N entries")
        self._check(self._lib.dgc_layer_set_labels(self._h, _dev(labels, "labels"), _stream_ptr(stream)))

    def aggregate(self, X, C, M, stream=None):
        self._check(self._lib.dgc_layer_aggregate(self._h, _dev(X, "X"), _ld(X, "X"), _dev(C, "C"), _ld(C, "C"),
                                                  _dev(M, "M"), int(M.stride(0)), _stream_ptr(stream)))
        return M

    def gather(self, C, halo, stream=None):
        self._check(self._lib.dgc_layer_gather(self._h, _dev(C, "C"), _ld(C, "C"), _dev(halo, "halo"),
                                               int(halo.stride(0)), _stream_ptr(stream)))
        return halo

    def shared_rows(self, stream=None) -> np.ndarray:
        """int64 [n_chunks, n_chunks]: rows every pair of chunks would load twice."""
        n = len(self.chunks)
        out = np.zeros((n, n), np.int64)
        self._check(self._lib.dgc_layer_shared_rows(self._h, out.ctypes.data_as(ct.c_void_p), _stream_ptr(stream)))
        return out

    # -- measurement
    def set_profiling(self, enable: bool):
        self._check(self._lib.dgc_layer_set_profiling(self._h, int(bool(enable))))

    def stage_times(self) -> np.ndarray:
        """Milliseconds per stage of the last profiled forward (waits for it)."""
        out = np.zeros(N_STAGES, np.float32)
        self._check(self._lib.dgc_layer_stage_times(self._h, out.ctypes.data_as(ct.c_void_p)))
        return out

    # -- inspection
    def packing(self, what: str) -> np.ndarray:
        need = ct.c_int64(0)
        rc = self._lib.dgc_layer_packing(self._h, what.encode(), None, 0, ct.byref(need))
        if rc not in (0, 1):     # 1 = destination too small: the size query itself
            self._check(rc)
        dt = np.dtype(_PACK_DTYPES[what])
        out = np.zeros(need.value // dt.itemsize, dt)
        if out.size:
            self._check(self._lib.dgc_layer_packing(self._h, what.encode(), out.ctypes.data_as(ct.c_void_p),
                                                    out.nbytes, ct.byref(need)))
        if what == "work_short":
            out = out.reshape(-1, 3)
        if what == "work_long":
            out = out.reshape(-1, 4)
        return out


# --------------------------------------------------------------------------- stale filter

STALE_RESULT_DTYPE = np.dtype([("n_send", np.int64), ("D", np.float32), ("theta", np.float32),
                               ("n_invalid", np.int64)])


def stale_theta_factor(l1: float, l_prev: float, variant: str = "printed") -> float:
    f = load().dgc_stale_theta_factor(float(l1), float(l_prev), THETA_VARIANT[variant])
    if f < 0:
        raise ValueError("stale_theta_factor: l1 must be > 0 and l_prev finite")
    return f


def stale_workspace_bytes(n_candidates: int) -> int:
    return int(load().dgc_stale_workspace_bytes(int(n_candidates)))


def stale_static_max_candidates() -> int:
    return int(load().dgc_stale_static_max_candidates())


def stale_filter(E, L, *, F=None, rows=None, n_rows=None, factor=None, theta=None, dist, send_idx, send_buf=None, result,
                 workspace=None, stream=None):
    """dgc_stale_filter on device tensors: E, L [R, ld] fp32 or bfloat16; rows int64 or None (n_rows: how many of
    its entries count, default all; torch gives an empty tensor a NULL pointer, so an empty list is a
    non-empty tensor with n_rows = 0); dist fp32 and
    send_idx int64 with one entry per candidate; send_buf [n, ld] or None; result: 24-byte device
    tensor (view it with STALE_RESULT_DTYPE after a synchronisation); workspace: device bytes, or
    None for dgc_stale_filter_static (the library's own fixed scratch, nothing allocated).
    Exactly one of factor / theta.  Only enqueues."""
    if (factor is None) == (theta is None):
        raise ValueError("give exactly one of factor and theta")
    for name, t in (("E", E), ("L", L)):
        if t.dim() != 2 or t.stride(1) != 1:
            raise ValueError(f"{name} must be [R, ld] with a contiguous last dimension")
    if E.dtype != L.dtype or (send_buf is not None and send_buf.dtype != E.dtype):
        raise ValueError("E, L and send_buf must have the same element type")
    lib = load()
    head = (_dev(E, "E"), int(E.stride(0)), _dev(L, "L"), int(L.stride(0)), int(E.shape[0]),
            int(E.shape[1] if F is None else F), DTYPE["bf16" if E.element_size() == 2 else "f32"], _dev(rows, "rows"),
            0 if rows is None else int(rows.numel() if n_rows is None else n_rows),
            -1.0 if factor is None else float(factor), 0.0 if theta is None else float(theta), _dev(dist, "dist"),
            _dev(send_idx, "send_idx"), _dev(send_buf, "send_buf"), 0 if send_buf is None else int(send_buf.stride(0)),
            _dev(result, "result"))
    if workspace is None:
        rc = lib.dgc_stale_filter_static(*head, _stream_ptr(stream))
    else:
        rc = lib.dgc_stale_filter(*head, _dev(workspace, "workspace"),
                                  int(workspace.numel() * workspace.element_size()), _stream_ptr(stream))
    if rc != 0:
        raise DgcError(rc, lib.dgc_last_error(None).decode())


# --------------------------------------------------------------------------- fusion selection, assignment


def fusion_select(shared: np.ndarray, mem: np.ndarray, cap: int) -> np.ndarray:
    shared = np.ascontiguousarray(shared, np.int64)
    mem = np.ascontiguousarray(mem, np.int64)
    n = mem.size
    if shared.shape != (n, n):
        raise ValueError("shared must be [n, n]")
    out = np.zeros(n, np.int32)
    lib = load()
    rc = lib.dgc_fusion_select(n, shared.ctypes.data_as(ct.c_void_p), mem.ctypes.data_as(ct.c_void_p), int(cap),
                               out.ctypes.data_as(ct.c_void_p))
    if rc != 0:
        raise DgcError(rc, lib.dgc_last_error(None).decode())
    return out


def chunk_assign(g: np.ndarray, h: np.ndarray, n_gpus: int) -> np.ndarray:
    g = np.ascontiguousarray(g, np.float64)
    h = np.ascontiguousarray(h, np.float64)
    n = g.size
    if h.shape != (n, n):
        raise ValueError("h must be [n, n]")
    out = np.zeros(n, np.int32)
    lib = load()
    rc = lib.dgc_chunk_assign(n, g.ctypes.data_as(ct.c_void_p), h.ctypes.data_as(ct.c_void_p), int(n_gpus),
                              out.ctypes.data_as(ct.c_void_p))
    if rc != 0:
        raise DgcError(rc, lib.dgc_last_error(None).decode())
    return out


# --------------------------------------------------------------------------- chunk generation


def chunk_generate(rowptr, colidx, N: int, *, w_s: int, w_t: int, cap: int, max_iters: int, labels, stream=None):
    """dgc_chunk_generate: rowptr / colidx lists of T device tensors, labels int32 device tensor
    [T*N] (written).  Returns (iterations, converged)."""
    T = len(rowptr)
    rp = (ct.c_void_p * T)(*[r.data_ptr() for r in rowptr])
    cj = (ct.c_void_p * T)(*[c.data_ptr() for c in colidx])
    graph = GraphT(T, N, rp, cj)
    if labels.numel() != T * N or labels.element_size() != 4 or not labels.is_contiguous():
        raise ValueError("labels must be a contiguous int32 device tensor of T*N elements")
    it, conv = ct.c_int32(0), ct.c_int32(0)
    lib = load()
    rc = lib.dgc_chunk_generate(ct.byref(graph), int(w_s), int(w_t), int(cap), int(max_iters), _dev(labels, "labels"),
                                ct.byref(it), ct.byref(conv), _stream_ptr(stream))
    if rc != 0:
        raise DgcError(rc, lib.dgc_last_error(None).decode())
    return it.value, bool(conv.value)
