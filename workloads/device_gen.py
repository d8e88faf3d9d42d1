"""Seeded generators that draw the large configurations directly in GPU memory (torch on the
device), for the sizes at which drawing on the host and uploading takes many minutes and tens
of gigabytes of host memory.  Same recipes as workloads/synth.py (Chung-Lu power-law
snapshots, N(0,1) features, cache = features + 0.1 N(0,1)), other random streams: the values
differ from the host generators', the distributions do not.

Only inputs are drawn here; none of the layer's arithmetic.  The CPU oracle reads copies of
exactly these bytes: `DeviceData.host_graph()` copies the CSR arrays back, `HostMirror`
copies back the rows of the tensors a sampled comparison reads.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import synth


def _gen(seed: int, name: str):
    import torch
    g = torch.Generator(device="cuda")
    g.manual_seed(int(np.random.SeedSequence([int(seed), synth.zlib.crc32(name.encode())]).generate_state(1)[0]))
    return g


def csr_from_undirected_dev(N: int, u, v):
    """Device twin of synth.csr_from_undirected: symmetric closure of the pairs, self-pairs and
    duplicates dropped, one self-loop per vertex, columns ascending.  Returns (rowptr int64 [N+1],
    col int32 [nnz]) on the device."""
    import torch
    keep = u != v
    u, v = u[keep], v[keep]
    loops = torch.arange(N, dtype=torch.int64, device=u.device)
    key = torch.cat([u * N + v, v * N + u, loops * N + loops])
    del u, v, keep, loops
    key = torch.unique(key)                      # sorted: row-major, columns ascending
    row = torch.div(key, N, rounding_mode="floor")
    col = (key - row * N).to(torch.int32)
    del key
    rowptr = torch.zeros(N + 1, dtype=torch.int64, device=col.device)
    rowptr[1:] = torch.cumsum(torch.bincount(row, minlength=N), 0)
    return rowptr, col


def chung_lu_dev(N: int, n_edges: int, cdf, gen, bounds=None, cdf0=None, p_inside: float = 0.0):
    """n_edges endpoint pairs, both endpoints drawn proportionally to the vertex weights (cdf =
    their running sum, float64 on the device).  With `bounds` (int64 device tensor of vertex-range
    boundaries) an edge keeps both endpoints inside the first endpoint's range with probability
    p_inside, the second endpoint then drawn proportionally to the weights within that range."""
    import torch
    dev = cdf.device

    def draw():
        return torch.rand(n_edges, generator=gen, device=dev, dtype=torch.float64)

    u = torch.searchsorted(cdf, draw(), right=True).clamp_(max=N - 1)
    v = torch.searchsorted(cdf, draw(), right=True).clamp_(max=N - 1)
    if bounds is not None:
        inside = draw() < p_inside
        blk = torch.searchsorted(bounds, u, right=True) - 1
        lo, hi = bounds[blk], bounds[blk + 1]
        r = cdf0[lo] + draw() * (cdf0[hi] - cdf0[lo])
        v_in = torch.minimum(torch.maximum(torch.searchsorted(cdf, r, right=True), lo), hi - 1)
        v = torch.where(inside, v_in, v)
        del inside, blk, lo, hi, r, v_in
    return csr_from_undirected_dev(N, u, v)


@dataclass
class DeviceData:
    """A workload whose graph and tensors live on the GPU.  Tensors are [T, N, ld] with ld the row
    pitch (a multiple of 4 floats, pad columns NaN); F, S are the logical widths."""
    name: str
    N: int
    rowptr: list                 # T device tensors int64 [N+1]
    col: list                    # T device tensors int32 [nnz_t]
    chunks: np.ndarray           # int64 [n, 4] host
    F: int
    S: int
    H: int
    time_kind: str
    n_struct_layers: int
    X: object
    C: object
    C1: Optional[object]
    H0: Optional[object]
    params: dict = field(default_factory=dict)
    notes: dict = field(default_factory=dict)
    on_device: bool = True

    @property
    def T(self) -> int:
        return len(self.rowptr)

    @property
    def rows(self) -> int:
        c = self.chunks
        return int(((c[:, 1] - c[:, 0]) * (c[:, 3] - c[:, 2])).sum())

    @property
    def nnz(self) -> int:
        return sum(int(c.numel()) for c in self.col)

    def host_graph(self) -> synth.DynamicGraph:
        return synth.DynamicGraph(self.N, [synth.Snapshot(r.cpu().numpy(), c.cpu().numpy())
                                           for r, c in zip(self.rowptr, self.col)])


def release(*objs) -> None:
    """Give device memory back at once, even if something (a failing test's traceback, say) still
    refers to the tensors: the full-size configurations need most of the GPU's memory each.  Takes
    tensors, DeviceData objects and anything with a `.layer` and a `.Y` (a created layer's holder:
    the layer is destroyed, its output tensor released; its inputs are views of the data's)."""
    import gc
    import torch
    for o in objs:
        if o is None:
            continue
        if isinstance(o, torch.Tensor):
            o.untyped_storage().resize_(0)
        elif hasattr(o, "layer"):
            o.layer.destroy()
            release(getattr(o, "Y", None))
        else:
            release(*[v for v in vars(o).values() if isinstance(v, torch.Tensor)], *o.rowptr, *o.col,
                    *[v for v in o.notes.values() if isinstance(v, torch.Tensor)])
    gc.collect()
    torch.cuda.empty_cache()


class HostMirror:
    """Host array [T, N, F] of which only the rows asked for hold the device tensor's values (the
    rest is untouched zero pages that take no memory): what the oracle is handed when it computes a
    sample of a tensor too large to copy back whole.  A row the oracle reads that was not copied
    would show as a parity failure, not pass silently: `covered` records what was copied and the
    callers check their reads against it."""

    def __init__(self, dev_tensor, F: int):
        T, N = int(dev_tensor.shape[0]), int(dev_tensor.shape[1])
        self.dev, self.F = dev_tensor, F
        self.host = np.zeros((T, N, F), np.float32)
        self.covered = [np.zeros(N, bool) for _ in range(T)]

    def fill_range(self, t: int, lo: int, hi: int) -> None:
        if self.covered[t][lo:hi].all():
            return
        self.host[t, lo:hi] = self.dev[t, lo:hi, :self.F].cpu().numpy()
        self.covered[t][lo:hi] = True

    def fill_rows(self, t: int, idx: np.ndarray) -> None:
        import torch
        idx = np.unique(np.asarray(idx, np.int64))
        idx = idx[~self.covered[t][idx]]
        if idx.size == 0:
            return
        sel = torch.from_numpy(idx).to(self.dev.device)
        self.host[t, idx] = self.dev[t].index_select(0, sel)[:, :self.F].cpu().numpy()
        self.covered[t][idx] = True


class RowFetcher:
    """Indexable as [t, ids] (ids an integer or an integer array) like a host array [T, N, F]:
    fetches those rows of a device tensor [T, N, ld]."""

    def __init__(self, dev_tensor, F: int):
        self.dev, self.F = dev_tensor, F

    def __getitem__(self, key):
        import torch
        t, idx = key
        if np.isscalar(idx) or getattr(idx, "ndim", 1) == 0:
            return self.dev[int(t), int(idx), :self.F].float().cpu().numpy()
        idx = np.asarray(idx, np.int64)
        if idx.size == 0:
            return np.zeros((0, self.F), np.float32)
        sel = torch.from_numpy(idx).to(self.dev.device)
        return self.dev[int(t)].index_select(0, sel)[:, :self.F].float().cpu().numpy()


def _pitched_normal(T: int, N: int, F: int, ld: int, gen, scale: float = 1.0, base=None, say=None, what=""):
    """[T, N, ld] fp32 on the device: columns < F are scale * N(0,1) (+ base), pad columns NaN."""
    import torch
    out = torch.empty((T, N, ld), dtype=torch.float32, device="cuda")
    for t in range(T):
        z = torch.randn((N, F), generator=gen, device="cuda", dtype=torch.float32)
        if scale != 1.0:
            z *= scale
        if base is not None:
            z += base[t, :, :F]
        out[t, :, :F] = z
        if ld > F:
            out[t, :, F:] = float("nan")
        del z
        if say and (t + 1) % 8 == 0:
            say(f"  {what}: {t + 1}/{T} snapshots")
    return out


def config3_window(seed: int = 0, scale: float = 1.0, window: int = 0, input_concat: bool = False, say=None,
                   n_time_layers: int = 1) -> DeviceData:
    """One 32-snapshot window of config 3 (2,000,000 * scale vertices, mean degree 20 with tail
    exponent 2.0, density varying 10x along a sinusoid of period 128 snapshots times (1 + 0.1 N(0,1)),
    85 % of the edge draws inside one of the window's 64 uneven vertex ranges; F = 172 at pitch 176,
    S = H = 128; cache = X + 0.1 N(0,1), second-layer cache N(0,1), window-start states 0.1 N(0,1)
    for windows after the first, zero for the first), drawn on the device.  `window` in 0..3 picks the
    quarter of the 128-snapshot density curve.  input_concat / n_time_layers = 2: parameters (and states)
    for the LSTM reading both GCN outputs / for two stacked LSTM layers (Section 6's MPNN-LSTM)."""
    import torch
    N = max(256, int(2_000_000 * scale))
    T, F, S, H, ld = 32, 172, 128, 128, 176
    w = synth.powerlaw_weights(N, 2.0, synth.stream(seed, "perm"))
    cdf_h = np.cumsum(w)
    cdf_h[-1] = 1.0
    cdf = torch.from_numpy(cdf_h).cuda()
    cdf0 = torch.cat([torch.zeros(1, dtype=torch.float64, device="cuda"), cdf])
    r_rng = synth.stream(seed, "ranges")
    bounds_all = [synth.uneven_ranges(N, 64, r_rng) for _ in range(window + 1)]
    bounds_h = bounds_all[window]
    bounds = torch.from_numpy(bounds_h).cuda()
    g_rng = synth.stream(seed, "graph")
    t_all = np.arange(128)
    dens = 10.0 ** (0.5 * np.sin(2 * np.pi * t_all / 128.0)) * (1.0 + 0.1 * g_rng.standard_normal(128))
    dens = np.clip(dens, 0.05, None)
    dens /= dens.mean()
    gen = _gen(seed, f"graph-dev-{window}")
    rowptr, col = [], []
    for t in range(T):
        n_edges = int(10 * N * dens[32 * window + t])
        rp, cj = chung_lu_dev(N, n_edges, cdf, gen, bounds, cdf0, 0.85)
        rowptr.append(rp)
        col.append(cj)
        if say and (t + 1) % 8 == 0:
            say(f"  graph: {t + 1}/{T} snapshots")
    del cdf, cdf0, bounds
    torch.cuda.empty_cache()
    chunks = synth.grid_chunks(T, 32, [bounds_h])
    X = _pitched_normal(T, N, F, ld, _gen(seed, "feat-dev"), say=say, what="features")
    C = _pitched_normal(T, N, F, ld, _gen(seed, "cache-dev"), 0.1, X, say=say, what="cache")
    C1 = _pitched_normal(T, N, S, S, _gen(seed, "cache1-dev"), say=say, what="second-layer cache")
    H0 = None
    if window > 0:
        H0 = 0.1 * torch.randn((2 * n_time_layers * N, H), generator=_gen(seed, "h0-dev"), device="cuda", dtype=torch.float32)
    torch.cuda.empty_cache()
    return DeviceData(f"config3@{scale:g}/window{window}", N, rowptr, col, chunks, F, S, H, "lstm", 2, X, C, C1, H0,
                      synth.layer_params(seed, F, S, H, "lstm", 2, False, input_concat=input_concat, n_time_layers=n_time_layers),
                      notes=dict({"input_concat": True} if input_concat else {}, n_time_layers=n_time_layers))


def config4(seed: int = 0, scale: float = 1.0, say=None):
    """Config 4 drawn on the device: 64 snapshots x (500,000 * scale) vertices, 8 N edge draws per
    snapshot with tail exponent 2.2, F = S = 256, 32 chunks = 4 windows of 16 snapshots x 8 even vertex
    ranges, cache = X + 0.1 N(0,1).  Returns (data, target) with target ~ N(0,1) [T, N, 256] on the device."""
    import torch
    T, F = 64, 256
    N = max(256, int(500_000 * scale))
    w = synth.powerlaw_weights(N, 2.2, synth.stream(seed, "perm"))
    cdf_h = np.cumsum(w)
    cdf_h[-1] = 1.0
    cdf = torch.from_numpy(cdf_h).cuda()
    gen = _gen(seed, "graph-dev")
    rowptr, col = [], []
    for t in range(T):
        rp, cj = chung_lu_dev(N, 8 * N, cdf, gen)
        rowptr.append(rp)
        col.append(cj)
        if say and (t + 1) % 16 == 0:
            say(f"  graph: {t + 1}/{T} snapshots")
    del cdf
    torch.cuda.empty_cache()
    bounds = [np.linspace(0, N, 9).astype(np.int64)] * 4
    chunks = synth.grid_chunks(T, 16, bounds)
    X = _pitched_normal(T, N, F, F, _gen(seed, "feat-dev"), say=say, what="features")
    C = _pitched_normal(T, N, F, F, _gen(seed, "cache-dev"), 0.1, X, say=say, what="cache")
    target = _pitched_normal(T, N, F, F, _gen(seed, "target-dev"), say=say, what="targets")
    torch.cuda.empty_cache()
    data = DeviceData(f"config4@{scale:g}", N, rowptr, col, chunks, F, F, F, "none", 1, X, C, None, None,
                      synth.evolve_params(seed, F, F, False))
    return data, target


def config5(seed: int = 0, scale: float = 1.0, say=None, window: int = 16):
    """Config 5 drawn on the device: 16 snapshots x (1,000,000 * scale) vertices, 6 N edge draws per
    snapshot with tail exponent 2.1, F = S = 128, 8 heads, 128 uneven vertex ranges x one 16-snapshot
    window; features, cache = features + 0.1 N(0,1) and targets ~ N(0,1), all bfloat16.
    window != 16: that many snapshots in one window, and 16 / window times the vertices (the same
    number of rows).  Returns (data, target)."""
    import torch
    T, F, heads = int(window), 128, 8
    N = max(1024, int(1_000_000 * scale * 16 / T))
    w = synth.powerlaw_weights(N, 2.1, synth.stream(seed, "perm"))
    cdf_h = np.cumsum(w)
    cdf_h[-1] = 1.0
    cdf = torch.from_numpy(cdf_h).cuda()
    gen = _gen(seed, "graph-dev")
    rowptr, col = [], []
    for t in range(T):
        rp, cj = chung_lu_dev(N, 6 * N, cdf, gen)
        rowptr.append(rp)
        col.append(cj)
    if say:
        say(f"  graph: {T} snapshots")
    del cdf
    chunks = synth.grid_chunks(T, T, [synth.uneven_ranges(N, 128, synth.stream(seed, "ranges"))])

    def bf16(gen_name, base=None, scale_=1.0):
        g = _gen(seed, gen_name)
        out = torch.empty((T, N, F), dtype=torch.bfloat16, device="cuda")
        for t in range(T):
            z = torch.randn((N, F), generator=g, device="cuda", dtype=torch.float32)
            if base is not None:
                z = z * scale_ + base[t]
            out[t] = z.to(torch.bfloat16)
        return out

    Xf = torch.empty((T, N, F), dtype=torch.float32, device="cuda")
    g = _gen(seed, "feat-dev")
    for t in range(T):
        Xf[t] = torch.randn((N, F), generator=g, device="cuda", dtype=torch.float32)
    C = bf16("cache-dev", Xf, 0.1)             # the cache drifts from the unrounded features, as in the host recipe
    X = Xf.to(torch.bfloat16)
    del Xf
    target = bf16("target-dev")
    torch.cuda.empty_cache()
    data = DeviceData(f"config5@{scale:g}", N, rowptr, col, chunks, F, F, F, "none", 1, X, C, None, None,
                      synth.dysat_params(seed, T, F, F, heads), notes={"heads": heads})
    return data, target
