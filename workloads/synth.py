"""Seeded synthetic dynamic graphs, features, parameters and chunk sets.

This module only *draws inputs*: it contains none of the layer's arithmetic
(no aggregation, no normalisation, no recurrence).  Both the CPU oracle and the
HIP path read the arrays it returns, so the two sides always see identical
bytes.  NumPy only; every stream is derived from (seed, stream name), so adding
a stream never shifts another one.

The workloads stand in for the paper's data sets (Table 1: very dense next to
very sparse snapshots, power-law degrees), which are not available here.
"""
from __future__ import annotations

import zlib
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np


def stream(seed: int, name: str) -> np.random.Generator:
    """Independent generator for the named sub-stream of a seed."""
    return np.random.default_rng(np.random.SeedSequence([int(seed), zlib.crc32(name.encode())]))


# --------------------------------------------------------------------------- graphs


@dataclass
class Snapshot:
    """One snapshot as CSR: rowptr int64[N+1], col int32[nnz] (sorted, unique, self-loop stored)."""

    rowptr: np.ndarray
    col: np.ndarray

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


@dataclass
class DynamicGraph:
    N: int
    snaps: List[Snapshot]

    @property
    def T(self) -> int:
        return len(self.snaps)

    @property
    def nnz(self) -> int:
        return sum(s.nnz for s in self.snaps)


def csr_from_undirected(N: int, u: np.ndarray, v: np.ndarray) -> Snapshot:
    """CSR of the symmetric closure of the pairs (u,v), self-pairs and duplicates dropped,
    plus one self-loop per vertex.  Columns ascending within a row."""
    u = np.asarray(u, dtype=np.int64)
    v = np.asarray(v, dtype=np.int64)
    keep = u != v
    u, v = u[keep], v[keep]
    loops = np.arange(N, dtype=np.int64)
    src = np.concatenate([u, v, loops])
    dst = np.concatenate([v, u, loops])
    key = np.unique(src * N + dst)  # sorted => row-major, columns ascending
    row = key // N
    col = (key - row * N).astype(np.int32)
    rowptr = np.zeros(N + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=N), out=rowptr[1:])
    return Snapshot(rowptr=rowptr, col=col)


def erdos_renyi_snapshot(N: int, avg_deg: float, rng: np.random.Generator) -> Snapshot:
    """G(n,p) with p = avg_deg/(N-1): the number of pairs is binomial, pairs uniform."""
    n_pairs = N * (N - 1) // 2
    m = int(rng.binomial(n_pairs, avg_deg / (N - 1)))
    # uniform pairs with replacement; duplicates are dropped by the CSR builder, so draw a
    # few more than m and trim after de-duplication to keep the expected count
    u = rng.integers(0, N, size=int(m * 1.05) + 8)
    v = rng.integers(0, N, size=u.size)
    ok = u != v
    u, v = u[ok], v[ok]
    lo, hi = np.minimum(u, v), np.maximum(u, v)
    _, first = np.unique(lo * N + hi, return_index=True)
    first.sort()
    first = first[:m]
    return csr_from_undirected(N, lo[first], hi[first])


def powerlaw_weights(N: int, alpha: float, rng: np.random.Generator) -> np.ndarray:
    """Vertex weights rank^(-1/(alpha-1)) over a shuffled vertex order: the expected degree
    sequence has tail exponent alpha."""
    rank = rng.permutation(N).astype(np.float64) + 1.0
    w = rank ** (-1.0 / (alpha - 1.0))
    return w / w.sum()


def chung_lu_snapshot(N: int, n_edges: int, w: np.ndarray, rng: np.random.Generator) -> Snapshot:
    """n_edges endpoint pairs, both endpoints drawn proportionally to w."""
    cdf = np.cumsum(w)
    cdf[-1] = 1.0
    u = np.searchsorted(cdf, rng.random(n_edges), side="right")
    v = np.searchsorted(cdf, rng.random(n_edges), side="right")
    return csr_from_undirected(N, u, v)


def chung_lu_blocked_snapshot(N: int, n_edges: int, w: np.ndarray, bounds: np.ndarray,
                              p_inside: float, rng: np.random.Generator) -> Snapshot:
    """Like chung_lu_snapshot, but an edge keeps both endpoints inside one vertex range
    (ranges given by `bounds`, ascending, bounds[0]=0, bounds[-1]=N) with probability
    p_inside; the second endpoint is then drawn proportionally to w within that range."""
    cdf = np.cumsum(w)
    cdf[-1] = 1.0
    u = np.searchsorted(cdf, rng.random(n_edges), side="right")
    v = np.searchsorted(cdf, rng.random(n_edges), side="right")
    inside = rng.random(n_edges) < p_inside
    blk = np.searchsorted(bounds, u, side="right") - 1
    cdf0 = np.concatenate([[0.0], cdf])
    lo_mass = cdf0[bounds[blk]]
    hi_mass = cdf0[bounds[blk + 1]]
    r = lo_mass + rng.random(n_edges) * (hi_mass - lo_mass)
    v_in = np.clip(np.searchsorted(cdf, r, side="right"), bounds[blk], bounds[blk + 1] - 1)
    v = np.where(inside, v_in, v)
    return csr_from_undirected(N, u, v)


# --------------------------------------------------------------------------- chunks


def uneven_ranges(N: int, n_ranges: int, rng: np.random.Generator, min_frac: float = 0.25) -> np.ndarray:
    """Split [0,N) into n_ranges contiguous ranges of uneven width, each at least
    min_frac of the mean width.  Returns the n_ranges+1 boundaries."""
    mean = N / n_ranges
    floor_w = int(min_frac * mean)
    rest = N - floor_w * n_ranges
    share = rng.dirichlet(np.ones(n_ranges))
    extra = np.floor(share * rest).astype(np.int64)
    extra[0] += rest - extra.sum()
    widths = floor_w + extra
    return np.concatenate([[0], np.cumsum(widths)]).astype(np.int64)


def grid_chunks(T: int, window: int, bounds_per_window: List[np.ndarray]) -> np.ndarray:
    """Chunks = time windows x vertex ranges, window-major.  int64 array [n,4] of
    (v_lo, v_hi, t_lo, t_hi), half-open."""
    out = []
    for k, t_lo in enumerate(range(0, T, window)):
        b = bounds_per_window[k]
        for r in range(len(b) - 1):
            out.append((int(b[r]), int(b[r + 1]), t_lo, min(T, t_lo + window)))
    return np.asarray(out, dtype=np.int64).reshape(-1, 4)


# --------------------------------------------------------------------------- parameters


def xavier_uniform(rng: np.random.Generator, fan_out: int, fan_in: int) -> np.ndarray:
    a = np.sqrt(6.0 / (fan_in + fan_out))
    return rng.uniform(-a, a, size=(fan_out, fan_in)).astype(np.float32)


def layer_params(seed: int, F: int, S: int, H: int, time_kind: str, n_struct_layers: int = 1,
                 random_bias: bool = False, input_concat: bool = False, n_time_layers: int = 1) -> dict:
    """Weights in (out, in) row-major order, Xavier-uniform.  Biases are zero unless
    random_bias (tests use non-zero biases so that a dropped bias fails).  input_concat: the
    time encoder reads both structure layers' outputs, so its input weights are [gH, 2S]."""
    rng = stream(seed, "param")
    g = {"gru": 3, "lstm": 4, "none": 0}[time_kind]
    p = {}
    dims_in = [F] + [S] * (n_struct_layers - 1)
    for l, fin in enumerate(dims_in):
        p[f"gcn{l}.weight"] = xavier_uniform(rng, S, fin)          # [S, fin]
        p[f"gcn{l}.bias"] = np.zeros(S, np.float32)
    if g:
        p["rnn.weight_ih"] = xavier_uniform(rng, g * H, 2 * S if input_concat else S)   # [gH, S or 2S]
        p["rnn.weight_hh"] = xavier_uniform(rng, g * H, H)          # [gH, H]
        p["rnn.bias_ih"] = np.zeros(g * H, np.float32)
        p["rnn.bias_hh"] = np.zeros(g * H, np.float32)
        if n_time_layers == 2:      # a second recurrent layer on top of the first (input width H)
            p["rnn1.weight_ih"] = xavier_uniform(rng, g * H, H)
            p["rnn1.weight_hh"] = xavier_uniform(rng, g * H, H)
            p["rnn1.bias_ih"] = np.zeros(g * H, np.float32)
            p["rnn1.bias_hh"] = np.zeros(g * H, np.float32)
    if random_bias:
        for k in p:
            if k.endswith("bias") or ".bias_" in k:
                p[k] = rng.uniform(-0.5, 0.5, size=p[k].shape).astype(np.float32)
    return p


EVOLVE_PARAMS = ["evolve.W_init", "evolve.U_z", "evolve.V_z", "evolve.B_z", "evolve.U_r", "evolve.V_r",
                 "evolve.B_r", "evolve.U_h", "evolve.V_h", "evolve.B_h"]


def evolve_params(seed: int, F: int, S: int, random_bias: bool = False) -> dict:
    """Parameters of the weight-evolving matrix GRU: W_init [F,S], U*, V* [F,F] Xavier-uniform,
    B* [F,S] zero (or small random)."""
    rng = stream(seed, "param")
    p = {}
    for name in EVOLVE_PARAMS:
        kind = name.split(".")[1][0]
        if kind == "W":
            p[name] = xavier_uniform(rng, F, S)
        elif kind in "UV":
            p[name] = xavier_uniform(rng, F, F)
        else:
            p[name] = (rng.uniform(-0.2, 0.2, size=(F, S)) if random_bias else np.zeros((F, S))).astype(np.float32)
    return p


# --------------------------------------------------------------------------- workloads


@dataclass
class Workload:
    name: str
    graph: DynamicGraph
    chunks: np.ndarray                      # int64 [n,4]
    F: int
    S: int
    H: int
    time_kind: str                          # "gru" | "lstm" | "none"
    n_struct_layers: int
    X: np.ndarray                           # fp32 [T,N,F]
    C: np.ndarray                           # fp32 [T,N,F] stale cache of layer-0 inputs
    C1: Optional[np.ndarray]                # fp32 [T,N,S] stale cache of layer-1 inputs (2-layer only)
    H0: Optional[np.ndarray]                # fp32 [sum chunk vertices, H] (then the cell state for LSTM)
    params: dict = field(default_factory=dict)
    notes: dict = field(default_factory=dict)

    @property
    def rows(self) -> int:
        c = self.chunks
        return int(((c[:, 1] - c[:, 0]) * (c[:, 3] - c[:, 2])).sum())


# Optional progress sink for the large generators: set to a callable taking one string (bench.py
# points it at stderr so that a long generation is seen to be alive); None = silent.
progress = None


def _say(msg: str) -> None:
    if progress is not None:
        progress(msg)


def _normal_f32(rng: np.random.Generator, shape) -> np.ndarray:
    """N(0,1) fp32.  Tensors [T, ...] are drawn snapshot by snapshot (the same stream as one call)."""
    if len(shape) == 3 and shape[0] > 1:
        out = np.empty(shape, np.float32)
        for t in range(shape[0]):
            out[t] = rng.standard_normal(size=shape[1:], dtype=np.float32)
            if (t + 1) % 8 == 0:
                _say(f"  normal tensor {tuple(shape)}: {t + 1}/{shape[0]} snapshots")
        return out
    return rng.standard_normal(size=shape, dtype=np.float32)


def _h0_for(chunks: np.ndarray, H: int, time_kind: str, rng: np.random.Generator) -> Optional[np.ndarray]:
    """Window-start state per chunk row: zeros for windows starting at t=0, a small
    N(0, 0.1^2) state (a stale temporal neighbour) for later windows."""
    if time_kind == "none":
        return None
    n_state = 2 if time_kind == "lstm" else 1
    tot = int((chunks[:, 1] - chunks[:, 0]).sum())
    h0 = np.zeros((n_state, tot, H), np.float32)
    off = 0
    for v_lo, v_hi, t_lo, _ in chunks:
        n = int(v_hi - v_lo)
        if t_lo > 0:
            h0[:, off:off + n] = 0.1 * _normal_f32(rng, (n_state, n, H))
        off += n
    return h0.reshape(n_state * tot, H)


def config1(seed: int = 0, random_bias: bool = False) -> Workload:
    """Tiny GCN+GRU: 8 snapshots x 1000 vertices, G(n,p) average degree 8, F=S=H=32,
    4 chunks of 250 contiguous vertices x all 8 snapshots, cache ~ N(0,1) independent of X."""
    T, N, F = 8, 1000, 32
    g_rng = stream(seed, "graph")
    graph = DynamicGraph(N, [erdos_renyi_snapshot(N, 8.0, g_rng) for _ in range(T)])
    bounds = np.arange(0, N + 1, 250, dtype=np.int64)
    chunks = grid_chunks(T, T, [bounds])
    X = _normal_f32(stream(seed, "feat"), (T, N, F))
    C = _normal_f32(stream(seed, "cache"), (T, N, F))
    return Workload("config1", graph, chunks, F, 32, 32, "gru", 1, X, C, None,
                    _h0_for(chunks, 32, "gru", stream(seed, "h0")),
                    layer_params(seed, F, 32, 32, "gru", 1, random_bias))


def _nonuniform_graph(seed: int, T: int, N: int, edge_mu: float, edge_sigma: float, edge_clip: Tuple[int, int],
                      alpha: float):
    g_rng = stream(seed, "graph")
    w = powerlaw_weights(N, alpha, stream(seed, "perm"))
    n_edges = np.clip(np.exp(edge_mu + edge_sigma * g_rng.standard_normal(T)),
                      edge_clip[0], edge_clip[1]).astype(np.int64)
    return DynamicGraph(N, [chung_lu_snapshot(N, int(m), w, g_rng) for m in n_edges]), n_edges


def config2_graph(seed: int = 0, scale: float = 1.0) -> DynamicGraph:
    """The dynamic graph of config2(seed, scale) alone (no features)."""
    N = max(64, int(100_000 * scale))
    return _nonuniform_graph(seed, 32, N, np.log(800_000 * scale), 1.0,
                             (max(1, int(80_000 * scale)), max(2, int(8_000_000 * scale))), 2.1)[0]


def nonuniform_powerlaw(seed: int, T: int, N: int, F: int, S: int, H: int, edge_mu: float,
                        edge_sigma: float, edge_clip: Tuple[int, int], alpha: float, window: int,
                        n_ranges: int, time_kind: str = "gru", n_struct_layers: int = 1,
                        uneven: bool = True, name: str = "config2",
                        random_bias: bool = False) -> Workload:
    """Snapshots with lognormal edge counts (dense next to sparse) and power-law degrees;
    chunks = windows x uneven vertex ranges; cache = X + 0.1 N(0,1) (small drift since the
    pass that filled it)."""
    graph, n_edges = _nonuniform_graph(seed, T, N, edge_mu, edge_sigma, edge_clip, alpha)
    r_rng = stream(seed, "ranges")
    n_win = (T + window - 1) // window
    if uneven:
        bounds = [uneven_ranges(N, n_ranges, r_rng) for _ in range(n_win)]
    else:
        bounds = [np.linspace(0, N, n_ranges + 1).astype(np.int64)] * n_win
    chunks = grid_chunks(T, window, bounds)
    X = _normal_f32(stream(seed, "feat"), (T, N, F))
    C = _normal_f32(stream(seed, "cache"), (T, N, F))
    C *= np.float32(0.1)
    C += X
    C1 = None
    if n_struct_layers == 2:
        C1 = _normal_f32(stream(seed, "cache1"), (T, N, S))
    wl = Workload(name, graph, chunks, F, S, H, time_kind, n_struct_layers, X, C, C1,
                  _h0_for(chunks, H, time_kind, stream(seed, "h0")),
                  layer_params(seed, F, S, H, time_kind, n_struct_layers, random_bias))
    wl.notes["edge_draws"] = n_edges
    return wl


def config2(seed: int = 0, scale: float = 1.0, random_bias: bool = False) -> Workload:
    """Non-uniform GCN+GRU: 32 snapshots x 100k vertices, edge draws per snapshot
    lognormal(ln 800k, 1) clipped to [80k, 8M], tail exponent 2.1, F=S=H=128, 64 chunks =
    4 windows of 8 snapshots x 16 uneven vertex ranges.  `scale` < 1 shrinks N and the edge
    counts together (same shape, for tests the oracle finishes in seconds)."""
    N = max(64, int(100_000 * scale))
    return nonuniform_powerlaw(seed, 32, N, 128, 128, 128, np.log(800_000 * scale), 1.0,
                               (max(1, int(80_000 * scale)), max(2, int(8_000_000 * scale))),
                               2.1, 8, 16, "gru", 1, True,
                               "config2" if scale == 1.0 else f"config2@{scale:g}", random_bias)


def config3(seed: int = 0, scale: float = 1.0, windows: int = 1, random_bias: bool = False,
            input_concat: bool = False) -> Workload:
    """Large 2-layer GCN + LSTM: N = 2,000,000 * scale vertices, mean degree 20 with tail exponent
    2.0, per-snapshot density varying 10x along a sinusoid of period 128 snapshots times
    (1 + 0.1 N(0,1)), F = 172, S = H = 128, windows of 32 snapshots x 64 uneven vertex ranges;
    an edge keeps both endpoints inside one vertex range with probability 0.85.  The full
    config (128 snapshots) is run one 32-snapshot window at a time (memory-capped fusion,
    Section 5.1.1); `windows` says how many of them this workload holds.  input_concat: the LSTM
    reads both GCN layers' outputs (256 wide), as the MPNN-LSTM of Section 6 does."""
    N = max(256, int(2_000_000 * scale))
    T = 32 * windows
    F, S, H = 172, 128, 128
    g_rng = stream(seed, "graph")
    w = powerlaw_weights(N, 2.0, stream(seed, "perm"))
    r_rng = stream(seed, "ranges")
    bounds = [uneven_ranges(N, 64, r_rng) for _ in range(windows)]
    t_all = np.arange(128)
    dens = 10.0 ** (0.5 * np.sin(2 * np.pi * t_all / 128.0)) * (1.0 + 0.1 * g_rng.standard_normal(128))
    dens = np.clip(dens, 0.05, None)
    dens /= dens.mean()
    snaps = []
    for t in range(T):
        n_edges = int(10 * N * dens[t])          # mean degree 20 = 2 * edges / N
        snaps.append(chung_lu_blocked_snapshot(N, n_edges, w, bounds[t // 32], 0.85, g_rng))
        if N >= 500_000 or (t + 1) % 8 == 0:
            _say(f"  graph: {t + 1}/{T} snapshots")
    graph = DynamicGraph(N, snaps)
    chunks = grid_chunks(T, 32, bounds)
    X = _normal_f32(stream(seed, "feat"), (T, N, F))
    C = _normal_f32(stream(seed, "cache"), (T, N, F))
    C *= np.float32(0.1)
    C += X
    C1 = _normal_f32(stream(seed, "cache1"), (T, N, S))
    wl = Workload("config3" if scale == 1.0 else f"config3@{scale:g}", graph, chunks, F, S, H, "lstm", 2, X, C, C1,
                  _h0_for(chunks, H, "lstm", stream(seed, "h0")),
                  layer_params(seed, F, S, H, "lstm", 2, random_bias, input_concat=input_concat),
                  notes={"input_concat": True} if input_concat else {})
    return wl


def config4(seed: int = 0, scale: float = 1.0, random_bias: bool = False):
    """EvolveGCN-O layer: 64 snapshots x (500,000 * scale) vertices, average degree 16 with tail
    exponent 2.2, F = S = 256, 32 chunks = 4 windows of 16 snapshots x 8 even vertex ranges,
    cache = X + 0.1 N(0,1), MSE targets ~ N(0,1).  Returns (workload, target)."""
    T, F = 64, 256
    N = max(256, int(500_000 * scale))
    g_rng = stream(seed, "graph")
    w = powerlaw_weights(N, 2.2, stream(seed, "perm"))
    snaps = []
    for t in range(T):
        snaps.append(chung_lu_snapshot(N, 8 * N, w, g_rng))
        if (t + 1) % 8 == 0:
            _say(f"  graph: {t + 1}/{T} snapshots")
    graph = DynamicGraph(N, snaps)
    bounds = [np.linspace(0, N, 9).astype(np.int64)] * 4
    chunks = grid_chunks(T, 16, bounds)
    X = _normal_f32(stream(seed, "feat"), (T, N, F))
    C = _normal_f32(stream(seed, "cache"), (T, N, F))
    C *= np.float32(0.1)
    C += X
    target = _normal_f32(stream(seed, "target"), (T, N, F))
    wl = Workload("config4" if scale == 1.0 else f"config4@{scale:g}", graph, chunks, F, F, F, "none", 1, X, C,
                  None, None, evolve_params(seed, F, F, random_bias))
    return wl, target


def random_small(seed: int, T: int, N: int, F: int, S: int, H: int, avg_deg: float,
                 chunks: np.ndarray, time_kind: str = "gru", n_struct_layers: int = 1,
                 hub: bool = False, input_concat: bool = False) -> Workload:
    """Small random workload with arbitrary chunk set and non-zero biases, for tests."""
    g_rng = stream(seed, "graph")
    snaps = []
    for _ in range(T):
        if N > 1 and avg_deg > 0:
            s = erdos_renyi_snapshot(N, min(avg_deg, N - 1.0), g_rng)
        else:
            s = csr_from_undirected(N, np.zeros(0, np.int64), np.zeros(0, np.int64))
        snaps.append(s)
    if hub and N > 2:
        # one vertex adjacent to all others in the middle snapshot
        t = T // 2
        h = int(g_rng.integers(0, N))
        others = np.array([i for i in range(N) if i != h], dtype=np.int64)
        old = snaps[t]
        rows = np.repeat(np.arange(N, dtype=np.int64), np.diff(old.rowptr))
        snaps[t] = csr_from_undirected(N, np.concatenate([rows, np.full(N - 1, h)]),
                                       np.concatenate([old.col.astype(np.int64), others]))
    graph = DynamicGraph(N, snaps)
    chunks = np.asarray(chunks, dtype=np.int64).reshape(-1, 4)
    X = _normal_f32(stream(seed, "feat"), (T, N, F))
    C = _normal_f32(stream(seed, "cache"), (T, N, F))
    C1 = _normal_f32(stream(seed, "cache1"), (T, N, S)) if n_struct_layers == 2 else None
    h0 = _h0_for(chunks, H, time_kind, stream(seed, "h0"))
    if h0 is not None:  # make every window start non-trivial
        h0 = (0.5 * _normal_f32(stream(seed, "h0b"), h0.shape)).astype(np.float32)
    return Workload(f"small{seed}", graph, chunks, F, S, H, time_kind, n_struct_layers, X, C, C1, h0,
                    layer_params(seed, F, S, H, time_kind, n_struct_layers, random_bias=True,
                                 input_concat=input_concat),
                    notes={"input_concat": True} if input_concat else {})


# --------------------------------------------------------------------------- bf16 workloads


def round_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bfloat16 (round to nearest even)."""
    out = np.array(a, dtype=np.float32, order="C")          # a copy; finite values only
    flat = out.reshape(-1).view(np.uint32)
    step = 1 << 24
    for lo in range(0, flat.size, step):                    # in pieces: no array-sized temporaries
        u = flat[lo:lo + step]
        u += ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
        u &= np.uint32(0xFFFF0000)
    return out


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of an fp32 array that is already bf16-representable."""
    return (np.ascontiguousarray(a, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


DYSAT_PARAMS = ["gat.weight", "gat.att_src", "gat.att_dst", "attn.pos", "attn.weight_q", "attn.weight_k",
                "attn.weight_v"]


def dysat_params(seed: int, T: int, F: int, S: int, heads: int) -> dict:
    """Parameters of the graph-attention + temporal self-attention layer, bf16-representable:
    gat.weight [S,F] (out, in), gat.att_src / gat.att_dst [heads, S/heads], attn.pos [T,S],
    attn.weight_q/k/v [S,S] (out, in).  Xavier-uniform; positions N(0, 0.1^2)."""
    rng = stream(seed, "param")
    D = S // heads
    p = {
        "gat.weight": xavier_uniform(rng, S, F),
        "gat.att_src": xavier_uniform(rng, heads, D),
        "gat.att_dst": xavier_uniform(rng, heads, D),
        "attn.pos": (0.1 * rng.standard_normal((T, S))).astype(np.float32),
        "attn.weight_q": xavier_uniform(rng, S, S),
        "attn.weight_k": xavier_uniform(rng, S, S),
        "attn.weight_v": xavier_uniform(rng, S, S),
    }
    return {k: round_bf16(v) for k, v in p.items()}


def dysat_small(seed: int, T: int, N: int, F: int, heads: int, avg_deg: float, chunks, hub: bool = False):
    """Small random graph-attention workload (S = F), all tensors bf16-representable."""
    wl = random_small(seed, T, N, F, F, F, avg_deg, chunks, "none", hub=hub)
    wl.X = round_bf16(wl.X)
    wl.C = round_bf16(wl.C)
    wl.params = dysat_params(seed, T, F, F, heads)
    wl.notes["heads"] = heads
    return wl


def config5(seed: int = 0, scale: float = 1.0):
    """Graph attention + causal temporal self-attention, bf16: 16 snapshots x (1,000,000 * scale)
    vertices, average degree 12 with tail exponent 2.1, F = S = 128, 8 heads, 128 uneven vertex
    ranges x one 16-snapshot window, cache = X + 0.1 N(0,1), MSE targets ~ N(0,1).
    Returns (workload, target)."""
    T, F, heads = 16, 128, 8
    N = max(1024, int(1_000_000 * scale))
    g_rng = stream(seed, "graph")
    w = powerlaw_weights(N, 2.1, stream(seed, "perm"))
    snaps = []
    for t in range(T):
        snaps.append(chung_lu_snapshot(N, 6 * N, w, g_rng))
        if (t + 1) % 4 == 0:
            _say(f"  graph: {t + 1}/{T} snapshots")
    graph = DynamicGraph(N, snaps)
    bounds = [uneven_ranges(N, 128, stream(seed, "ranges"))]
    chunks = grid_chunks(T, 16, bounds)
    X = _normal_f32(stream(seed, "feat"), (T, N, F))
    C = _normal_f32(stream(seed, "cache"), (T, N, F))
    C *= np.float32(0.1)
    C += X
    X, C = round_bf16(X), round_bf16(C)
    target = round_bf16(_normal_f32(stream(seed, "target"), (T, N, F)))
    wl = Workload("config5" if scale == 1.0 else f"config5@{scale:g}", graph, chunks, F, F, F, "none", 1,
                  X, C, None, None, dysat_params(seed, T, F, F, heads))
    wl.notes["heads"] = heads
    return wl, target


# --------------------------------------------------------------------------- vertex presence


def presence(seed: int, T: int, N: int, p_lo: float = 0.15, p_hi: float = 1.0) -> np.ndarray:
    """uint8 [T,N]: vertex i is present in snapshot t with its own probability p_i ~ U(p_lo, p_hi),
    independently per snapshot: sequences of very different lengths, with gaps."""
    rng = stream(seed, "presence")
    p = rng.uniform(p_lo, p_hi, size=N)
    return (rng.random((T, N)) < p[None, :]).astype(np.uint8)


# --------------------------------------------------------------------------- embedding drift


def drifted_copies(seed: int, R: int, F: int, median: float = 0.34, sigma: float = 1.0,
                   unchanged: float = 0.1, kind: str = "lognormal", d_max: float = 2.0):
    """Current embeddings E ~ N(0,1) [R,F] and the copies L sent last, fp32.  Row r has drifted by a
    Gaussian vector of a drawn length; a fraction `unchanged` of the rows has not moved at all
    (L = E bit for bit).  kind="lognormal": lengths log-normal (median `median`, log-std `sigma`):
    about 85 % of the distances below 1 and a long tail above, as in the distance CDFs the paper
    plots.  kind="triangular": length = d_max (1 - sqrt(U)), i.e. a fraction (1 - x)^2 of the rows
    lies beyond x times the largest distance: 49 / 25 / 9 / 1 % at x = 0.3 / 0.5 / 0.7 / 0.9, the
    traffic left over at those static thresholds in the paper's accuracy table (its Amazon and
    Epinion rows) within a few points."""
    rng = stream(seed, "drift")
    E = _normal_f32(rng, (R, F))
    if kind == "lognormal":
        length = np.exp(rng.normal(np.log(median), sigma, size=R)).astype(np.float32)
    elif kind == "triangular":
        length = (d_max * (1.0 - np.sqrt(rng.random(R)))).astype(np.float32)
    else:
        raise ValueError(kind)
    length[rng.random(R) < unchanged] = 0.0
    L = np.empty_like(E)
    step = 1 << 18
    for a in range(0, R, step):
        b = min(R, a + step)
        d = rng.standard_normal((b - a, F), dtype=np.float32)
        d *= (length[a:b] / np.sqrt((d * d).sum(axis=1)).clip(1e-30))[:, None]   # drift of exactly that length
        np.subtract(E[a:b], d, out=L[a:b])
    return E, L


def boundary_rows(seed: int, R: int, frac: float) -> np.ndarray:
    """Ascending int64 subset of range(R): each row is a candidate with probability `frac`."""
    rng = stream(seed, "boundary")
    return np.flatnonzero(rng.random(R) < frac).astype(np.int64)
