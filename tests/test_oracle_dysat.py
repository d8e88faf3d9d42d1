"""Pins of the graph-attention + temporal self-attention oracle (CPU only): a dense brute-force
forward written with explicit loops from an edge list, closed forms (uniform attention = mean
aggregation, single-neighbour rows, zero queries = causal running mean), causality, chunking
invariants, the library's scaled-dot-product attention, and finite differences for the gradients."""
import math

import numpy as np
import pytest
import torch

from oracle import dysat
from workloads import synth
from refs import edges_of


def _brute_forward(wl, heads):
    """Dense, loop-by-loop forward from the undirected edge list; float64."""
    g, P = wl.graph, {k: v.astype(np.float64) for k, v in wl.params.items()}
    T, N, S = g.T, g.N, wl.S
    D = S // heads
    X, C = wl.X.astype(np.float64), wl.C.astype(np.float64)
    Y = np.zeros((T, N, S))
    U = np.zeros((T, N, S))
    for v_lo, v_hi, t_lo, t_hi in wl.chunks.tolist():
        G = np.zeros((t_hi - t_lo, v_hi - v_lo, S))
        for t in range(t_lo, t_hi):
            adj = np.eye(N, dtype=bool)
            for a, b in edges_of(g.snaps[t]):
                adj[a, b] = adj[b, a] = True
            mix = C[t].copy()
            mix[v_lo:v_hi] = X[t, v_lo:v_hi]
            Z = mix @ P["gat.weight"].T                       # z of every vertex as this chunk sees it
            for i in range(v_lo, v_hi):
                nb = np.flatnonzero(adj[i])
                for h in range(heads):
                    sl = slice(h * D, (h + 1) * D)
                    e = np.array([P["gat.att_dst"][h] @ Z[i, sl] + P["gat.att_src"][h] @ Z[j, sl] for j in nb])
                    e = np.where(e > 0, e, 0.2 * e)
                    a = np.exp(e - e.max())
                    a /= a.sum()
                    U[t, i, sl] = sum(a[k] * Z[j, sl] for k, j in enumerate(nb))
            u = U[t, v_lo:v_hi]
            G[t - t_lo] = np.where(u > 0, u, np.expm1(u))
        w = t_hi - t_lo
        Pm = G + P["attn.pos"][t_lo:t_hi, None, :]
        Q, K, V = (Pm @ P[f"attn.weight_{n}"].T for n in "qkv")
        for v in range(v_hi - v_lo):
            for h in range(heads):
                sl = slice(h * D, (h + 1) * D)
                for s in range(w):
                    sc = np.array([Q[s, v, sl] @ K[r, v, sl] / math.sqrt(D) for r in range(s + 1)])
                    a = np.exp(sc - sc.max())
                    a /= a.sum()
                    Y[t_lo + s, v_lo + v, sl] = sum(a[r] * V[r, v, sl] for r in range(s + 1))
    return Y, U


CHUNKS = [[0, 5, 0, 4], [5, 12, 0, 2], [5, 12, 2, 4]]


def _small(seed=1, heads=2, F=8, chunks=CHUNKS, N=12, T=4, deg=3.0, hub=True):
    return synth.dysat_small(seed, T, N, F, heads, deg, chunks, hub=hub)


def test_forward_equals_dense_brute_force():
    wl = _small()
    got = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)
    Y, U = _brute_forward(wl, 2)
    np.testing.assert_allclose(got["U"], U, rtol=0, atol=1e-12)
    np.testing.assert_allclose(got["Y"], Y, rtol=0, atol=1e-12)
    assert np.abs(Y).max() > 0.1


def test_zero_attention_vectors_give_mean_aggregation():
    """a_src = a_dst = 0: all logits equal, alpha = 1/deg, so u_i is the mean of the neighbours'
    z - a row-normalised dense adjacency product."""
    wl = _small(seed=2, chunks=[[0, 12, 0, 4]])
    wl.params["gat.att_src"][:] = 0
    wl.params["gat.att_dst"][:] = 0
    got = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["U"]
    for t in range(4):
        adj = np.eye(12)
        for a, b in edges_of(wl.graph.snaps[t]):
            adj[a, b] = adj[b, a] = 1
        want = (adj / adj.sum(1, keepdims=True)) @ (wl.X[t].astype(np.float64) @ wl.params["gat.weight"].T.astype(np.float64))
        np.testing.assert_allclose(got[t], want, atol=1e-12)


def test_isolated_vertex_attends_to_itself_only():
    wl = _small(seed=3, deg=0.0, hub=False)    # only self-loops
    got = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["U"]
    want = wl.X.astype(np.float64) @ wl.params["gat.weight"].T.astype(np.float64)
    np.testing.assert_allclose(got, want, atol=1e-12)


def test_alpha_is_a_convex_combination():
    """With the identity as weight and a constant feature column, every u keeps that constant
    (attention weights are non-negative and sum to one) whatever the attention vectors are."""
    wl = _small(seed=4, chunks=[[0, 12, 0, 4]])
    wl.params["gat.weight"] = np.eye(8, dtype=np.float32)
    wl.X[:, :, 3] = 2.5
    wl.X[:, :, 7] = -1.25
    got = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["U"]
    np.testing.assert_allclose(got[:, :, 3], 2.5, atol=1e-12)
    np.testing.assert_allclose(got[:, :, 7], -1.25, atol=1e-12)


def test_zero_queries_give_causal_running_mean():
    wl = _small(seed=5)
    wl.params["attn.weight_q"][:] = 0
    out = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)
    U = out["U"]
    G = np.where(U > 0, U, np.expm1(U))
    for v_lo, v_hi, t_lo, t_hi in wl.chunks.tolist():
        V = (G[t_lo:t_hi, v_lo:v_hi] + wl.params["attn.pos"][t_lo:t_hi, None, :]) @ wl.params["attn.weight_v"].T.astype(np.float64)
        want = np.cumsum(V, axis=0) / np.arange(1, t_hi - t_lo + 1)[:, None, None]
        np.testing.assert_allclose(out["Y"][t_lo:t_hi, v_lo:v_hi], want, atol=1e-12)


def test_temporal_attention_equals_library_sdpa():
    wl = _small(seed=6, heads=4, F=16, chunks=[[0, 12, 0, 4]])
    out = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 4)
    U = torch.from_numpy(out["U"])
    P = torch.nn.functional.elu(U) + torch.from_numpy(wl.params["attn.pos"]).double()[:, None, :]
    q, k, v = ((P @ torch.from_numpy(wl.params[f"attn.weight_{n}"]).double().T).view(4, 12, 4, 4).permute(1, 2, 0, 3)
               for n in "qkv")                     # [vertex, head, step, D]
    want = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    np.testing.assert_allclose(out["Y"], want.permute(2, 0, 1, 3).reshape(4, 12, 16).numpy(), atol=1e-12)


def test_causality():
    wl = _small(seed=7, chunks=[[0, 12, 0, 4]])
    a = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["Y"]
    wl.X[2:] += 1.0
    wl.C[2:] -= 1.0
    b = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["Y"]
    np.testing.assert_array_equal(a[:2], b[:2])
    assert np.abs(a[2:] - b[2:]).max() > 1e-3


def test_cache_equal_to_input_makes_vertex_chunking_invisible():
    wl = _small(seed=8, chunks=[[0, 4, 0, 4], [4, 9, 0, 4], [9, 12, 0, 4]])
    whole = dysat.forward(wl.graph, [[0, 12, 0, 4]], wl.params, wl.X, wl.X, 2)["Y"]
    parts = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.X, 2)["Y"]
    np.testing.assert_allclose(parts, whole, atol=1e-12)
    stale = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["Y"]
    assert np.abs(stale - whole).max() > 1e-3


def test_fused_equals_one_by_one():
    wl = _small(seed=9)
    fused = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2)["Y"]
    acc = np.zeros_like(fused)
    for c in wl.chunks[::-1]:
        acc += dysat.forward(wl.graph, c[None], wl.params, wl.X, wl.C, 2)["Y"]
    np.testing.assert_array_equal(acc, fused)


@pytest.mark.parametrize("mode", ["target", "dY"])
def test_gradients_match_finite_differences(mode):
    wl = _small(seed=10)
    rng = np.random.default_rng(0)
    extra = rng.standard_normal(wl.X.shape)
    kw = {"target": extra} if mode == "target" else {"dY": extra}
    base = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2, **kw)

    def loss_at(params):
        Y = dysat.forward(wl.graph, wl.chunks, params, wl.X, wl.C, 2)["Y"]
        cov = np.zeros(Y.shape[:2], bool)
        for v_lo, v_hi, t_lo, t_hi in wl.chunks.tolist():
            cov[t_lo:t_hi, v_lo:v_hi] = True
        if mode == "target":
            return float((((Y - extra) ** 2)[cov]).sum() / (cov.sum() * Y.shape[2]))
        return float((Y * extra)[cov].sum())

    assert abs(loss_at(wl.params) - base["loss"]) < 1e-12 * max(1.0, abs(base["loss"]))
    for name in dysat.PARAMS:
        for _ in range(2):
            d = rng.standard_normal(wl.params[name].shape)
            eps = 1e-6
            plus = {k: v.astype(np.float64) for k, v in wl.params.items()}
            minus = {k: v.astype(np.float64) for k, v in wl.params.items()}
            plus[name] = plus[name] + eps * d
            minus[name] = minus[name] - eps * d
            fd = (loss_at(plus) - loss_at(minus)) / (2 * eps)
            an = float((base["grads"][name] * d).sum())
            assert abs(fd - an) < 1e-6 * max(1.0, abs(an)), (name, fd, an)


def test_input_gradient_matches_finite_differences():
    """dL/dX by central differences along random directions; rows no chunk covers and the cache
    get no gradient."""
    wl = _small(seed=12, chunks=[[0, 5, 0, 4], [5, 8, 1, 3]])
    rng = np.random.default_rng(3)
    dY = rng.standard_normal(wl.X.shape)
    base = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2, dY=dY, want_dx=True)
    cov = np.zeros(wl.X.shape[:2], bool)
    for v_lo, v_hi, t_lo, t_hi in np.asarray(wl.chunks).tolist():
        cov[t_lo:t_hi, v_lo:v_hi] = True
    assert (~cov).any() and np.abs(base["dX"][~cov]).max() == 0.0
    assert np.abs(base["dX"][cov]).max() > 1e-3

    def loss_at(X):
        Y = dysat.forward(wl.graph, wl.chunks, wl.params, X, wl.C, 2)["Y"]
        return float((Y * dY)[cov].sum())

    X0 = wl.X.astype(np.float64)
    for _ in range(4):
        d = rng.standard_normal(X0.shape)
        eps = 1e-6
        fd = (loss_at(X0 + eps * d) - loss_at(X0 - eps * d)) / (2 * eps)
        an = float((base["dX"] * d).sum())
        assert abs(fd - an) < 1e-6 * max(1.0, abs(an)), (fd, an)


def test_cache_is_a_constant_but_its_projection_carries_weight_gradient():
    """Halo rows enter as W c: the gradient of gat.weight changes when the cache changes, and
    uncovered snapshots / vertices contribute nothing."""
    wl = _small(seed=11, chunks=[[0, 5, 0, 4]])
    dY = np.random.default_rng(1).standard_normal(wl.X.shape)
    a = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 2, dY=dY)["grads"]["gat.weight"]
    C2 = wl.C.copy()
    C2[:, 5:] *= 2.0
    b = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, C2, 2, dY=dY)["grads"]["gat.weight"]
    assert np.abs(a - b).max() > 1e-3
    X2 = wl.X.copy()
    X2[:, 5:] += 3.0          # inputs of vertices outside the only chunk are never read
    c = dysat.gradients(wl.graph, wl.chunks, wl.params, X2, wl.C, 2, dY=dY)["grads"]["gat.weight"]
    np.testing.assert_array_equal(a, c)


def test_oracle_module_is_test_only():
    import os
    text = open(os.path.join(os.path.dirname(dysat.__file__), "dysat.py")).read()
    assert "TEST INFRASTRUCTURE ONLY" in text and "paper_2309_03523_amd" not in text
