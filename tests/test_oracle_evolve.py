"""Pins for the oracle's EvolveGCN-O layer (weight-evolving matrix GRU + GCN + MSE loss and its
gradients): torch autograd in float64 built from dense adjacency matrices, and central finite
differences.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from workloads import synth
from refs import dense_norm_adj, edges_of


def _torch_layer(wl, chunks, P, target, Xt=None):
    """The layer by its definition with torch ops on dense matrices; returns (Y, loss).
    Xt: the input as a torch tensor (to differentiate with respect to it)."""
    T, N = wl.graph.T, wl.graph.N
    W = P["evolve.W_init"]
    rows, tgts = [], []
    Y = torch.full((T, N, W.shape[1]), float("nan"), dtype=torch.float64)
    Ws = []
    for t in range(T):
        Zg = torch.sigmoid(P["evolve.U_z"] @ W + P["evolve.V_z"] @ W + P["evolve.B_z"])
        Rg = torch.sigmoid(P["evolve.U_r"] @ W + P["evolve.V_r"] @ W + P["evolve.B_r"])
        Wc = torch.tanh(P["evolve.U_h"] @ W + P["evolve.V_h"] @ (Rg * W) + P["evolve.B_h"])
        W = (1 - Zg) * W + Zg * Wc
        Ws.append(W)
    sq, cnt = 0.0, 0
    for v_lo, v_hi, t_lo, t_hi in np.asarray(chunks).tolist():
        for t in range(t_lo, t_hi):
            Ahat = torch.from_numpy(dense_norm_adj(N, edges_of(wl.graph.snaps[t])))
            mix = torch.from_numpy(wl.C[t].astype(np.float64)).clone()
            mix[v_lo:v_hi] = (torch.from_numpy(wl.X[t, v_lo:v_hi].astype(np.float64)) if Xt is None
                              else Xt[t, v_lo:v_hi])
            y = torch.relu(Ahat[v_lo:v_hi] @ mix @ Ws[t])
            Y[t, v_lo:v_hi] = y.detach()
            sq = sq + ((y - torch.from_numpy(target[t, v_lo:v_hi].astype(np.float64))) ** 2).sum()
            cnt += y.numel()
    return Y, sq / cnt, torch.stack(Ws)


@pytest.mark.parametrize("F,S", [(6, 6), (5, 7)])
def test_evolve_forward_and_gradients_equal_torch_autograd(F, S):
    T, N = 4, 13
    chunks = np.array([[0, 5, 0, 4], [5, 13, 0, 2], [5, 13, 2, 4]], np.int64)
    wl = synth.random_small(91, T, N, F, 32, 32, 3.0, chunks, "none", hub=True)
    params = synth.evolve_params(7, F, S, random_bias=True)
    target = synth.stream(7, "target").standard_normal((T, N, S)).astype(np.float32)
    got = oracle.evolve(wl.graph, chunks, params, wl.X, wl.C, target, want_grads=True, want_dx=True)
    P = {k: torch.tensor(v.astype(np.float64), requires_grad=True) for k, v in params.items()}
    Xt = torch.tensor(wl.X.astype(np.float64), requires_grad=True)
    Y, loss, Ws = _torch_layer(wl, chunks, P, target, Xt)
    loss.backward()
    # gradient w.r.t. the input rows: only through the rows of the same chunk (the cache is a constant)
    gx = Xt.grad.numpy()
    assert np.abs(got["dX"] - gx).max() < 1e-12 * max(1.0, np.abs(gx).max()) and np.abs(gx).max() > 0
    assert np.abs(got["Wt"] - Ws.detach().numpy()).max() < 1e-12
    assert np.nanmax(np.abs(got["Y"] - Y.numpy())) < 1e-5
    assert abs(got["loss"] - loss.item()) < 1e-10 * max(1.0, abs(loss.item()))
    for k in oracle.EVOLVE_PARAMS:
        g_t = P[k].grad.numpy()
        assert np.abs(got["grads"][k] - g_t).max() < 1e-10 * max(1.0, np.abs(g_t).max()), k
        assert np.abs(g_t).max() > 0  # every parameter matters in this example


def test_evolve_gradient_by_finite_differences():
    T, N, F, S = 3, 9, 4, 4
    chunks = np.array([[0, 9, 0, 3]], np.int64)
    wl = synth.random_small(92, T, N, F, 32, 32, 2.5, chunks, "none")
    params = {k: v.astype(np.float64) for k, v in synth.evolve_params(8, F, S, random_bias=True).items()}
    target = synth.stream(8, "target").standard_normal((T, N, S)).astype(np.float32)
    base = oracle.evolve(wl.graph, chunks, params, wl.X, wl.C, target, want_grads=True)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for k in oracle.EVOLVE_PARAMS:
        for _ in range(3):
            idx = tuple(int(rng.integers(0, d)) for d in params[k].shape)
            hi = {n: v.copy() for n, v in params.items()}
            lo = {n: v.copy() for n, v in params.items()}
            hi[k][idx] += eps
            lo[k][idx] -= eps
            fd = (oracle.evolve(wl.graph, chunks, hi, wl.X, wl.C, target)["loss"]
                  - oracle.evolve(wl.graph, chunks, lo, wl.X, wl.C, target)["loss"]) / (2 * eps)
            assert abs(fd - base["grads"][k][idx]) < 1e-6 * max(1.0, abs(fd)), (k, idx)


def test_evolve_weights_do_not_depend_on_chunking_and_identity_gate():
    """The weight recurrence is global; with U = V = 0 and B_z very negative the update gate closes
    and every W_t equals W_init, so the layer is a plain GCN with that weight."""
    T, N, F = 3, 11, 5
    wl = synth.random_small(93, T, N, F, 32, 32, 3.0, [[0, N, 0, T]], "none")
    params = synth.evolve_params(9, F, F, random_bias=True)
    a = oracle.evolve(wl.graph, [[0, N, 0, T]], params, wl.X, wl.X)
    b = oracle.evolve(wl.graph, [[0, 4, 0, T], [4, N, 0, 1], [4, N, 1, T]], params, wl.X, wl.X)
    assert np.array_equal(a["Wt"], b["Wt"]) and np.abs(a["Y"] - b["Y"]).max() < 1e-6
    for k in params:
        if k != "evolve.W_init":
            params[k] = np.zeros_like(params[k])
    params["evolve.B_z"] = np.full_like(params["evolve.B_z"], -60.0)
    c = oracle.evolve(wl.graph, [[0, N, 0, T]], params, wl.X, wl.X)
    assert np.abs(c["Wt"] - params["evolve.W_init"][None]).max() < 1e-12
    p_gcn = {"gcn0.weight": params["evolve.W_init"].T.copy(), "gcn0.bias": np.zeros(F, np.float32)}
    want = oracle.forward(wl.graph, [[0, N, 0, T]], p_gcn, wl.X, wl.X, time_kind="none", act_out="relu")
    assert np.abs(c["Y"] - want).max() < 1e-6
