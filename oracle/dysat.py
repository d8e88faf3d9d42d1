"""CPU oracle of the graph-attention + temporal self-attention layer (the DySAT-style DGNN the
paper trains: Sections 2.1 and 6 name a one-layer graph attention structure encoder and a
one-layer scaled dot-product self-attention time encoder; Section 5.2 gives the stale cache that
out-of-chunk neighbours are read from).

TEST INFRASTRUCTURE ONLY: plain PyTorch CPU operations in float64, one chunk and one snapshot at
a time, no blocking or fusion.  Nothing in the product path may import this module.

Definition (per chunk = vertex range [v_lo, v_hi) x window [t_lo, t_hi), `heads` heads of
D = S / heads dims; all parameters in (out, in) layout):
  structure encoder, snapshot t, row i in the range, neighbours j = the stored CSR row (self-loop
  included):
    z_i = W x_{t,i};   z_j = W x_{t,j} if j is in the range, else W c_{t,j}  (cache, a constant)
    e_ij^h = LeakyReLU_0.2( a_dst^h . z_i^h + a_src^h . z_j^h )
    alpha_ij^h = softmax over j of e_ij^h;   u_i^h = sum_j alpha_ij^h z_j^h;   g_i = ELU(u_i)
  time encoder, vertex i over the chunk's window (causal, inside the window only):
    p_s = g_{s,i} + pos[s];  q, k, v = W_q p, W_k p, W_v p
    A^h_{s,r} = softmax over r <= s of q_s^h . k_r^h / sqrt(D);   y_s^h = sum_r A^h_{s,r} v_r^h
  Y[s,i] = concat_h y_s^h.
Gradients come from reverse-mode differentiation of exactly this forward (torch autograd); the
loss is either sum(dY * Y) for a given upstream gradient or the mean squared error against a
target over all covered elements.
"""
from __future__ import annotations

import math

import numpy as np
import torch

PARAMS = ["gat.weight", "gat.att_src", "gat.att_dst", "attn.pos", "attn.weight_q", "attn.weight_k",
          "attn.weight_v"]


def _t64(a, requires_grad=False):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(torch.float64)
    return t.requires_grad_(requires_grad)


def _structure(snap_rowptr, snap_col, v_lo, v_hi, Xt, Ct, W, a_src, a_dst, heads):
    """u (pre-ELU graph attention output) for rows [v_lo, v_hi) of one snapshot; [nv, S]."""
    nv = v_hi - v_lo
    S = W.shape[0]
    D = S // heads
    lo, hi = int(snap_rowptr[v_lo]), int(snap_rowptr[v_hi])
    cols = torch.from_numpy(snap_col[lo:hi].astype(np.int64))
    deg = np.diff(snap_rowptr[v_lo:v_hi + 1])
    rows = torch.from_numpy(np.repeat(np.arange(nv, dtype=np.int64), deg))
    inside = (cols >= v_lo) & (cols < v_hi)
    src = torch.where(inside[:, None], Xt[cols], Ct[cols])        # [E, F] neighbour inputs
    zj = (src @ W.T).view(-1, heads, D)                            # [E, heads, D]
    zi = (Xt[v_lo:v_hi] @ W.T).view(nv, heads, D)
    s_dst = (zi * a_dst).sum(-1)                                   # [nv, heads]
    s_src = (zj * a_src).sum(-1)                                   # [E, heads]
    e = torch.nn.functional.leaky_relu(s_dst[rows] + s_src, 0.2)
    m = torch.full((nv, heads), -math.inf, dtype=torch.float64).scatter_reduce(
        0, rows[:, None].expand(-1, heads), e.detach(), "amax")
    ex = torch.exp(e - m[rows])
    den = torch.zeros(nv, heads, dtype=torch.float64).index_add(0, rows, ex)
    alpha = ex / den[rows]
    u = torch.zeros(nv, heads, D, dtype=torch.float64).index_add(0, rows, alpha[:, :, None] * zj)
    return u.reshape(nv, S)


def _temporal(G, pos, Wq, Wk, Wv, heads):
    """G [w, nv, S] -> Y [w, nv, S]: causal multi-head attention of every vertex over the window."""
    w, nv, S = G.shape
    D = S // heads
    P = G + pos[:, None, :]
    Q = (P @ Wq.T).view(w, nv, heads, D)
    K = (P @ Wk.T).view(w, nv, heads, D)
    V = (P @ Wv.T).view(w, nv, heads, D)
    scores = torch.einsum("svhd,rvhd->vhsr", Q, K) / math.sqrt(D)
    future = torch.triu(torch.ones(w, w, dtype=torch.bool), diagonal=1)   # r > s
    A = torch.softmax(scores.masked_fill(future, -math.inf), dim=-1)
    return torch.einsum("vhsr,rvhd->svhd", A, V).reshape(w, nv, S)


def _forward_t(graph, chunks, P, X, C, heads):
    """Torch forward; returns (Y [T,N,S] with uncovered rows zero, U likewise, covered mask)."""
    T, N = graph.T, graph.N
    S = P["gat.weight"].shape[0]
    Y = torch.zeros(T, N, S, dtype=torch.float64)
    U = torch.zeros(T, N, S, dtype=torch.float64)
    covered = torch.zeros(T, N, dtype=torch.bool)
    Ys, Us = [], []
    for (v_lo, v_hi, t_lo, t_hi) in np.asarray(chunks, dtype=np.int64).reshape(-1, 4).tolist():
        us = []
        for t in range(t_lo, t_hi):
            s = graph.snaps[t]
            us.append(_structure(s.rowptr, s.col, v_lo, v_hi, X[t], C[t], P["gat.weight"], P["gat.att_src"],
                                 P["gat.att_dst"], heads))
        u = torch.stack(us)                                          # [w, nv, S]
        y = _temporal(torch.nn.functional.elu(u), P["attn.pos"][t_lo:t_hi], P["attn.weight_q"],
                      P["attn.weight_k"], P["attn.weight_v"], heads)
        Ys.append((v_lo, v_hi, t_lo, t_hi, y))
        Us.append(u)
        covered[t_lo:t_hi, v_lo:v_hi] = True
    # assemble without in-place writes into a leaf (keeps autograd simple)
    Yfull = Y.clone()
    Ufull = U.clone()
    for (v_lo, v_hi, t_lo, t_hi, y), u in zip(Ys, Us):
        Yfull[t_lo:t_hi, v_lo:v_hi] = y
        Ufull[t_lo:t_hi, v_lo:v_hi] = u.detach()
    return Yfull, Ufull, covered


def forward(graph, chunks, params, X, C, heads):
    """Y [T,N,S] float64 (rows no chunk covers are zero) and the pre-ELU structure output U."""
    with torch.no_grad():
        P = {k: _t64(params[k]) for k in PARAMS}
        Y, U, _ = _forward_t(graph, chunks, P, _t64(X), _t64(C), heads)
    return {"Y": Y.numpy(), "U": U.numpy()}


def gradients(graph, chunks, params, X, C, heads, *, target=None, dY=None, want_dx=False):
    """Forward + gradients of the loss with respect to every parameter (and, with want_dx, the
    input X: "dX", zero on rows no chunk covers).  Exactly one of target (mean squared error
    over the covered elements) and dY (loss = sum(dY * Y) over the covered elements).  The cache
    is a constant.  Returns dict(Y, loss, grads[, dX])."""
    assert (target is None) != (dY is None)
    P = {k: _t64(params[k], True) for k in PARAMS}
    Xt = _t64(X, want_dx)
    Y, _, covered = _forward_t(graph, chunks, P, Xt, _t64(C), heads)
    cm = covered[:, :, None].to(torch.float64)
    if target is not None:
        count = float(covered.sum().item() * Y.shape[2])
        loss = (((Y - _t64(target)) ** 2) * cm).sum() / count
    else:
        loss = (Y * _t64(dY) * cm).sum()
    loss.backward()
    out = {"Y": Y.detach().numpy(), "loss": float(loss.item()),
           "grads": {k: P[k].grad.numpy() for k in PARAMS}}
    if want_dx:
        out["dX"] = Xt.grad.numpy()
    return out
