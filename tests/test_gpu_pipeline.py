"""One worker's share of two training epochs' forward passes, every step on the device against the
chain of oracles: chunk generation (Section 4.1) -> the layer over the generated chunks -> the
stale filter on the changed inputs (Section 5.2), which updates the embedding cache in place ->
the states that left their chunks become the next epoch's state cache -> the layer again."""
import numpy as np
import pytest

from oracle import chunkgen, labelled, stale
from workloads import synth
from refs import rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_two_epochs_over_generated_chunks(kind):
    import torch
    from paper_2309_03523_amd import binding
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F, S = 6, 150, 16, 64
    wl = synth.random_small(123, T, N, F, S, S, 4.0, [[0, N, 0, T]], kind, hub=True)
    g = wl.graph
    V = T * N
    n_state = 2 if kind == "lstm" else 1
    rng = np.random.default_rng(9)
    wl.C = (wl.X + 0.01 * rng.standard_normal(wl.X.shape)).astype(np.float32)    # the cache: copies sent a little earlier
    dw = DeviceWorkload(wl)

    # chunk generation: bit-exact
    lab_d = torch.empty(V, dtype=torch.int32, device="cuda")
    iters, conv = binding.chunk_generate(dw.rowptr, dw.colidx, N, w_s=1, w_t=1, cap=60, max_iters=300, labels=lab_d)
    ref = chunkgen.propagate(g, 1, 1, 60, 300)
    np.testing.assert_array_equal(lab_d.cpu().numpy(), ref["labels"])
    assert (iters, conv) == (ref["iterations"], ref["converged"])
    lab = ref["labels"].reshape(T, N)
    dw.layer.set_labels(lab_d)

    # epoch 1
    Hc0 = (0.3 * rng.standard_normal((n_state * V, S))).astype(np.float32)
    HN = torch.full((n_state * V, S), float("nan"), dtype=torch.float32, device="cuda")
    dw.layer.forward(dw.X, dw.C, dw.Y, H0=torch.from_numpy(Hc0).cuda(), HN=HN)
    torch.cuda.synchronize()
    want_Y, want_HN = labelled.forward(g, lab, wl.params, wl.X, wl.C, time_kind=kind, Hc=Hc0)
    e1 = rel_err(dw.Y.cpu().numpy(), want_Y)
    left = ~np.isnan(want_HN)
    np.testing.assert_array_equal(np.isnan(HN.cpu().numpy()), ~left)
    assert e1 < TOL and rel_err(HN.cpu().numpy()[left], want_HN[left]) < TOL

    # between the epochs: inputs change; boundary rows whose change is large enough are re-sent
    drift = np.where(rng.random((V, 1)) < 0.5, 1.0, 0.002) * rng.standard_normal((V, F))
    X2 = (wl.X.reshape(V, F) + drift).astype(np.float32)
    boundary = np.zeros((T, N), bool)           # rows that some row of another chunk reads
    for t, sn in enumerate(g.snaps):
        row = np.repeat(np.arange(N), np.diff(sn.rowptr))
        cut = lab[t][row] != lab[t][sn.col]
        boundary[t, sn.col[cut]] = True
    cand = np.flatnonzero(boundary.reshape(-1)).astype(np.int64)
    assert 0 < cand.size < V
    theta = 0.5                                 # no distance comes near it: tiny drifts ~0.01, large ones ~4
    want_f = stale.stale_filter(X2, wl.C.reshape(V, F), theta=theta, rows=cand)
    assert np.abs(want_f["dist"] - theta).min() > 0.05
    X2d = torch.from_numpy(X2).cuda()
    Cd = dw.C.reshape(V, F)                     # the layer's cache tensor, updated in place
    dist = torch.empty(cand.size, device="cuda")
    send_idx = torch.full((cand.size,), -1, dtype=torch.int64, device="cuda")
    send_buf = torch.empty(cand.size, F, device="cuda")
    result = torch.zeros(24, dtype=torch.uint8, device="cuda")
    ws = torch.empty(binding.stale_workspace_bytes(cand.size), dtype=torch.uint8, device="cuda")
    binding.stale_filter(X2d, Cd, rows=torch.from_numpy(cand).cuda(), theta=theta, dist=dist, send_idx=send_idx,
                         send_buf=send_buf, result=result, workspace=ws)
    torch.cuda.synchronize()
    k = int(result.cpu().numpy().view(binding.STALE_RESULT_DTYPE)[0]["n_send"])
    np.testing.assert_array_equal(send_idx.cpu().numpy()[:k], want_f["send_idx"])
    np.testing.assert_array_equal(Cd.cpu().numpy(), want_f["L_new"].astype(np.float32))
    assert 0 < k < cand.size

    # the states that left their chunks arrive as the next epoch's state cache (one snapshot later)
    def next_state_cache(hn, old):
        new = old.copy()
        for part in range(n_state):
            src = hn[part * V: part * V + V - N]
            wrote = ~np.isnan(src).any(axis=1)
            new[part * V + N: (part + 1) * V][wrote] = src[wrote]
        return new

    Hc1_dev = next_state_cache(HN.cpu().numpy(), Hc0)        # each side from its own states
    Hc1_ref = next_state_cache(want_HN, Hc0.astype(np.float64))

    # epoch 2
    X2_3d = X2d.reshape(T, N, F)
    dw.layer.forward(X2_3d, dw.C, dw.Y, H0=torch.from_numpy(Hc1_dev).cuda(), HN=HN)
    torch.cuda.synchronize()
    want_Y2, _ = labelled.forward(g, lab, wl.params, X2.reshape(T, N, F), want_f["L_new"].reshape(T, N, F), time_kind=kind,
                                  Hc=Hc1_ref)
    e2 = rel_err(dw.Y.cpu().numpy(), want_Y2)
    print(f"{kind}: {len(np.unique(lab))} chunks after {iters} iterations, {cand.size} boundary rows, {k} re-sent; "
          f"rel_err epoch 1 {e1:.3e}, epoch 2 {e2:.3e}", flush=True)
    assert e2 < TOL
    assert rel_err(want_Y2, want_Y) > 1e-2          # the second epoch really differs
    dw.layer.destroy()
