"""Temporal fusion on the GPU against the oracle: the lane packing bit-exact, the layer's output on
every present row within the fp32 tolerance, absent rows untouched."""
import numpy as np
import pytest

import oracle
from oracle import tfusion
from workloads import synth
from refs import rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4
CHUNKS = [[0, 70, 0, 8], [70, 201, 0, 5], [70, 201, 5, 8], [201, 260, 2, 8]]


def _run(kind, S, n_layers, seed, dense="auto"):
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F = 8, 260, 48
    wl = synth.random_small(seed, T, N, F, S, S, 4.0, CHUNKS, kind, n_struct_layers=n_layers, hub=True)
    present = synth.presence(seed, T, N)
    dw = DeviceWorkload(wl, dense_kernel=dense)
    dw.layer.set_presence(torch.from_numpy(present).cuda())
    got_pack = {k: dw.layer.packing(k) for k in ("lane_ptr", "slot_row", "slot_reset")}
    want_pack = tfusion.pack(present, wl.chunks)
    np.testing.assert_array_equal(got_pack["lane_ptr"], want_pack["lane_ptr"])
    np.testing.assert_array_equal(got_pack["slot_row"].reshape(want_pack["slot_row"].shape), want_pack["slot_row"])
    np.testing.assert_array_equal(got_pack["slot_reset"].reshape(want_pack["slot_reset"].shape), want_pack["slot_reset"])
    Y = dw.forward(use_h0=False).cpu().numpy()
    Z = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", n_struct_layers=n_layers,
                       C1=wl.C1, act_hidden="relu", act_out="none").astype(np.float64)
    want = tfusion.run_separate(np.nan_to_num(Z), present, wl.chunks, wl.params, kind)
    m = ~np.isnan(want)
    assert m.sum() > 500
    e = rel_err(Y[m], want[m])
    print(f"{kind} S={S} layers={n_layers} {dense}: lanes {want_pack['slot_row'].shape[1]} for "
          f"{int(m.any(axis=2).sum())} present rows, rel_err {e:.3e}", flush=True)
    assert e < TOL
    assert np.isnan(Y[~m.any(axis=2)]).all()       # absent and uncovered rows are not written
    return dw


@pytest.mark.parametrize("kind,S,n_layers,dense", [("gru", 64, 1, "auto"), ("gru", 96, 1, "tile"), ("lstm", 128, 1, "auto"),
                                                   ("lstm", 32, 2, "auto")])
def test_temporal_fusion_parity(kind, S, n_layers, dense):
    dw = _run(kind, S, n_layers, 20 + S, dense)
    dw.layer.destroy()


def test_temporal_fusion_errors():
    import torch
    from paper_2309_03523_amd.binding import DgcError
    from paper_2309_03523_amd.runner import DeviceWorkload
    dw = _run("gru", 32, 1, 7)
    present = torch.ones(8, 260, dtype=torch.uint8, device="cuda")
    with pytest.raises(DgcError) as ei:          # once per layer
        dw.layer.set_presence(present)
    assert ei.value.code == 7
    with pytest.raises(DgcError) as ei:          # the reset flags are the packing's own
        dw.forward(use_h0=False, reset_mask=np.zeros((8, 260), np.uint8))
    assert ei.value.code == 1
    dw.layer.destroy()
    wl = synth.random_small(3, 4, 40, 32, 32, 32, 3.0, [[0, 40, 0, 4]], "none")
    dw2 = DeviceWorkload(wl)
    with pytest.raises(DgcError) as ei:          # needs a recurrent time encoder
        dw2.layer.set_presence(torch.ones(4, 40, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == 4
    with pytest.raises(DgcError) as ei:          # no packing to read
        dw2.layer.packing("slot_row")
    assert ei.value.code == 7
    dw2.layer.destroy()


@pytest.mark.parametrize("seed", range(10))
def test_temporal_fusion_random_shapes(seed):
    """Random chunk sets and presence patterns: nobody present, everybody present, tiny vertex
    counts, windows of one snapshot, gaps in the coverage."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    rng = np.random.default_rng(5000 + seed)
    N = int(rng.choice([1, 2, 7, 33, 64, 100]))
    T = int(rng.integers(1, 7))
    cuts = sorted(set([0, N] + rng.integers(0, N + 1, size=rng.integers(0, 3)).tolist()))
    chunks = []
    for a, b in zip(cuts, cuts[1:]):
        tcuts = sorted(set([0, T] + rng.integers(0, T + 1, size=rng.integers(0, 3)).tolist()))
        chunks += [[a, b, t0, t1] for t0, t1 in zip(tcuts, tcuts[1:]) if rng.random() < 0.85]
    if not chunks:
        chunks = [[0, N, 0, T]]
    kind = str(rng.choice(["gru", "lstm"]))
    S = int(rng.choice([32, 64]))
    layers = int(rng.choice([1, 2]))
    wl = synth.random_small(6000 + seed, T, N, 5, S, S, 3.0, chunks, kind, n_struct_layers=layers)
    p_lo, p_hi = [(0.0, 0.0), (1.0, 1.0), (0.1, 1.0), (0.0, 0.6)][seed % 4]
    present = synth.presence(seed, T, N, p_lo, p_hi)
    dw = DeviceWorkload(wl, dense_kernel=str(rng.choice(["auto", "tile"])))
    dw.layer.set_presence(torch.from_numpy(present).cuda())
    want_pack = tfusion.pack(present, wl.chunks)
    np.testing.assert_array_equal(dw.layer.packing("lane_ptr"), want_pack["lane_ptr"])
    np.testing.assert_array_equal(dw.layer.packing("slot_row").reshape(want_pack["slot_row"].shape), want_pack["slot_row"])
    np.testing.assert_array_equal(dw.layer.packing("slot_reset").reshape(want_pack["slot_reset"].shape),
                                  want_pack["slot_reset"])
    Y = dw.forward(use_h0=False).cpu().numpy()
    Z = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", n_struct_layers=layers,
                       C1=wl.C1, act_hidden="relu", act_out="none").astype(np.float64)
    want = tfusion.run_separate(np.nan_to_num(Z), present, wl.chunks, wl.params, kind)
    m = ~np.isnan(want)
    print(f"seed {seed}: N={N} T={T} chunks={len(chunks)} {kind} S={S} layers={layers} p=({p_lo},{p_hi}) "
          f"present rows {int(m.any(axis=2).sum())}, lanes {want_pack['slot_row'].shape[1]}", flush=True)
    if m.any():
        assert rel_err(Y[m], want[m]) < TOL
    assert np.isnan(Y[~m.any(axis=2)]).all()
    dw.layer.destroy()


def _states(kind, S, seed, dense, chunks=CHUNKS, T=8, N=260, p=(0.0, 1.0), use_h0=True):
    """Forward with initial states: Y and HN against every sequence run by itself from its row."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    wl = synth.random_small(seed, T, N, 24, S, S, 4.0, chunks, kind, hub=True)
    present = synth.presence(seed, T, N, *p)
    dw = DeviceWorkload(wl, dense_kernel=dense)
    dw.layer.set_presence(torch.from_numpy(present).cuda())
    Y, HN = dw.forward(use_h0=use_h0, want_state=True)
    Y, HN = Y.cpu().numpy(), HN.cpu().numpy()
    Z = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", C1=wl.C1, act_hidden="relu",
                       act_out="none").astype(np.float64)
    H0 = wl.H0.astype(np.float64) if use_h0 else None
    want, want_HN = tfusion.run_separate(np.nan_to_num(Z), present, wl.chunks, wl.params, kind, H0=H0, return_state=True)
    m = ~np.isnan(want)
    assert not np.isnan(HN).any()                  # every state row is written
    e_y = rel_err(Y[m], want[m]) if m.any() else 0.0
    e_h = rel_err(HN, want_HN) if np.abs(want_HN).max() > 0 else float(np.abs(HN).max())
    # rows of vertices that never appear: the state passes through bit for bit
    off = tfusion.state_rows(wl.chunks)
    idle = np.concatenate([~present[t0:t1, a:b].any(axis=0) for a, b, t0, t1 in np.asarray(wl.chunks).tolist()])
    V = int(off[-1])
    for part in range(HN.shape[0] // V):
        got = HN[part * V:(part + 1) * V][idle]
        ref = wl.H0[part * V:(part + 1) * V][idle] if use_h0 else np.zeros_like(got)
        np.testing.assert_array_equal(got, ref)
    print(f"{kind} S={S} {dense} h0={use_h0}: present rows {int(m.any(axis=2).sum())}, idle state rows {int(idle.sum())}, "
          f"rel_err Y {e_y:.3e} HN {e_h:.3e}", flush=True)
    assert e_y < TOL and e_h < TOL
    assert np.isnan(Y[~m.any(axis=2)]).all()
    dw.layer.destroy()


@pytest.mark.parametrize("kind,S,dense,use_h0", [("gru", 64, "auto", True), ("gru", 96, "tile", True),
                                                   ("lstm", 128, "auto", True), ("lstm", 64, "tile", True),
                                                   ("gru", 32, "auto", False), ("lstm", 32, "tile", False)])
def test_temporal_fusion_states(kind, S, dense, use_h0):
    _states(kind, S, 300 + S, dense, use_h0=use_h0)


@pytest.mark.parametrize("seed", range(6))
def test_temporal_fusion_states_random_shapes(seed):
    rng = np.random.default_rng(7000 + seed)
    N = int(rng.choice([1, 3, 40, 65, 130]))
    T = int(rng.integers(1, 7))
    cuts = sorted(set([0, N] + rng.integers(0, N + 1, size=rng.integers(0, 3)).tolist()))
    chunks = []
    for a, b in zip(cuts, cuts[1:]):
        tcuts = sorted(set([0, T] + rng.integers(0, T + 1, size=rng.integers(0, 3)).tolist()))
        chunks += [[a, b, t0, t1] for t0, t1 in zip(tcuts, tcuts[1:])]
    p = [(0.0, 0.0), (1.0, 1.0), (0.1, 1.0), (0.0, 0.6)][seed % 4]
    _states(str(rng.choice(["gru", "lstm"])), int(rng.choice([32, 64])), 7100 + seed, str(rng.choice(["auto", "tile"])),
            chunks=chunks, T=T, N=N, p=p)


@pytest.mark.parametrize("kind,dense", [("gru", "auto"), ("lstm", "tile")])
def test_temporal_fusion_chained_windows(kind, dense):
    """Two layers over the two halves of a window, the second fed the first one's final states,
    against one layer over the whole window: the same outputs and final states."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, S = 8, 150, 64
    ranges = [[0, 64], [64, 150]]
    whole = [[a, b, 0, T] for a, b in ranges]
    wl = synth.random_small(41, T, N, 16, S, S, 4.0, whole, kind)
    present = synth.presence(41, T, N)
    dev_present = torch.from_numpy(present).cuda()
    dw = DeviceWorkload(wl, dense_kernel=dense)
    dw.layer.set_presence(dev_present)
    Y_all, HN_all = dw.forward(want_state=True)
    Y_all, HN_all = Y_all.cpu().numpy(), HN_all.clone()
    dw.layer.destroy()
    state = torch.from_numpy(wl.H0).cuda()
    Y_parts = np.full_like(Y_all, np.nan)
    for t0, t1 in ((0, 3), (3, T)):
        import dataclasses
        part = dataclasses.replace(wl, chunks=np.asarray([[a, b, t0, t1] for a, b in ranges], np.int64))
        dp = DeviceWorkload(part, dense_kernel=dense)
        dp.layer.set_presence(dev_present)
        dp.H0 = state
        Yp, state = dp.forward(want_state=True)
        Y_parts[t0:t1] = Yp.cpu().numpy()[t0:t1]
        state = state.clone()
        dp.layer.destroy()
    m = ~np.isnan(Y_all)
    np.testing.assert_array_equal(np.isnan(Y_parts), ~m)
    # the same arithmetic in the same order: equal up to the rounding of a different tile placement
    assert rel_err(Y_parts[m], Y_all[m].astype(np.float64)) < 1e-5
    assert rel_err(state.cpu().numpy(), HN_all.cpu().numpy().astype(np.float64)) < 1e-5
