"""Temporal fusion over generated chunks on the GPU (dgc_layer_set_labels, then
dgc_layer_set_presence) against the oracle: the lane packing bit for bit, the outputs and the
states that leave their chunks; all-present and one-label cases against the layers they reduce to;
labels from the device label propagation; refusals."""
import numpy as np
import pytest

from oracle import labelled
from workloads import synth
from refs import parity_str, rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _random_labels(rng, T, N, n_labels, p_keep):
    lab = np.zeros((T, N), np.int64)
    lab[0] = np.sort(rng.integers(0, n_labels, N))
    for t in range(1, T):
        keep = rng.random(N) < p_keep
        lab[t] = np.where(keep, lab[t - 1], rng.integers(0, n_labels, N))
    return lab


def _device(wl, labels, present, Hc, **kw):
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    dw = DeviceWorkload(wl, **kw)
    dw.layer.set_labels(torch.from_numpy(np.ascontiguousarray(labels, np.int32).reshape(-1)).cuda())
    dw.layer.set_presence(torch.from_numpy(np.ascontiguousarray(present, np.uint8)).cuda())
    T, N = wl.graph.T, wl.graph.N
    n_state = 2 if wl.time_kind == "lstm" else 1
    HN = torch.full((n_state * T * N, wl.H), float("nan"), dtype=torch.float32, device="cuda")
    H0 = torch.from_numpy(Hc.astype(np.float32)).cuda() if Hc is not None else None
    dw.Y.fill_(float("nan"))
    dw.layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=H0, HN=HN)
    torch.cuda.synchronize()
    return dw, dw.Y.cpu().numpy(), HN.cpu().numpy()


def _check(wl, labels, present, Hc, dw, Y, HN, layers, tag):
    T, N = wl.graph.T, wl.graph.N
    p = labelled.pack(labels, present)
    lane_ptr = dw.layer.packing("lane_ptr")
    assert lane_ptr.tolist() == [0, p["n_lanes"]]
    if p["n_lanes"]:
        np.testing.assert_array_equal(dw.layer.packing("slot_row").reshape(T, -1), p["slot_row"])
        np.testing.assert_array_equal(dw.layer.packing("slot_reset").reshape(T, -1), p["slot_reset"])
    want, want_HN = labelled.forward(wl.graph, labels, wl.params, wl.X, wl.C, time_kind=wl.time_kind,
                                     n_struct_layers=layers, C1=wl.C1, Hc=Hc, present=present)
    here = present.astype(bool)
    assert np.isnan(Y[~here]).all() and not np.isnan(Y[here]).any()          # absent rows are not written
    msg = f"{tag}: {p['n_lanes']} lanes for {int(here.sum())} instances of {T * N}"
    if here.any():
        e_y = rel_err(Y[here], want[here])
        msg += f"; Y {parity_str(Y[here], want[here])}"
        assert e_y < TOL, msg
    m = ~np.isnan(want_HN)
    np.testing.assert_array_equal(np.isnan(HN), ~m)           # written exactly where a sequence ends
    if m.any():
        e_h = rel_err(HN[m], want_HN[m])
        msg += f"; HN {e_h:.3e} ({int(m.any(axis=1).sum())} state rows)"
        assert e_h < TOL, msg
    print(msg, flush=True)


@pytest.mark.parametrize("kind,S,layers,dense", [("gru", 64, 1, "auto"), ("gru", 96, 1, "tile"), ("lstm", 128, 2, "auto"),
                                                   ("lstm", 32, 1, "tile"), ("gru", 128, 2, "auto")])
def test_random_labels_and_presence(kind, S, layers, dense):
    T, N, F = 7, 170, 20
    wl = synth.random_small(190 + S, T, N, F, S, S, 4.0, [[0, N, 0, T]], kind, n_struct_layers=layers, hub=True)
    rng = np.random.default_rng(S + 1)
    lab = _random_labels(rng, T, N, 6, 0.7)
    present = synth.presence(S, T, N)
    n_state = 2 if kind == "lstm" else 1
    Hc = (0.5 * rng.standard_normal((n_state * T * N, S))).astype(np.float32)
    dw, Y, HN = _device(wl, lab, present, Hc, dense_kernel=dense)
    _check(wl, lab, present, Hc, dw, Y, HN, layers, f"labels + presence {kind} S={S} layers={layers} {dense}")
    dw.layer.destroy()


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes(seed):
    rng = np.random.default_rng(700 + seed)
    T = int(rng.choice([1, 2, 5, 9]))
    N = int(rng.choice([1, 3, 33, 64, 101]))
    kind = str(rng.choice(["gru", "lstm"]))
    S = int(rng.choice([32, 64, 128]))
    layers = int(rng.integers(1, 3))
    wl = synth.random_small(800 + seed, T, N, 12, S, S, float(rng.choice([0.0, 3.0])), [[0, N, 0, T]], kind,
                            n_struct_layers=layers, hub=bool(rng.integers(0, 2)))
    lab = _random_labels(rng, T, N, int(rng.integers(1, 5)), float(rng.choice([0.3, 0.9])))
    p = rng.random(N) * rng.choice([1.0, 0.5])
    present = (rng.random((T, N)) < np.maximum(p, 0.1)[None, :]).astype(np.uint8)
    if seed == 3:
        present[:] = 0                    # nobody is ever present
    Hc = (0.5 * rng.standard_normal(((2 if kind == "lstm" else 1) * T * N, S))).astype(np.float32) if seed % 2 == 0 else None
    dw, Y, HN = _device(wl, lab, present, Hc)
    _check(wl, lab, present, Hc, dw, Y, HN, layers, f"seed {seed}: T={T} N={N} {kind} S={S} layers={layers}")
    dw.layer.destroy()


def test_all_present_equals_the_labelled_layer_and_one_label_the_fused_rectangle():
    """Device against device: with every instance present the result is the labelled layer's bit for
    bit in Y where a vertex keeps its label over the whole window (same kernels, other tables);
    with one label it is temporal fusion of the single rectangle."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, S = 6, 120, 64
    wl = synth.random_small(321, T, N, 16, S, S, 4.0, [[0, N, 0, T]], "gru", hub=True)
    rng = np.random.default_rng(5)
    lab = _random_labels(rng, T, N, 5, 0.8)
    Hc = (0.5 * rng.standard_normal((T * N, S))).astype(np.float32)
    ones = np.ones((T, N), np.uint8)
    dw, Y, HN = _device(wl, lab, ones, Hc)
    dw2 = DeviceWorkload(wl)
    dw2.layer.set_labels(torch.from_numpy(lab.astype(np.int32).reshape(-1)).cuda())
    HN2 = torch.full((T * N, S), float("nan"), device="cuda")
    dw2.layer.forward(dw2.X, dw2.C, dw2.Y, H0=torch.from_numpy(Hc).cuda(), HN=HN2)
    torch.cuda.synchronize()
    assert rel_err(Y, dw2.Y.cpu().numpy()) < 2e-6
    np.testing.assert_array_equal(np.isnan(HN), np.isnan(HN2.cpu().numpy()))
    dw.layer.destroy(); dw2.layer.destroy()
    # one label + presence: the fused rectangle, states re-indexed
    present = synth.presence(11, T, N)
    one = np.zeros((T, N), np.int64)
    H0 = (0.5 * rng.standard_normal((N, S))).astype(np.float32)
    Hc1 = np.zeros((T * N, S), np.float32)
    for i in range(N):
        ts = np.flatnonzero(present[:, i])
        if len(ts):
            Hc1[ts[0] * N + i] = H0[i]
    dw, Y, HN = _device(wl, one, present, Hc1)
    dw3 = DeviceWorkload(wl)
    dw3.layer.set_presence(torch.from_numpy(present).cuda())
    dw3.Y.fill_(float("nan"))
    HN3 = torch.zeros((N, S), device="cuda")
    dw3.layer.forward(dw3.X, dw3.C, dw3.Y, H0=torch.from_numpy(H0).cuda(), HN=HN3)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Y, dw3.Y.cpu().numpy())             # same lanes, same kernels: bit for bit
    HN3 = HN3.cpu().numpy()
    for i in range(N):
        ts = np.flatnonzero(present[:, i])
        if len(ts):
            np.testing.assert_array_equal(HN[ts[-1] * N + i], HN3[i])
    dw.layer.destroy(); dw3.layer.destroy()


def test_labels_from_label_propagation_with_presence():
    """Labels straight from dgc_chunk_generate on the same graph, then a presence matrix."""
    import torch
    from paper_2309_03523_amd import binding
    T, N, S = 6, 300, 64
    wl = synth.random_small(55, T, N, 24, S, S, 5.0, [[0, N, 0, T]], "gru", hub=True)
    from paper_2309_03523_amd.runner import DeviceWorkload
    dw = DeviceWorkload(wl)
    labels = torch.empty(T * N, dtype=torch.int32, device="cuda")
    rp = [torch.from_numpy(s.rowptr).cuda() for s in wl.graph.snaps]
    ci = [torch.from_numpy(s.col).cuda() for s in wl.graph.snaps]
    binding.chunk_generate(rp, ci, N, w_s=2, w_t=1, cap=200, max_iters=200, labels=labels)
    lab = labels.cpu().numpy().reshape(T, N).astype(np.int64)
    assert len(np.unique(lab)) > 1
    present = synth.presence(77, T, N)
    rng = np.random.default_rng(9)
    Hc = (0.5 * rng.standard_normal((T * N, S))).astype(np.float32)
    dw.layer.set_labels(labels)
    dw.layer.set_presence(torch.from_numpy(present).cuda())
    HN = torch.full((T * N, S), float("nan"), device="cuda")
    dw.Y.fill_(float("nan"))
    dw.layer.forward(dw.X, dw.C, dw.Y, H0=torch.from_numpy(Hc).cuda(), HN=HN)
    torch.cuda.synchronize()
    _check(wl, lab, present, Hc, dw, dw.Y.cpu().numpy(), HN.cpu().numpy(), 1, f"label propagation ({len(np.unique(lab))} chunks) + presence")
    dw.layer.destroy()


def test_refusals():
    import torch
    from paper_2309_03523_amd.binding import DgcError
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, S = 4, 40, 32
    wl = synth.random_small(5, T, N, 8, S, S, 3.0, [[0, N, 0, T]], "gru")
    lab = torch.zeros(T * N, dtype=torch.int32, device="cuda")
    present = torch.ones((T, N), dtype=torch.uint8, device="cuda")
    dw = DeviceWorkload(wl)
    dw.layer.set_labels(lab)
    dw.layer.set_presence(present)
    with pytest.raises(DgcError) as ei:          # labels come first, and not again afterwards
        dw.layer.set_labels(lab)
    assert ei.value.code == 7
    with pytest.raises(DgcError) as ei:          # once per layer
        dw.layer.set_presence(present)
    assert ei.value.code == 7
    dw.layer.destroy()
    dw = DeviceWorkload(wl)
    dw.layer.set_presence(present)
    with pytest.raises(DgcError) as ei:          # labels after presence
        dw.layer.set_labels(lab)
    assert ei.value.code == 7
    dw.layer.destroy()
