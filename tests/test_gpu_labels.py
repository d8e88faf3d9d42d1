"""Generated (labelled) chunks as the layer's input on the GPU against the oracle: random
labels, labels from the device label propagation, rectangular labels against the rectangular
layer, re-labelling, refusals."""
import numpy as np
import pytest

import oracle
from oracle import labelled
from workloads import synth
from refs import rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _device(wl, labels, Hc, **kw):
    """Forward of a one-chunk layer with labels; returns Y, HN (NaN where not written)."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    dw = DeviceWorkload(wl, **kw)
    dw.layer.set_labels(torch.from_numpy(np.ascontiguousarray(labels, np.int32).reshape(-1)).cuda())
    T, N = wl.graph.T, wl.graph.N
    HN = None
    H0 = None
    if wl.time_kind != "none":
        n_state = 2 if wl.time_kind == "lstm" else 1
        HN = torch.full((n_state * T * N, wl.H), float("nan"), dtype=torch.float32, device="cuda")
        H0 = torch.from_numpy(Hc.astype(np.float32)).cuda() if Hc is not None else None
    dw.layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=H0, HN=HN)
    torch.cuda.synchronize()
    return dw, dw.Y.cpu().numpy(), (HN.cpu().numpy() if HN is not None else None)


def _check(wl, labels, Hc, Y, HN, layers, tag):
    want, want_HN = labelled.forward(wl.graph, labels, wl.params, wl.X, wl.C, time_kind=wl.time_kind,
                                     n_struct_layers=layers, C1=wl.C1, Hc=Hc)
    e_y = rel_err(Y, want)
    msg = f"{tag}: rel_err Y {e_y:.3e}"
    assert e_y < TOL, msg
    if want_HN is not None:
        m = ~np.isnan(want_HN)
        np.testing.assert_array_equal(np.isnan(HN), ~m)       # written exactly where a state leaves a chunk
        e_h = rel_err(HN[m], want_HN[m])
        msg += f" HN {e_h:.3e} ({int(m.any(axis=1).sum())} state rows leave their chunk)"
        assert e_h < TOL, msg
    print(msg, flush=True)


def _random_labels(rng, T, N, n_labels, p_keep):
    """Blocky random labels: a vertex keeps its label from one snapshot to the next with
    probability p_keep, neighbours in index tend to share labels."""
    lab = np.zeros((T, N), np.int64)
    lab[0] = np.sort(rng.integers(0, n_labels, N))
    for t in range(1, T):
        keep = rng.random(N) < p_keep
        lab[t] = np.where(keep, lab[t - 1], rng.integers(0, n_labels, N))
    return lab


@pytest.mark.parametrize("kind,S,layers,dense", [("gru", 64, 1, "auto"), ("gru", 96, 1, "tile"), ("lstm", 128, 2, "auto"),
                                                   ("lstm", 32, 1, "tile"), ("none", 64, 2, "auto")])
def test_random_labels(kind, S, layers, dense):
    T, N, F = 6, 150, 20
    wl = synth.random_small(90 + S, T, N, F, S, S, 4.0, [[0, N, 0, T]], kind, n_struct_layers=layers, hub=True)
    rng = np.random.default_rng(S)
    lab = _random_labels(rng, T, N, 7, 0.7)
    n_state = 2 if kind == "lstm" else 1
    Hc = (0.5 * rng.standard_normal((n_state * T * N, S))).astype(np.float32) if kind != "none" else None
    dw, Y, HN = _device(wl, lab, Hc, dense_kernel=dense)
    _check(wl, lab, Hc, Y, HN, layers, f"random labels {kind} S={S} layers={layers} {dense}")
    dw.layer.destroy()


def test_labels_from_label_propagation_and_relabelling():
    """The device label propagation's output goes straight into the layer; then other labels
    replace them on the same layer."""
    import torch
    from paper_2309_03523_amd import binding
    T, N, F, S = 5, 120, 12, 32
    wl = synth.random_small(77, T, N, F, S, S, 5.0, [[0, N, 0, T]], "gru")
    rp = [torch.from_numpy(s.rowptr).cuda() for s in wl.graph.snaps]
    ci = [torch.from_numpy(s.col).cuda() for s in wl.graph.snaps]
    labels = torch.empty(T * N, dtype=torch.int32, device="cuda")
    iters, conv = binding.chunk_generate(rp, ci, N, w_s=2, w_t=1, cap=40, max_iters=200, labels=labels)
    lab = labels.cpu().numpy().reshape(T, N)
    n_chunks = len(np.unique(lab))
    assert 1 < n_chunks < T * N
    rng = np.random.default_rng(1)
    Hc = (0.5 * rng.standard_normal((T * N, S))).astype(np.float32)
    dw, Y, HN = _device(wl, lab, Hc)
    _check(wl, lab, Hc, Y, HN, 1, f"label propagation ({n_chunks} chunks, {iters} iterations)")
    lab2 = _random_labels(rng, T, N, 3, 0.5)
    dw.layer.set_labels(torch.from_numpy(lab2.astype(np.int32).reshape(-1)).cuda())
    HN2 = torch.full((T * N, S), float("nan"), dtype=torch.float32, device="cuda")
    dw.layer.forward(dw.X, dw.C, dw.Y, H0=torch.from_numpy(Hc).cuda(), HN=HN2)
    torch.cuda.synchronize()
    _check(wl, lab2, Hc, dw.Y.cpu().numpy(), HN2.cpu().numpy(), 1, "after re-labelling")
    dw.layer.destroy()


def test_rectangular_labels_equal_the_rectangular_layer():
    """Labels that are vertex ranges x windows: the same numbers as the layer created with those
    rectangles (device against device, same kernels on other tables)."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F, S = 6, 140, 16, 64
    rect = np.array([[0, 50, 0, 6], [50, 140, 0, 2], [50, 140, 2, 6]], np.int64)
    wl = synth.random_small(55, T, N, F, S, S, 4.0, rect, "lstm", hub=True)
    dr = DeviceWorkload(wl)
    Yr, HNr = dr.forward(want_state=True)
    Yr, HNr = Yr.cpu().numpy(), HNr.cpu().numpy()
    dr.layer.destroy()
    import dataclasses
    one = dataclasses.replace(wl, chunks=np.array([[0, N, 0, T]], np.int64))
    V = T * N
    tot = int((rect[:, 1] - rect[:, 0]).sum())
    Hc = np.zeros((2 * V, S), np.float32)
    off = 0
    for v_lo, v_hi, t_lo, _ in rect.tolist():
        for part in range(2):
            Hc[part * V + t_lo * N + v_lo: part * V + t_lo * N + v_hi] = wl.H0[part * tot + off: part * tot + off + v_hi - v_lo]
        off += v_hi - v_lo
    dw, Y, HN = _device(one, labelled.labels_of_chunks(rect, T, N), Hc)
    assert rel_err(Y, Yr.astype(np.float64)) < 1e-5
    off = 0
    for v_lo, v_hi, _, t_hi in rect.tolist():
        for part in range(2):
            got = HN[part * V + (t_hi - 1) * N + v_lo: part * V + (t_hi - 1) * N + v_hi]
            assert rel_err(got, HNr[part * tot + off: part * tot + off + v_hi - v_lo].astype(np.float64)) < 1e-5
        off += v_hi - v_lo
    dw.layer.destroy()


def test_label_refusals():
    import torch
    from paper_2309_03523_amd.binding import DgcError
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N = 4, 40
    lab = torch.zeros(T * N, dtype=torch.int32, device="cuda")
    wl = synth.random_small(3, T, N, 8, 32, 32, 3.0, [[0, 20, 0, T], [20, N, 0, T]], "gru")
    dw = DeviceWorkload(wl)
    with pytest.raises(DgcError) as ei:           # needs the single all-covering chunk
        dw.layer.set_labels(lab)
    assert ei.value.code == 7
    dw.layer.destroy()
    wl = synth.random_small(3, T, N, 8, 32, 32, 3.0, [[0, N, 0, T]], "gru")
    dw = DeviceWorkload(wl, gather_mode="staged")
    with pytest.raises(DgcError) as ei:
        dw.layer.set_labels(lab)
    assert ei.value.code == 4
    dw.layer.destroy()
    dw = DeviceWorkload(wl)
    dw.layer.set_labels(lab)
    with pytest.raises(DgcError) as ei:           # the sequences are the labels' own
        dw.forward(use_h0=False, reset_mask=np.zeros((T, N), np.uint8))
    assert ei.value.code == 1
    with pytest.raises(ValueError):
        dw.layer.set_labels(lab[:-1])
    dw.layer.destroy()


@pytest.mark.parametrize("seed", range(8))
def test_random_shapes_and_labellings(seed):
    """Tiny and ragged shapes (one vertex, one snapshot, one label, all labels different), both
    dense kernels, every time encoder, with and without a state cache."""
    rng = np.random.default_rng(8000 + seed)
    N = int(rng.choice([1, 2, 31, 33, 64, 97]))
    T = int(rng.integers(1, 7))
    kind = str(rng.choice(["gru", "lstm", "none"]))
    S = int(rng.choice([32, 64, 96]))
    layers = int(rng.choice([1, 2]))
    F = int(rng.choice([1, 5, 32, 40]))
    wl = synth.random_small(8100 + seed, T, N, F, S, S, 3.0, [[0, N, 0, T]], kind, n_struct_layers=layers)
    mode = seed % 4
    if mode == 0:
        lab = np.zeros((T, N), np.int64)                       # one chunk
    elif mode == 1:
        lab = np.arange(T * N).reshape(T, N)                   # every pair its own chunk
    else:
        lab = _random_labels(rng, T, N, int(rng.integers(2, 6)), float(rng.choice([0.3, 0.8])))
    n_state = 2 if kind == "lstm" else 1
    Hc = None
    if kind != "none" and seed % 2 == 0:
        Hc = (0.5 * rng.standard_normal((n_state * T * N, S))).astype(np.float32)
    dw, Y, HN = _device(wl, lab, Hc, dense_kernel=str(rng.choice(["auto", "tile"])))
    _check(wl, lab, Hc, Y, HN, layers, f"seed {seed}: N={N} T={T} F={F} S={S} {kind} layers={layers} labelling {mode} "
                                       f"cache={'yes' if Hc is not None else 'no'}")
    dw.layer.destroy()


@pytest.mark.parametrize("F,agg", [(32, "table"), (64, "walk"), (128, "table"), (256, "table")])
def test_evolving_weights_over_generated_chunks(F, agg):
    """EvolveGCN-O with labels: outputs, loss, the ten parameter gradients and the input gradient against
    the labelled oracle (torch float64 autograd on the definition); split hub rows included."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N = 5, 140
    wl = synth.random_small(400 + F, T, N, F, F, F, 4.0, [[0, N, 0, T]], "none", hub=True)
    wl.params = synth.evolve_params(400 + F, F, F, random_bias=True)
    rng = np.random.default_rng(F)
    lab = _random_labels(rng, T, N, 5, 0.7)
    target = synth.stream(F, "target-lab").standard_normal((T, N, F)).astype(np.float32)
    dw = DeviceWorkload(wl, struct_kind="evolve_gcn_o", act_out="relu", agg_kernel=agg, long_nnz=24, part_nnz=8)
    dw.layer.set_labels(torch.from_numpy(lab.astype(np.int32).reshape(-1)).cuda())
    Y = dw.forward()
    want = labelled.evolve(wl.graph, lab, wl.params, wl.X, wl.C, target, want_dx=True)
    e_y = rel_err(Y.cpu().numpy(), want["Y"])
    tgt = torch.from_numpy(target).cuda()
    loss = torch.zeros(1, device="cuda")
    dX = torch.full((T, N, F), float("nan"), device="cuda")
    dw.layer.backward(Y, target=tgt, loss_out=loss, dX=dX)
    torch.cuda.synchronize()
    assert e_y < TOL and abs(loss.item() - want["loss"]) < 1e-5 * want["loss"]
    worst = 0.0
    for name in oracle.EVOLVE_PARAMS:
        g = dw.layer.get_param(name + ".grad", wl.params[name].shape)
        worst = max(worst, rel_err(g, want["grads"][name]))
    e_x = rel_err(dX.cpu().numpy(), want["dX"])
    print(f"EvolveGCN-O over labels F={F} {agg}: Y {e_y:.2e}, parameter gradients {worst:.2e}, dX {e_x:.2e}", flush=True)
    assert worst < TOL and e_x < TOL
    dw.layer.destroy()
