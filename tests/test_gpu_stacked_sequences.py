"""The stacked time encoder (two recurrent layers, Section 6's MPNN-LSTM) over sequences on the
device: with temporal fusion on rectangular chunks, over generated chunks, and with both, against
the oracles; outputs and the states of both layers."""
import numpy as np
import pytest

import oracle
from oracle import labelled, tfusion
from refs import parity_str, rel_err
from workloads import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4
CHUNKS = [[0, 70, 0, 8], [70, 201, 0, 5], [70, 201, 5, 8], [201, 260, 2, 8]]


def _workload(seed, T, N, F, S, chunks, kind, layers):
    wl = synth.random_small(seed, T, N, F, S, S, 4.0, chunks, kind, n_struct_layers=layers, hub=True)
    wl.params = synth.layer_params(seed, F, S, S, kind, layers, random_bias=True, n_time_layers=2)
    return wl


@pytest.mark.parametrize("kind,S,layers", [("lstm", 64, 1), ("gru", 128, 1), ("lstm", 128, 2), ("gru", 32, 2)])
def test_stacked_with_temporal_fusion(kind, S, layers):
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F = 8, 260, 40
    wl = _workload(500 + S, T, N, F, S, CHUNKS, kind, layers)
    present = synth.presence(500 + S, T, N)
    n_state = 2 if kind == "lstm" else 1
    tot = int(sum(c[1] - c[0] for c in CHUNKS))
    H0 = (0.5 * synth.stream(S, "h0-stacked-tf").standard_normal((2 * n_state * tot, S))).astype(np.float32)
    dw = DeviceWorkload(wl, n_time_layers=2, act_hidden="relu", act_out="none")
    dw.layer.set_presence(torch.from_numpy(present).cuda())
    dw.H0 = torch.from_numpy(H0).cuda()
    Y, HN = dw.forward(want_state=True)
    Y, HN = Y.cpu().numpy(), HN.cpu().numpy()
    Z = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", n_struct_layers=layers, C1=wl.C1,
                       act_hidden="relu", act_out="none").astype(np.float64)
    want, want_HN = tfusion.run_separate(np.nan_to_num(Z), present, wl.chunks, wl.params, kind, H0=H0.astype(np.float64),
                                         return_state=True, n_time_layers=2)
    m = ~np.isnan(want)
    assert m.sum() > 500 and np.isnan(Y[~m.any(axis=2)]).all()
    e_y, e_h = rel_err(Y[m], want[m]), rel_err(HN, want_HN)
    print(f"stacked {kind} S={S} layers={layers} + presence: Y " + parity_str(Y[m], want[m]) + f"; HN {e_h:.2e}", flush=True)
    assert e_y < TOL and e_h < TOL
    dw.layer.destroy()


def _random_labels(rng, T, N, n_labels, p_keep):
    lab = np.zeros((T, N), np.int64)
    lab[0] = np.sort(rng.integers(0, n_labels, N))
    for t in range(1, T):
        keep = rng.random(N) < p_keep
        lab[t] = np.where(keep, lab[t - 1], rng.integers(0, n_labels, N))
    return lab


@pytest.mark.parametrize("kind,S,layers,with_presence", [("lstm", 64, 1, False), ("gru", 128, 2, False), ("lstm", 128, 1, True),
                                                           ("gru", 64, 2, True), ("lstm", 32, 2, True)])
def test_stacked_over_generated_chunks(kind, S, layers, with_presence):
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F = 7, 170, 20
    wl = _workload(600 + S + layers, T, N, F, S, [[0, N, 0, T]], kind, layers)
    rng = np.random.default_rng(S + layers)
    lab = _random_labels(rng, T, N, 6, 0.7)
    present = synth.presence(S, T, N) if with_presence else None
    n_state = 2 if kind == "lstm" else 1
    Hc = (0.5 * rng.standard_normal((2 * n_state * T * N, S))).astype(np.float32)
    dw = DeviceWorkload(wl, n_time_layers=2, act_hidden="relu", act_out="none")
    dw.layer.set_labels(torch.from_numpy(lab.astype(np.int32).reshape(-1)).cuda())
    if with_presence:
        dw.layer.set_presence(torch.from_numpy(present).cuda())
    HN = torch.full((2 * n_state * T * N, S), float("nan"), device="cuda")
    dw.Y.fill_(float("nan"))
    dw.layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=torch.from_numpy(Hc).cuda(), HN=HN)
    torch.cuda.synchronize()
    Y, HN = dw.Y.cpu().numpy(), HN.cpu().numpy()
    want, want_HN = labelled.forward(wl.graph, lab, wl.params, wl.X, wl.C, time_kind=kind, n_struct_layers=layers, C1=wl.C1,
                                     Hc=Hc, present=present, n_time_layers=2)
    here = ~np.isnan(want).any(axis=2)
    assert np.array_equal(np.isnan(Y).any(axis=2), ~here)
    m = ~np.isnan(want_HN)
    np.testing.assert_array_equal(np.isnan(HN), ~m)
    e_y, e_h = rel_err(Y[here], want[here]), rel_err(HN[m], want_HN[m])
    print(f"stacked {kind} S={S} layers={layers} over labels{' + presence' if with_presence else ''}: Y "
          + parity_str(Y[here], want[here]) + f"; HN {e_h:.2e} ({int(m.any(axis=1).sum())} state rows)", flush=True)
    assert e_y < TOL and e_h < TOL
    dw.layer.destroy()
