"""The stacked time encoder (two recurrent layers, Section 6's MPNN-LSTM) on the device against the
oracle: outputs and the final states of both layers, with initial states, with a reset mask, after
one and two GCN layers, with the LSTM reading both GCN outputs."""
import numpy as np
import pytest

import oracle
from refs import parity_str, rel_err
from workloads import synth

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _run(wl, H0, mask=None, **okw):
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    dw = DeviceWorkload(wl, n_time_layers=2, act_hidden="relu", act_out="none")
    dw.H0 = None if H0 is None else torch.from_numpy(H0).cuda()
    Y, HN = dw.forward(reset_mask=mask, want_state=True)
    want_Y, want_HN = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind=wl.time_kind,
                                     n_struct_layers=wl.n_struct_layers, C1=wl.C1, H0=H0, reset_mask=mask,
                                     return_state=True, n_time_layers=2, act_hidden="relu", act_out="none", **okw)
    got = Y.cpu().numpy()
    cov = ~np.isnan(want_Y)
    assert np.array_equal(np.isnan(got), ~cov)
    e_y, e_h = rel_err(got[cov], want_Y[cov]), rel_err(HN.cpu().numpy(), want_HN)
    dw.layer.destroy()
    return e_y, e_h, got[cov], want_Y[cov]


@pytest.mark.parametrize("kind", ["lstm", "gru"])
@pytest.mark.parametrize("F,S,layers", [(20, 32, 1), (77, 64, 2), (128, 128, 1), (172, 128, 2)])
def test_stacked_time_encoder_matches_oracle(kind, F, S, layers):
    N, T = 203, 6
    chunks = [[0, 70, 0, 6], [70, 131, 0, 3], [70, 131, 3, 6], [131, 203, 1, 5]]
    wl = synth.random_small(900 + F, T, N, F, S, S, 5.0, chunks, kind, layers, hub=True)
    wl.params = synth.layer_params(900 + F, F, S, S, kind, layers, random_bias=True, n_time_layers=2)
    tot = int(sum(c[1] - c[0] for c in chunks))
    n_state = 2 if kind == "lstm" else 1
    H0 = (0.5 * synth.stream(F, "h0-stacked").standard_normal((2 * n_state * tot, S))).astype(np.float32)
    e_y, e_h, got, want = _run(wl, H0)
    print(f"{kind} F={F} S={S} layers={layers}: Y " + parity_str(got, want) + f"; HN {e_h:.2e}", flush=True)
    assert e_y < TOL and e_h < TOL
    mask = (synth.stream(F, "mask").random((T, N)) < 0.2).astype(np.uint8)
    e_y, e_h, _, _ = _run(wl, None, mask)
    assert e_y < TOL and e_h < TOL


def test_stacked_lstm_on_both_gcn_outputs():
    """The paper's MPNN-LSTM as Section 6 describes it: two GCN layers, the LSTM input their outputs
    side by side, two LSTM layers."""
    N, T, F, S = 150, 5, 44, 64
    chunks = [[0, 80, 0, 5], [80, 150, 0, 5]]
    wl = synth.random_small(77, T, N, F, S, S, 4.0, chunks, "lstm", 2, hub=True, input_concat=True)
    wl.params = synth.layer_params(77, F, S, S, "lstm", 2, random_bias=True, input_concat=True, n_time_layers=2)
    e_y, e_h, got, want = _run(wl, None, input_concat=True)
    print("two GCN layers, concatenated input, two LSTM layers: " + parity_str(got, want), flush=True)
    assert e_y < TOL and e_h < TOL


def test_stacked_argument_errors():
    from paper_2309_03523_amd.binding import DgcError
    from paper_2309_03523_amd.runner import DeviceWorkload
    wl = synth.random_small(5, 2, 40, 8, 96, 96, 3.0, [[0, 40, 0, 2]], "lstm")       # S = 96: tile kernel only
    wl.params = synth.layer_params(5, 8, 96, 96, "lstm", 1, n_time_layers=2)
    with pytest.raises(DgcError) as ei:
        DeviceWorkload(wl, n_time_layers=2)
    assert ei.value.code == 4
    wl = synth.random_small(6, 2, 40, 8, 32, 32, 3.0, [[0, 40, 0, 2]], "none")
    with pytest.raises(DgcError) as ei:
        DeviceWorkload(wl, n_time_layers=2)
    assert ei.value.code == 1
    wl = synth.random_small(7, 2, 40, 8, 32, 32, 3.0, [[0, 40, 0, 2]], "gru")
    wl.params = synth.layer_params(7, 8, 32, 32, "gru", 1, n_time_layers=2)
    with pytest.raises(DgcError) as ei:          # the workgroup-tile kernel has no stacked variant
        DeviceWorkload(wl, n_time_layers=2, dense_kernel="tile")
    assert ei.value.code == 4
