"""The LSTM fed with both GCN layers' outputs side by side (Section 6, MPNN-LSTM) on the GPU
against the oracle: outputs and final states, with and without temporal fusion."""
import numpy as np
import pytest

import oracle
from oracle import tfusion
from workloads import synth
from refs import rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4
CHUNKS = [[0, 70, 0, 6], [70, 201, 0, 4], [70, 201, 4, 6], [201, 230, 1, 6]]


@pytest.mark.parametrize("S,F,gather", [(32, 20, "in_place"), (64, 48, "staged"), (128, 172, "in_place")])
def test_concat_parity(S, F, gather):
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N = 6, 230
    wl = synth.random_small(50 + S, T, N, F, S, S, 4.0, CHUNKS, "lstm", n_struct_layers=2, hub=True, input_concat=True)
    wl.params["rnn.weight_ih"][:, :S] *= 1.5          # unequal halves: swapped halves must fail
    dw = DeviceWorkload(wl, gather_mode=gather)
    Y, HN = dw.forward(want_state=True)
    want, want_HN = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="lstm", n_struct_layers=2,
                                   C1=wl.C1, H0=wl.H0, return_state=True, input_concat=True)
    m = ~np.isnan(want)
    e_y, e_h = rel_err(Y.cpu().numpy()[m], want[m].astype(np.float64)), rel_err(HN.cpu().numpy(), want_HN.astype(np.float64))
    print(f"concat S={S} F={F} {gather}: rel_err Y {e_y:.3e} HN {e_h:.3e}", flush=True)
    assert e_y < TOL and e_h < TOL
    assert np.isnan(Y.cpu().numpy()[~m]).all()
    # the first half of the input matters: without it the result is another one
    other = oracle.forward(wl.graph, wl.chunks, {**wl.params, "rnn.weight_ih": np.ascontiguousarray(wl.params["rnn.weight_ih"][:, S:])},
                           wl.X, wl.C, time_kind="lstm", n_struct_layers=2, C1=wl.C1, H0=wl.H0)
    assert rel_err(other[m].astype(np.float64), want[m].astype(np.float64)) > 1e-2
    dw.layer.destroy()


@pytest.mark.parametrize("S", [32, 128])
def test_concat_with_temporal_fusion(S):
    """Lanes instead of padded windows: a slot reads the first layer's row of its own
    (snapshot, vertex).  The oracle runs every present vertex's own sequence on [Z1, Z2]."""
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F = 6, 230, 24
    wl = synth.random_small(80 + S, T, N, F, S, S, 4.0, CHUNKS, "lstm", n_struct_layers=2, input_concat=True)
    present = synth.presence(80 + S, T, N)
    dw = DeviceWorkload(wl)
    dw.layer.set_presence(torch.from_numpy(present).cuda())
    Y, HN = dw.forward(want_state=True)
    Z2 = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", n_struct_layers=2, C1=wl.C1,
                        act_hidden="relu", act_out="none").astype(np.float64)
    Z1 = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", n_struct_layers=1,
                        act_out="relu").astype(np.float64)
    Zc = np.nan_to_num(np.concatenate([Z1, Z2], axis=2))
    want, want_HN = tfusion.run_separate(Zc, present, wl.chunks, wl.params, "lstm", H0=wl.H0.astype(np.float64),
                                         return_state=True)
    m = ~np.isnan(want)
    assert m.sum() > 500
    e_y, e_h = rel_err(Y.cpu().numpy()[m], want[m]), rel_err(HN.cpu().numpy(), want_HN)
    print(f"concat + temporal fusion S={S}: rel_err Y {e_y:.3e} HN {e_h:.3e}", flush=True)
    assert e_y < TOL and e_h < TOL
    dw.layer.destroy()


def test_concat_refusals():
    import torch
    from paper_2309_03523_amd.binding import DgcError, DgcLayer
    wl = synth.random_small(3, 2, 40, 8, 32, 32, 3.0, [[0, 40, 0, 2]], "lstm", n_struct_layers=2)
    rp = [torch.from_numpy(s.rowptr).cuda() for s in wl.graph.snaps]
    ci = [torch.from_numpy(s.col).cuda() for s in wl.graph.snaps]

    def create(**kw):
        args = dict(F=8, S=32, H=32, time_kind="lstm", n_struct_layers=2, lstm_input_concat=True)
        args.update(kw)
        DgcLayer(rp, ci, 40, wl.chunks, **args).destroy()

    create()
    for kw, code in [(dict(time_kind="gru"), 1), (dict(n_struct_layers=1), 1), (dict(S=96, H=96), 4),
                     (dict(S=64, H=32), 4), (dict(dense_kernel="tile"), 4)]:
        with pytest.raises(DgcError) as ei:
            create(**kw)
        assert ei.value.code == code, (kw, ei.value)
    layer = DgcLayer(rp, ci, 40, wl.chunks, F=8, S=32, H=32, time_kind="lstm", n_struct_layers=2, lstm_input_concat=True)
    with pytest.raises(DgcError):          # the input weights are [4H, 2S] now
        layer.set_param("rnn.weight_ih", np.zeros((128, 32), np.float32))
    layer.set_param("rnn.weight_ih", np.zeros((128, 64), np.float32))
    layer.destroy()


@pytest.mark.parametrize("seed", range(6))
def test_concat_random_shapes(seed):
    """Tiny and ragged shapes: one vertex, one snapshot, windows of one snapshot, F below 8."""
    from paper_2309_03523_amd.runner import DeviceWorkload
    rng = np.random.default_rng(9000 + seed)
    N = int(rng.choice([1, 2, 31, 33, 65]))
    T = int(rng.integers(1, 6))
    S = int(rng.choice([32, 64, 128]))
    F = int(rng.choice([1, 7, 32, 50]))
    cut = int(rng.integers(0, N + 1))
    chunks = [c for c in ([0, cut, 0, T], [cut, N, 0, max(1, T // 2)], [cut, N, max(1, T // 2), T]) if c[0] < c[1] and c[2] < c[3]]
    wl = synth.random_small(9100 + seed, T, N, F, S, S, 3.0, chunks, "lstm", n_struct_layers=2, input_concat=True)
    dw = DeviceWorkload(wl, gather_mode=str(rng.choice(["in_place", "staged"])))
    Y, HN = dw.forward(want_state=True)
    want, want_HN = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="lstm", n_struct_layers=2,
                                   C1=wl.C1, H0=wl.H0, return_state=True, input_concat=True)
    m = ~np.isnan(want)
    e_y = rel_err(Y.cpu().numpy()[m], want[m].astype(np.float64))
    e_h = rel_err(HN.cpu().numpy(), want_HN.astype(np.float64))
    print(f"seed {seed}: N={N} T={T} F={F} S={S} chunks={len(chunks)}: rel_err Y {e_y:.3e} HN {e_h:.3e}", flush=True)
    assert e_y < TOL and e_h < TOL
    assert np.isnan(Y.cpu().numpy()[~m]).all()
    dw.layer.destroy()
