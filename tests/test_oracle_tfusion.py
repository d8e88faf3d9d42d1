"""Pins of the temporal-fusion oracle (CPU only): the paper's own drawn example, brute-force
properties of the packing on random presence patterns, the per-sequence recurrence against
torch.nn.GRU / LSTM on the compressed sequences, and the paper's claim that concatenated
sequences with the mask give the outputs of the separate sequences."""
import os

import numpy as np
import pytest
import torch

from oracle import tfusion
from workloads import synth

HERE = os.path.dirname(os.path.abspath(__file__))


def _golden():
    d = {}
    for line in open(os.path.join(HERE, "golden", "temporal_fusion_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        d[k] = np.array([int(x) for x in v])
    return d


def test_paper_example():
    g = _golden()
    T, N = int(g["T"][0]), int(g["N"][0])
    present = g["present"].reshape(T, N).astype(np.uint8)
    p = tfusion.pack(present, [[0, N, 0, T]])
    np.testing.assert_array_equal(p["lane_ptr"], g["lane_ptr"])
    np.testing.assert_array_equal(p["slot_row"], g["slot_row"].reshape(T, -1))
    np.testing.assert_array_equal(p["slot_reset"], g["slot_reset"].reshape(T, -1))


CHUNKS = [[0, 17, 0, 8], [17, 40, 0, 5], [17, 40, 5, 8], [40, 61, 2, 8]]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_packing_properties(seed):
    T, N = 8, 61
    present = synth.presence(seed, T, N)
    p = tfusion.pack(present, CHUNKS)
    rows = p["slot_row"][p["slot_row"] >= 0]
    want = sorted(t * N + i for v_lo, v_hi, t_lo, t_hi in CHUNKS for t in range(t_lo, t_hi)
                  for i in range(v_lo, v_hi) if present[t, i])
    assert sorted(rows.tolist()) == want                      # every present covered row exactly once
    for k, (v_lo, v_hi, t_lo, t_hi) in enumerate(CHUNKS):
        L = t_hi - t_lo
        n_seq = sum(1 for i in range(v_lo, v_hi) if present[t_lo:t_hi, i].any())
        total = int(present[t_lo:t_hi, v_lo:v_hi].sum())
        lanes = range(int(p["lane_ptr"][k]), int(p["lane_ptr"][k + 1]))
        assert -(-total // L) <= len(lanes) <= n_seq        # between the volume bound and no fusion at all
        for lane in lanes:
            col, rst = p["slot_row"][:, lane], p["slot_reset"][:, lane]
            assert (col[L:] == -1).all()                       # nothing beyond the chunk's window
            used = col[col >= 0]
            assert len(used) == (col[:len(used)] >= 0).sum()   # occupied slots are a prefix
            prev_v = -1
            for s, r in enumerate(used):
                t, i = divmod(int(r), N)
                assert v_lo <= i < v_hi and t_lo <= t < t_hi
                assert rst[s] == (i != prev_v)                 # reset exactly where a new sequence starts
                if i == prev_v:
                    assert t > prev_t                          # a sequence keeps its order
                prev_v, prev_t = i, t
            assert not rst[len(used):].any()
    # first-fit decreasing never leaves two lanes of a chunk that would fit into one
    for k in range(len(CHUNKS)):
        L = CHUNKS[k][3] - CHUNKS[k][2]
        fill = [(p["slot_row"][:, lane] >= 0).sum() for lane in range(int(p["lane_ptr"][k]), int(p["lane_ptr"][k + 1]))]
        assert sum(1 for f in fill if 2 * f <= L) <= 1


def _params(kind, S=5, H=4, seed=3):
    return synth.layer_params(seed, S, S, H, kind, random_bias=True)


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_separate_run_equals_library_rnn(kind):
    T, N, S, H = 8, 61, 5, 4
    present = synth.presence(4, T, N)
    P = _params(kind, S, H)
    Z = np.random.default_rng(0).standard_normal((T, N, S))
    Y = tfusion.run_separate(Z, present, CHUNKS, P, kind)
    rnn = (torch.nn.GRU if kind == "gru" else torch.nn.LSTM)(S, H).double()
    with torch.no_grad():
        rnn.weight_ih_l0.copy_(torch.from_numpy(P["rnn.weight_ih"]))
        rnn.weight_hh_l0.copy_(torch.from_numpy(P["rnn.weight_hh"]))
        rnn.bias_ih_l0.copy_(torch.from_numpy(P["rnn.bias_ih"]))
        rnn.bias_hh_l0.copy_(torch.from_numpy(P["rnn.bias_hh"]))
        checked = 0
        for v_lo, v_hi, t_lo, t_hi in CHUNKS:
            for i in range(v_lo, v_hi):
                ts = [t for t in range(t_lo, t_hi) if present[t, i]]
                if not ts:
                    continue
                out, _ = rnn(torch.from_numpy(Z[ts, i])[:, None, :])
                np.testing.assert_allclose(Y[ts, i], out[:, 0].numpy(), atol=1e-12)
                checked += 1
    assert checked > 50
    cov = np.zeros((T, N), bool)
    for v_lo, v_hi, t_lo, t_hi in CHUNKS:
        cov[t_lo:t_hi, v_lo:v_hi] = True
    assert np.isnan(Y[~(cov & present.astype(bool))]).all()


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_concatenated_with_mask_equals_separate(kind):
    T, N, S, H = 8, 61, 5, 4
    present = synth.presence(5, T, N)
    P = _params(kind, S, H)
    Z = np.random.default_rng(1).standard_normal((T, N, S))
    sep = tfusion.run_separate(Z, present, CHUNKS, P, kind)
    packing = tfusion.pack(present, CHUNKS)
    fused = tfusion.run_lanes(Z, packing, P, kind)
    np.testing.assert_allclose(fused, sep, atol=1e-13, equal_nan=True)
    # without the mask the state of one sequence leaks into the next one
    leaky = tfusion.run_lanes(Z, dict(packing, slot_reset=np.zeros_like(packing["slot_reset"])), P, kind)
    m = ~np.isnan(sep)
    assert np.abs(leaky[m] - sep[m]).max() > 1e-2


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_chained_windows_with_state_equal_one_long_window(kind):
    # two windows over the same vertices, the second started from the first one's final states:
    # every vertex then sees one sequence over both windows, whatever its gaps
    T, N, S, H = 8, 40, 5, 4
    present = synth.presence(6, T, N, 0.0, 1.0)
    present[:, 3] = 0                        # absent throughout
    present[:4, 5] = 0                       # absent in the first window only
    present[4:, 7] = 0                       # absent in the second window only
    P = _params(kind, S, H)
    Z = np.random.default_rng(2).standard_normal((T, N, S))
    whole = [[0, N, 0, T]]
    first, second = [[0, N, 0, 4]], [[0, N, 4, T]]
    n_state = 2 if kind == "lstm" else 1
    H0 = 0.3 * np.random.default_rng(3).standard_normal((n_state * N, H))
    Yw, HNw = tfusion.run_separate(Z, present, whole, P, kind, H0=H0, return_state=True)
    Y1, HN1 = tfusion.run_separate(Z, present, first, P, kind, H0=H0, return_state=True)
    Y2, HN2 = tfusion.run_separate(Z, present, second, P, kind, H0=HN1, return_state=True)
    np.testing.assert_allclose(np.where(np.isnan(Y1), Y2, Y1), Yw, atol=1e-13, equal_nan=True)
    np.testing.assert_allclose(HN2, HNw, atol=1e-13)
    np.testing.assert_array_equal(HNw[3], H0[3])                     # never present: state untouched
    np.testing.assert_array_equal(HN1[5], H0[5])                     # absent in the first window: carried through
    np.testing.assert_array_equal(HN2[7], HN1[7])
    assert np.abs(HNw[0] - H0[0]).max() > 1e-3
    # the initial state matters, and the library recurrence started from it agrees
    Y0 = tfusion.run_separate(Z, present, whole, P, kind)
    m = ~np.isnan(Yw)
    assert np.abs(Y0[m] - Yw[m]).max() > 1e-3
    rnn = (torch.nn.GRU if kind == "gru" else torch.nn.LSTM)(S, H).double()
    with torch.no_grad():
        rnn.weight_ih_l0.copy_(torch.from_numpy(P["rnn.weight_ih"]))
        rnn.weight_hh_l0.copy_(torch.from_numpy(P["rnn.weight_hh"]))
        rnn.bias_ih_l0.copy_(torch.from_numpy(P["rnn.bias_ih"]))
        rnn.bias_hh_l0.copy_(torch.from_numpy(P["rnn.bias_hh"]))
        for i in (0, 5, 7, 11):
            ts = [t for t in range(T) if present[t, i]]
            if not ts:
                continue
            h0 = torch.from_numpy(H0[i])[None, None]
            st = h0 if kind == "gru" else (h0, torch.from_numpy(H0[N + i])[None, None])
            out, fin = rnn(torch.from_numpy(Z[ts, i])[:, None, :], st)
            np.testing.assert_allclose(Yw[ts, i], out[:, 0].numpy(), atol=1e-12)
            np.testing.assert_allclose(HNw[i], (fin if kind == "gru" else fin[0])[0, 0].numpy(), atol=1e-12)
            if kind == "lstm":
                np.testing.assert_allclose(HNw[N + i], fin[1][0, 0].numpy(), atol=1e-12)


@pytest.mark.parametrize("kind", ["gru", "lstm"])
def test_lanes_with_state_equal_separate(kind):
    T, N, S, H = 8, 61, 5, 4
    present = synth.presence(7, T, N, 0.0, 1.0)
    P = _params(kind, S, H)
    Z = np.random.default_rng(4).standard_normal((T, N, S))
    V = sum(c[1] - c[0] for c in CHUNKS)
    H0 = 0.3 * np.random.default_rng(5).standard_normal(((2 if kind == "lstm" else 1) * V, H))
    Ys, HNs = tfusion.run_separate(Z, present, CHUNKS, P, kind, H0=H0, return_state=True)
    Yl, HNl = tfusion.run_lanes(Z, tfusion.pack(present, CHUNKS), P, kind, chunks=CHUNKS, H0=H0, return_state=True)
    np.testing.assert_allclose(Yl, Ys, atol=1e-13, equal_nan=True)
    np.testing.assert_allclose(HNl, HNs, atol=1e-13)
    # without H0 the lane run with chunks still returns the final states of zero-started sequences
    Y0, HN0 = tfusion.run_lanes(Z, tfusion.pack(present, CHUNKS), P, kind, chunks=CHUNKS, return_state=True)
    Yz, HNz = tfusion.run_separate(Z, present, CHUNKS, P, kind, return_state=True)
    np.testing.assert_allclose(HN0, HNz, atol=1e-13)
