"""Seeded random small shapes through the whole layer against the oracle: tiny vertex counts, one
snapshot, one-vertex chunks, gaps in the coverage, odd feature counts, both dense kernels, both
gather modes, one or two structure layers, with and without a reset mask."""
import numpy as np
import pytest

import oracle
from workloads import synth
from refs import rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _random_chunks(rng, N, T):
    """Random disjoint rectangles: a random partition of the vertex axis, each range cut into random
    windows, each piece kept with probability 0.8 (so there are gaps)."""
    cuts = sorted(set([0, N] + rng.integers(0, N + 1, size=rng.integers(0, 4)).tolist()))
    chunks = []
    for a, b in zip(cuts, cuts[1:]):
        tcuts = sorted(set([0, T] + rng.integers(0, T + 1, size=rng.integers(0, 3)).tolist()))
        for t0, t1 in zip(tcuts, tcuts[1:]):
            if rng.random() < 0.8:
                chunks.append([a, b, t0, t1])
    if not chunks:
        chunks = [[0, N, 0, T]]
    order = rng.permutation(len(chunks))
    return [chunks[k] for k in order]


@pytest.mark.parametrize("seed", range(24))
def test_random_shape(seed):
    from paper_2309_03523_amd.runner import DeviceWorkload
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.choice([1, 2, 3, 7, 31, 32, 33, 64, 65, 100, 129]))
    T = int(rng.integers(1, 6))
    F = int(rng.choice([1, 2, 3, 5, 8, 17, 32, 33, 100]))
    S = int(rng.choice([32, 64, 96]))
    H = int(rng.choice([32, 64]))
    kind = str(rng.choice(["gru", "lstm", "none"]))
    layers = int(rng.choice([1, 1, 2]))
    mode = str(rng.choice(["in_place", "staged"]))
    dense = str(rng.choice(["auto", "tile"]))
    chunks = _random_chunks(rng, N, T)
    wl = synth.random_small(2000 + seed, T, N, F, S, H, float(rng.choice([0.0, 1.5, 6.0])), chunks, kind,
                            n_struct_layers=layers, hub=bool(rng.integers(0, 2)))
    dw = DeviceWorkload(wl, gather_mode=mode, dense_kernel=dense, act_hidden="relu", act_out="none",
                        rows_per_group=int(rng.choice([0, 1, 5, 32])), long_nnz=int(rng.choice([0, 4, 40])),
                        part_nnz=int(rng.choice([0, 3, 16])), validate_level=1)
    mask = None
    if kind != "none" and rng.random() < 0.5:
        mask = (rng.random((T, N)) < 0.3).astype(np.uint8)
    Y, HN = dw.forward(reset_mask=mask, want_state=True)
    want_Y, want_HN = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind=kind,
                                     n_struct_layers=layers, C1=wl.C1, H0=wl.H0, return_state=True,
                                     reset_mask=mask, act_hidden="relu", act_out="none")
    got = Y.cpu().numpy()
    covered = ~np.isnan(want_Y)
    print(f"seed {seed}: N={N} T={T} F={F} S={S} H={H} {kind} layers={layers} {mode} {dense} chunks={len(chunks)} "
          f"covered={int(covered.any(axis=2).sum())} mask={mask is not None}", flush=True)
    assert np.array_equal(np.isnan(got), ~covered)
    if covered.any():
        assert rel_err(got[covered], want_Y[covered]) < TOL
    if want_HN is not None:
        assert rel_err(HN.cpu().numpy(), want_HN) < TOL
    dw.layer.destroy()
