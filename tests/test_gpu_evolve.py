"""Parity of the EvolveGCN-O path (weight evolution, forward, MSE loss, parameter gradients)
against the CPU oracle, through the C ABI."""
import numpy as np
import pytest

import oracle
from workloads import synth
from refs import rel_err

pytestmark = pytest.mark.gpu

TOL = 1e-4


def _workload(seed, T, N, F, chunks, deg=4.0):
    wl = synth.random_small(seed, T, N, F, F, F, deg, chunks, "none", hub=True)
    wl.params = synth.evolve_params(seed, F, F, random_bias=True)
    return wl


def _dw(wl, **kw):
    from paper_2309_03523_amd.runner import DeviceWorkload
    return DeviceWorkload(wl, struct_kind="evolve_gcn_o", act_out="relu", **kw)


@pytest.mark.parametrize("F", [32, 64, 128, 256])
@pytest.mark.parametrize("dense", ["auto", "tile"])
def test_evolve_forward_and_gradients(F, dense):
    import torch
    T, N = 6, 150
    chunks = [[0, 40, 0, 6], [40, 97, 0, 3], [40, 97, 3, 6], [97, 150, 0, 6]]
    wl = _workload(300 + F, T, N, F, chunks)
    target = synth.stream(F, "target").standard_normal((T, N, F)).astype(np.float32)
    dw = _dw(wl, dense_kernel=dense, long_nnz=24, part_nnz=8)
    Y = dw.forward()
    want = oracle.evolve(wl.graph, wl.chunks, wl.params, wl.X, wl.C, target, want_grads=True)
    got = Y.cpu().numpy()
    assert rel_err(got, want["Y"]) < TOL
    tgt = torch.from_numpy(target).cuda()
    loss = torch.zeros(1, device="cuda")
    dw.layer.backward(Y, target=tgt, loss_out=loss)
    torch.cuda.synchronize()
    assert abs(loss.item() - want["loss"]) < 1e-5 * want["loss"]
    for name in oracle.EVOLVE_PARAMS:
        g = dw.layer.get_param(name + ".grad", wl.params[name].shape)
        e = rel_err(g, want["grads"][name])
        assert e < TOL, (name, e)
    # explicit upstream gradient: dY = 2 (Y - target) / count reproduces the same gradients
    dY = (2.0 * (Y - tgt) / float(wl.rows * F)).contiguous()
    dw.layer.backward(Y, dY=dY)
    torch.cuda.synchronize()
    for name in oracle.EVOLVE_PARAMS:
        g = dw.layer.get_param(name + ".grad", wl.params[name].shape)
        assert rel_err(g, want["grads"][name]) < TOL, name
    dw.layer.destroy()


@pytest.mark.parametrize("F,dense,pitch", [(32, "auto", 32), (64, "tile", 68), (128, "auto", 128), (256, "auto", 260)])
def test_evolve_input_gradient(F, dense, pitch):
    """dL/dX: through the rows of a row's own chunk only (the cache is a constant); rows outside
    every chunk and the pitch padding stay untouched; the saved rows are used up by it."""
    import torch
    from paper_2309_03523_amd.binding import DgcError
    T, N = 6, 150
    chunks = [[0, 40, 0, 6], [40, 97, 0, 3], [40, 97, 3, 6], [97, 150, 1, 5]]
    wl = _workload(500 + F, T, N, F, chunks)
    target = synth.stream(F, "target").standard_normal((T, N, F)).astype(np.float32)
    dw = _dw(wl, dense_kernel=dense, long_nnz=24, part_nnz=8)
    Y = dw.forward()
    want = oracle.evolve(wl.graph, wl.chunks, wl.params, wl.X, wl.C, target, want_grads=True, want_dx=True)
    tgt = torch.from_numpy(target).cuda()
    buf = torch.full((T, N, pitch), float("nan"), device="cuda")
    dX = buf[:, :, :F]
    dw.layer.backward(Y, target=tgt, dX=dX)
    torch.cuda.synchronize()
    got = dX.cpu().numpy()
    covered = ~np.isnan(want["Y"]).any(axis=2)
    assert np.isnan(got[~covered]).all() and not np.isnan(got[covered]).any()
    assert np.isnan(buf[:, :, F:].cpu().numpy()).all()
    e = rel_err(got[covered], want["dX"][covered])
    print(f"F={F} {dense}: dX rel_err {e:.3e}, max |dX| {np.abs(want['dX']).max():.3e}", flush=True)
    assert e < TOL and np.abs(want["dX"][covered]).max() > 0
    for name in oracle.EVOLVE_PARAMS:      # the parameter gradients of the same call are unaffected
        g = dw.layer.get_param(name + ".grad", wl.params[name].shape)
        assert rel_err(g, want["grads"][name]) < TOL, name
    with pytest.raises(DgcError, match="forward again"):
        dw.layer.backward(Y, target=tgt)
    dw.forward()
    dw.layer.backward(Y, target=tgt)         # fine again after a forward
    torch.cuda.synchronize()
    dw.layer.destroy()


@pytest.mark.parametrize("F", [64, 256])
def test_evolve_long_recurrence(F):
    """64 snapshots: the weight recurrence and its back-propagation run the full length of the
    workload the metric is quoted on; chunk windows of 16 snapshots."""
    import torch
    T, N = 64, 96
    chunks = [[v0, v1, t0, t0 + 16] for (v0, v1) in ((0, 50), (50, 96)) for t0 in range(0, 64, 16)]
    wl = _workload(900 + F, T, N, F, chunks)
    target = synth.stream(F, "target64").standard_normal((T, N, F)).astype(np.float32)
    dw = _dw(wl)
    Y = dw.forward()
    want = oracle.evolve(wl.graph, wl.chunks, wl.params, wl.X, wl.C, target, want_grads=True)
    got = Y.cpu().numpy()
    for t in (0, 31, 63):
        e = rel_err(got[t], want["Y"][t])
        print(f"F={F} t={t} Y rel_err {e:.3e}", flush=True)
        assert e < TOL, (t, e)
    loss = torch.zeros(1, device="cuda")
    dw.layer.backward(Y, target=torch.from_numpy(target).cuda(), loss_out=loss)
    torch.cuda.synchronize()
    assert abs(loss.item() - want["loss"]) < 1e-5 * want["loss"]
    for name in oracle.EVOLVE_PARAMS:
        g = dw.layer.get_param(name + ".grad", wl.params[name].shape)
        e = rel_err(g, want["grads"][name])
        print(f"F={F} grad {name} rel_err {e:.3e}", flush=True)
        assert e < TOL, (name, e)
    dw.layer.destroy()


def _sampled_problem(wl, picks):
    from workloads import sampling
    return sampling.one_hop_problem(wl.graph, picks, wl.X, wl.C, wl.F)


@pytest.mark.timeout(600)
def test_config4_eighth_size_sampled():
    """Config 4 at an eighth of its vertex count, as bench.py's config4s workload launches it (64
    snapshots, F = S = 256, 32 chunks in 4 windows): outputs of a seeded sample of vertices of every
    chunk and of the largest hubs against the oracle, which evolves the same 64 weight matrices."""
    wl, _ = synth.config4(seed=0, scale=0.125)
    dw = _dw(wl)
    got = dw.forward().cpu().numpy()
    assert not np.isnan(got).any()              # the chunks cover every (vertex, snapshot)
    rng = synth.stream(0, "parity-sample")
    hubs = set(np.argsort(np.diff(wl.graph.snaps[0].rowptr))[-2:].tolist())
    picks = []
    for ch in wl.chunks.tolist():
        pick = set((rng.choice(ch[1] - ch[0], size=3, replace=False) + ch[0]).tolist()) | {ch[0], ch[1] - 1}
        pick |= {h for h in hubs if ch[0] <= h < ch[1]}
        picks += [(v, ch) for v in sorted(pick)]
    g1, c1, X1, C1 = _sampled_problem(wl, picks)
    want = oracle.evolve(g1, c1, wl.params, X1, C1)["Y"]
    gs = np.stack([got[ch[2]:ch[3], v] for v, ch in picks])
    ws = np.stack([want[ch[2]:ch[3], i] for i, (_, ch) in enumerate(picks)])
    assert not np.isnan(ws).any()
    e = rel_err(gs, ws)
    print(f"config4@0.125: {len(picks)} sampled vertices ({g1.N} local vertices), Y rel_err {e:.3e}", flush=True)
    assert len(picks) >= 32 * 4 and e < TOL
    dw.layer.destroy()


def test_evolve_argument_errors():
    import torch
    from paper_2309_03523_amd.binding import DgcError
    wl = _workload(5, 2, 40, 32, [[0, 40, 0, 2]])
    dw = _dw(wl)
    with pytest.raises(DgcError) as ei:
        dw.layer.backward(dw.Y, target=dw.Y)
    assert ei.value.code == 7
    Y = dw.forward()
    with pytest.raises(DgcError) as ei:
        dw.layer.backward(Y)
    assert ei.value.code == 1
    with pytest.raises(DgcError) as ei:
        dw.layer.backward(Y, target=Y, dY=Y)
    assert ei.value.code == 1
    with pytest.raises(DgcError) as ei:      # dX with a pitch that is not a multiple of 4 floats
        dw.layer.backward(Y, target=Y, dX=torch.zeros(dw.X.shape[0], dw.X.shape[1], 34, device="cuda")[:, :, :32])
    assert ei.value.code == 1
    with pytest.raises(DgcError) as ei:
        dw.layer.set_param("evolve.U_z.grad", np.zeros((32, 32), np.float32))
    assert ei.value.code == 1
    dw.layer.destroy()
    from paper_2309_03523_amd.runner import DeviceWorkload
    with pytest.raises(DgcError) as ei:   # F != S
        wl2 = synth.random_small(6, 2, 40, 64, 32, 32, 3.0, [[0, 40, 0, 2]], "none")
        DeviceWorkload(wl2, struct_kind="evolve_gcn_o", act_out="relu")
    assert ei.value.code == 1


@pytest.mark.parametrize("seed", range(8))
def test_evolve_random_shapes(seed):
    """Tiny vertex counts, one snapshot, gaps in the coverage: forward, loss, parameter and input gradients."""
    import torch
    rng = np.random.default_rng(7000 + seed)
    N = int(rng.choice([1, 2, 3, 33, 70]))
    T = int(rng.integers(1, 6))
    F = int(rng.choice([32, 64]))
    cuts = sorted(set([0, N] + rng.integers(0, N + 1, size=rng.integers(0, 3)).tolist()))
    chunks = []
    for a, b in zip(cuts, cuts[1:]):
        tcuts = sorted(set([0, T] + rng.integers(0, T + 1, size=rng.integers(0, 3)).tolist()))
        chunks += [[a, b, t0, t1] for t0, t1 in zip(tcuts, tcuts[1:]) if rng.random() < 0.85]
    if not chunks:
        chunks = [[0, N, 0, T]]
    wl = _workload(8000 + seed, T, N, F, chunks, deg=float(rng.choice([0.0, 2.0, 5.0])))
    target = synth.stream(seed, "target").standard_normal((T, N, F)).astype(np.float32)
    dw = _dw(wl, dense_kernel=str(rng.choice(["auto", "tile"])))
    Y = dw.forward()
    want = oracle.evolve(wl.graph, wl.chunks, wl.params, wl.X, wl.C, target, want_grads=True, want_dx=True)
    covered = ~np.isnan(want["Y"]).any(axis=2)
    got = Y.cpu().numpy()
    assert rel_err(got[covered], want["Y"][covered]) < TOL and np.isnan(got[~covered]).all()
    loss = torch.zeros(1, device="cuda")
    dX = torch.full((T, N, F), float("nan"), device="cuda")
    dw.layer.backward(Y, target=torch.from_numpy(target).cuda(), loss_out=loss, dX=dX)
    torch.cuda.synchronize()
    assert abs(loss.item() - want["loss"]) < 1e-5 * want["loss"]
    gx = dX.cpu().numpy()
    e = rel_err(gx[covered], want["dX"][covered])
    print(f"seed {seed}: N={N} T={T} F={F} chunks={len(chunks)} rows={int(covered.sum())}: dX {e:.2e}", flush=True)
    assert e < TOL and np.isnan(gx[~covered]).all()
    for name in oracle.EVOLVE_PARAMS:
        g = dw.layer.get_param(name + ".grad", wl.params[name].shape)
        assert rel_err(g, want["grads"][name]) < TOL, name
    dw.layer.destroy()
