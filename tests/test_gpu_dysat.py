"""Parity of the graph-attention + temporal self-attention layer (bf16) against the CPU oracle,
through the C ABI.  Tolerance: 2e-2 on max |g - o| / max(|o|, RMS(o)): the output Y and the
stored gradients (dU, dQ, dK, dV, dz) are bf16, each rounding is up to 2^-9 relative to the rounded
value, and what reaches an output element through the dense products is an absolute error of that
order times the RMS, whatever the element's own size."""
import numpy as np
import pytest

from oracle import dysat
from workloads import synth
from refs import parity_str, rel_err

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _covered(wl):
    cov = np.zeros((wl.graph.T, wl.graph.N), bool)
    for v_lo, v_hi, t_lo, t_hi in wl.chunks.tolist():
        cov[t_lo:t_hi, v_lo:v_hi] = True
    return cov


CASES = {
    "ragged": dict(T=7, N=203, deg=5.0, chunks=[[0, 61, 0, 7], [61, 130, 0, 3], [61, 130, 3, 7], [130, 203, 1, 6]]),
    "full16": dict(T=16, N=97, deg=4.0, chunks=[[0, 33, 0, 16], [33, 97, 0, 16]]),
    "single": dict(T=3, N=40, deg=3.0, chunks=[[5, 6, 0, 3], [6, 40, 1, 2]]),
    # rows longer than 24 non-zeros (the hub, and more at degree 9) are split into parts of 8
    "split": dict(T=6, N=150, deg=9.0, chunks=[[0, 70, 0, 6], [70, 150, 0, 4]], kw=dict(long_nnz=24, part_nnz=8)),
    # windows longer than 16 snapshots: one vertex per 32-row tile
    "wide32": dict(T=32, N=67, deg=4.0, chunks=[[0, 33, 0, 32], [33, 67, 0, 32]]),
    "wide17": dict(T=17, N=35, deg=3.0, chunks=[[0, 35, 0, 17]]),
    "wide_mixed": dict(T=24, N=90, deg=5.0, chunks=[[0, 40, 0, 24], [40, 90, 0, 9], [40, 90, 9, 24]]),
}


@pytest.mark.parametrize("case", list(CASES))
def test_forward_parity(case):
    from paper_2309_03523_amd.runner import DysatDevice
    c = CASES[case]
    wl = synth.dysat_small(40 + len(case), c["T"], c["N"], 128, 8, c["deg"], c["chunks"], hub=True)
    dd = DysatDevice(wl, validate_level=1, **c.get("kw", {}))
    got = dd.forward().float().cpu().numpy()
    want = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 8)["Y"]
    cov = _covered(wl)
    e = rel_err(got[cov], want[cov], floor=1.0)
    print(f"{case}: Y rel_err {e:.3e}", flush=True)
    assert e < TOL
    assert np.isnan(got[~cov]).all()        # rows no chunk covers are not written
    dd.layer.destroy()


@pytest.mark.parametrize("case", list(CASES))
@pytest.mark.parametrize("mode", ["target", "dY"])
def test_backward_parity(case, mode):
    """Gradients of all seven parameter tensors; sums over many rows, so the bf16 roundings of
    the stored gradients (dU, dQ, dK, dV, dz) largely average out."""
    import torch
    from paper_2309_03523_amd.runner import DysatDevice
    c = CASES[case]
    wl = synth.dysat_small(40 + len(case), c["T"], c["N"], 128, 8, c["deg"], c["chunks"], hub=True)
    extra = synth.round_bf16(synth.stream(3, "extra").standard_normal(wl.X.shape).astype(np.float32))
    dd = DysatDevice(wl, **c.get("kw", {}))
    dd.forward()
    dev = torch.from_numpy(extra).cuda().to(torch.bfloat16)
    if mode == "target":
        want = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 8, target=extra)
        grads, loss = dd.backward(target=dev)
        assert abs(loss - want["loss"]) < 2e-3 * want["loss"]
    else:
        want = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 8, dY=extra)
        grads, _ = dd.backward(dY=dev)
    for name in dysat.PARAMS:
        e = rel_err(grads[name], want["grads"][name], floor=1.0)
        print(f"{case}/{mode}: grad {name} rel_err {e:.3e}", flush=True)
        assert e < TOL, (name, e)
    dd.layer.destroy()


def test_config5_scaled_forward_and_gradients():
    """Config 5 at 1/100 of its vertex count (same generator, 128 uneven chunks, power-law
    degrees with split hub rows at the default thresholds): every covered output and all seven
    gradients against the oracle."""
    import torch
    from paper_2309_03523_amd.runner import DysatDevice
    wl, target = synth.config5(seed=0, scale=0.01)
    dd = DysatDevice(wl, validate_level=1, long_nnz=256, part_nnz=128)
    got = dd.forward().float().cpu().numpy()
    want = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 8, target=target)
    e = rel_err(got, want["Y"], floor=1.0)
    print(f"config5@0.01: Y rel_err {e:.3e}", flush=True)
    assert e < TOL
    grads, loss = dd.backward(target=torch.from_numpy(target).cuda().to(torch.bfloat16))
    assert abs(loss - want["loss"]) < 2e-3 * want["loss"]
    for name in dysat.PARAMS:
        e = rel_err(grads[name], want["grads"][name], floor=1.0)
        print(f"config5@0.01: grad {name} rel_err {e:.3e}", flush=True)
        assert e < TOL, (name, e)
    dd.layer.destroy()


def _one_vertex_problem(wl, v, chunk):
    from workloads import sampling
    return sampling.one_vertex_problem(wl.graph, v, chunk, wl.X, wl.C, wl.F, wl.params)


@pytest.mark.timeout(600)            # the full-size case takes about 100 s, most of it generating the inputs
@pytest.mark.parametrize("scale", [0.25, 1.0])
def test_config5_sampled(scale):
    """Config 5 at full size and at a quarter of its vertex count, as bench.py's config5 / config5s
    workloads launch it (default split thresholds, 128 uneven chunks, hub rows of tens of thousands
    of neighbours): outputs of a seeded sample of vertices of every chunk, and of the largest hubs,
    each computed by the oracle on its own."""
    from paper_2309_03523_amd.runner import DysatDevice
    wl, _ = synth.config5(seed=0, scale=scale)
    dd = DysatDevice(wl)
    got = dd.forward().float().cpu().numpy()
    assert not np.isnan(got).any()              # the chunks cover every (vertex, snapshot)
    rng = synth.stream(0, "parity-sample")
    deg0 = np.diff(wl.graph.snaps[0].rowptr)
    hubs = set(np.argsort(deg0)[-4:].tolist())
    worst, n, gs, ws = 0.0, 0, [], []
    for chunk in wl.chunks.tolist():
        v_lo, v_hi = chunk[0], chunk[1]
        pick = set((rng.choice(v_hi - v_lo, size=2, replace=False) + v_lo).tolist()) | {v_lo, v_hi - 1}
        pick |= {h for h in hubs if v_lo <= h < v_hi}
        for v in sorted(pick):
            g1, c1, p1, X1, C1 = _one_vertex_problem(wl, v, chunk)
            want = dysat.forward(g1, c1, p1, X1, C1, 8)["Y"][:, 0]
            gs.append(got[chunk[2]:chunk[3], v])
            ws.append(want)
            worst = max(worst, rel_err(gs[-1], want, floor=1.0))
            n += 1
    e = rel_err(np.stack(gs), np.stack(ws), floor=1.0)
    print(f"config5@{scale:g}: {n} sampled vertices (largest degree {int(deg0.max())}), Y rel_err {e:.3e} "
          f"(worst vertex against its own RMS {worst:.3e}); " + parity_str(np.stack(gs), np.stack(ws)), flush=True)
    assert n >= 128 * 3 and e < TOL and worst < TOL
    dd.layer.destroy()


def test_attention_argument_errors():
    import torch
    from paper_2309_03523_amd.binding import DgcError
    from paper_2309_03523_amd.runner import DysatDevice
    wl = synth.dysat_small(3, 4, 40, 128, 8, 3.0, [[0, 40, 0, 4]])
    dd = DysatDevice(wl)
    with pytest.raises(DgcError) as ei:      # backward before forward
        dd.layer.backward(dd.Y, target=dd.Y)
    assert ei.value.code == 7
    dd.forward()
    with pytest.raises(DgcError) as ei:      # neither dY nor target
        dd.layer.backward(dd.Y)
    assert ei.value.code == 1
    with pytest.raises(DgcError) as ei:      # fp32 pitch rules do not apply: bf16 pitch must be a multiple of 8
        dd.layer.forward(torch.zeros(4, 40, 132, dtype=torch.bfloat16, device="cuda")[:, :, :128], dd.C, dd.Y)
    assert ei.value.code == 1
    with pytest.raises(DgcError) as ei:      # no recurrent state for this layer
        dd.layer.forward(dd.X, dd.C, dd.Y, H0=torch.zeros(40, 128, device="cuda"))
    assert ei.value.code == 1
    dd.layer.destroy()
    wl2 = synth.dysat_small(4, 33, 40, 128, 8, 3.0, [[0, 40, 0, 33]])
    with pytest.raises(DgcError) as ei:      # window longer than 32 snapshots
        DysatDevice(wl2)
    assert ei.value.code == 4


@pytest.mark.parametrize("case", ["ragged", "split", "single", "wide_mixed"])
def test_input_gradient_parity(case):
    """dL/dX of the covered rows (bf16) against the oracle; rows no chunk covers are not written;
    asking for it does not change the parameter gradients."""
    import torch
    from paper_2309_03523_amd.runner import DysatDevice
    c = CASES[case]
    wl = synth.dysat_small(40 + len(case), c["T"], c["N"], 128, 8, c["deg"], c["chunks"], hub=True)
    extra = synth.round_bf16(synth.stream(3, "extra").standard_normal(wl.X.shape).astype(np.float32))
    dd = DysatDevice(wl, **c.get("kw", {}))
    dd.forward()
    dev = torch.from_numpy(extra).cuda().to(torch.bfloat16)
    plain, _ = dd.backward(dY=dev)
    dX = torch.full((wl.graph.T, wl.graph.N, 136), float("nan"), dtype=torch.bfloat16, device="cuda")[:, :, :128]
    grads, _ = dd.backward(dY=dev, dX=dX)
    for name in dysat.PARAMS:
        np.testing.assert_array_equal(grads[name], plain[name])
    want = dysat.gradients(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 8, dY=extra, want_dx=True)["dX"]
    got = dX.float().cpu().numpy()
    cov = _covered(wl)
    g, w = got[cov].astype(np.float64), want[cov]
    # A row's gradient is one product of that row's dz with W: nothing averages the bf16 roundings
    # of the stored intermediates out (as the sums over rows of the weight gradients do), and
    # rows differ in scale by more than 10x (a vertex with only its self-loop keeps all of its
    # row's gradient).  So every element is measured against its own row's RMS, and each row as a
    # whole against its norm.
    row_rms = np.sqrt((w * w).mean(axis=1))
    assert row_rms.min() > 0
    e = float((np.abs(g - w) / np.maximum(np.abs(w), row_rms[:, None])).max())
    e_row = float((np.sqrt(((g - w) ** 2).mean(axis=1)) / row_rms).max())
    print(f"{case}: dX max element error {e:.3e} (floor: the row's RMS), max row error {e_row:.3e} ({int(cov.sum())} rows)",
          flush=True)
    assert e < TOL and e_row < 1e-2
    assert np.isnan(got[~cov]).all()
    dd.layer.destroy()
