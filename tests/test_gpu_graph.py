"""The forward pass under HIP graph capture: the entry point only enqueues kernels (no
allocation, no memset, no synchronisation), so a caller can capture it once and replay it.
Every replay is checked against the eager result for the inputs of that moment, with eager
work and synchronisations between the replays."""
import numpy as np
import pytest

from workloads import synth

pytestmark = pytest.mark.gpu


def _capture_and_replay(dw, forward, new_inputs):
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        forward()                                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        forward()
    for k in range(4):
        new_inputs(k)                              # eager work between the replays
        forward()
        torch.cuda.synchronize()
        eager = dw.Y.clone()
        dw.Y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(torch.nan_to_num(dw.Y, nan=-7.0), torch.nan_to_num(eager, nan=-7.0)), f"replay {k}"


@pytest.mark.parametrize("kind,layers,S", [("gru", 1, 32), ("lstm", 2, 128), ("gru", 1, 96)])
def test_forward_replays_from_a_graph(kind, layers, S):
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F = 8, 1000, 32
    chunks = [[0, 250, 0, 8], [250, 500, 0, 8], [500, 750, 0, 8], [750, 1000, 0, 8]]
    wl = synth.random_small(5, T, N, F, S, S, 8.0, chunks, kind, n_struct_layers=layers, hub=True)
    dw = DeviceWorkload(wl)
    gen = torch.Generator(device="cuda").manual_seed(1)

    def forward():
        dw.layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=dw.H0)

    def new_inputs(k):
        dw.X.copy_(torch.randn(dw.X.shape, device="cuda", generator=gen))
        dw.C.mul_(0.5).add_(0.1 * k)

    _capture_and_replay(dw, forward, new_inputs)
    dw.layer.destroy()


def test_temporal_fusion_replays_from_a_graph():
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F, S = 8, 600, 24, 64
    chunks = [[0, 300, 0, 8], [300, 600, 0, 4], [300, 600, 4, 8]]
    wl = synth.random_small(6, T, N, F, S, S, 5.0, chunks, "gru")
    dw = DeviceWorkload(wl)
    dw.layer.set_presence(torch.from_numpy(synth.presence(6, T, N)).cuda())
    gen = torch.Generator(device="cuda").manual_seed(2)
    n_state = dw.H0.shape[0]
    HN = torch.zeros(n_state, S, device="cuda")

    def forward():
        dw.layer.forward(dw.X, dw.C, dw.Y, H0=dw.H0, HN=HN)

    def new_inputs(k):
        dw.X.copy_(torch.randn(dw.X.shape, device="cuda", generator=gen))
        dw.H0.mul_(0.9)

    _capture_and_replay(dw, forward, new_inputs)
    dw.layer.destroy()


def _replay_training_step(step, read_grads, new_inputs):
    """Capture forward + backward once (after an eager step, which also makes the layer's lazy
    allocations), replay it for changing inputs and compare loss and gradients with eager runs."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for k in range(3):
        new_inputs(k)
        step()
        torch.cuda.synchronize()
        eager = read_grads()
        graph.replay()
        torch.cuda.synchronize()
        replayed = read_grads()
        for name in eager:
            np.testing.assert_array_equal(replayed[name], eager[name], err_msg=f"replay {k}: {name}")


def test_evolve_training_step_replays_from_a_graph():
    import torch
    import oracle
    from paper_2309_03523_amd.runner import DeviceWorkload
    T, N, F = 6, 300, 64
    chunks = [[0, 100, 0, 6], [100, 300, 0, 3], [100, 300, 3, 6]]
    wl = synth.random_small(9, T, N, F, F, F, 5.0, chunks, "none", hub=True)
    wl.params = synth.evolve_params(9, F, F, random_bias=True)
    dw = DeviceWorkload(wl, struct_kind="evolve_gcn_o", act_out="relu")
    gen = torch.Generator(device="cuda").manual_seed(4)
    target = torch.randn(T, N, F, device="cuda", generator=gen)
    loss = torch.zeros(1, device="cuda")
    dX = torch.zeros(T, N, F, device="cuda")

    def step():
        dw.layer.forward(dw.X, dw.C, dw.Y)
        dw.layer.backward(dw.Y, target=target, loss_out=loss, dX=dX)

    def read_grads():
        out = {n: dw.layer.get_param(n + ".grad", wl.params[n].shape) for n in oracle.EVOLVE_PARAMS}
        out["loss"] = loss.cpu().numpy()
        out["dX"] = dX.cpu().numpy()
        return out

    def new_inputs(k):
        dw.X.copy_(torch.randn(dw.X.shape, device="cuda", generator=gen))
        target.mul_(0.5)

    _replay_training_step(step, read_grads, new_inputs)
    dw.layer.destroy()


@pytest.mark.parametrize("T,chunks", [(6, [[0, 70, 0, 6], [70, 150, 0, 4]]), (20, [[0, 70, 0, 20], [70, 150, 3, 12]])])
def test_attention_training_step_replays_from_a_graph(T, chunks):
    """(the second case has a window of more than 16 snapshots: one vertex per tile in the temporal kernels)"""
    import torch
    from oracle import dysat
    from paper_2309_03523_amd.runner import DysatDevice
    wl = synth.dysat_small(11, T, 150, 128, 8, 4.0, chunks, hub=True)
    dd = DysatDevice(wl)
    gen = torch.Generator(device="cuda").manual_seed(5)
    target = torch.randn(dd.X.shape, device="cuda", generator=gen).to(torch.bfloat16)
    loss = torch.zeros(1, device="cuda")
    dX = torch.zeros_like(dd.X)

    def step():
        dd.layer.forward(dd.X, dd.C, dd.Y)
        dd.layer.backward(dd.Y, target=target, loss_out=loss, dX=dX)

    def read_grads():
        out = {n: dd.layer.get_param(n + ".grad", wl.params[n].shape) for n in dysat.PARAMS}
        out["loss"] = loss.cpu().numpy()
        out["dX"] = dX.float().cpu().numpy()
        return out

    def new_inputs(k):
        dd.X.copy_(torch.randn(dd.X.shape, device="cuda", generator=gen).to(torch.bfloat16))

    _replay_training_step(step, read_grads, new_inputs)
    dd.layer.destroy()
