"""The forward pass under HIP graph capture: the entry point only enqueues kernels (no
allocation, no memset, no synchronisation), so a caller can capture it once and replay it.
Every replay is checked against the eager result for the inputs of that moment, with eager
work and synchronisations between the replays."""
import numpy as np
import pytest

from paper_2309_03523_amd import synth

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
