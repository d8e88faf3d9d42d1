"""Results do not depend on the order in which workgroups happen to run: no kernel adds floating
point numbers with atomics, split rows and gradient partial sums are merged in a fixed order.  Two
runs of the same call give the same bits (forward outputs, final states, losses, gradients)."""
import numpy as np
import pytest

from workloads import synth

pytestmark = pytest.mark.gpu


def test_recurrent_layers_forward_twice():
    from paper_2309_03523_amd.runner import DeviceWorkload
    for wl, kw in ((synth.config2(seed=3, scale=0.02), {}),
                   (synth.config3(seed=3, scale=0.004), dict(act_hidden="relu", act_out="none")),
                   (synth.config3(seed=3, scale=0.004, input_concat=True), dict(act_hidden="relu", act_out="none"))):
        dw = DeviceWorkload(wl, long_nnz=64, part_nnz=16, **kw)      # many split rows
        Y, HN = dw.forward(want_state=True)
        y1, h1 = Y.cpu().numpy().copy(), HN.cpu().numpy().copy()
        dw.Y.fill_(float("nan"))
        Y, HN = dw.forward(want_state=True)
        np.testing.assert_array_equal(Y.cpu().numpy(), y1)
        np.testing.assert_array_equal(HN.cpu().numpy(), h1)
        dw.layer.destroy()


def test_evolving_gcn_training_step_twice():
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload
    wl, target = synth.config4(seed=3, scale=0.004)
    dw = DeviceWorkload(wl, struct_kind="evolve_gcn_o", act_out="relu", long_nnz=64, part_nnz=16)
    tgt = torch.from_numpy(target).cuda()
    runs = []
    for _ in range(2):
        Y = dw.forward()
        loss = torch.zeros(1, device="cuda")
        dX = torch.full_like(dw.X, float("nan"))
        dw.layer.backward(Y, target=tgt, loss_out=loss, dX=dX)
        torch.cuda.synchronize()
        grads = {k: dw.layer.get_param(k + ".grad", v.shape).copy() for k, v in wl.params.items()}
        runs.append((Y.cpu().numpy().copy(), float(loss.item()), dX.cpu().numpy().copy(), grads))
    (y1, l1, x1, g1), (y2, l2, x2, g2) = runs
    np.testing.assert_array_equal(y1, y2)
    assert l1 == l2
    np.testing.assert_array_equal(x1, x2)
    for k in g1:
        np.testing.assert_array_equal(g1[k], g2[k])
    dw.layer.destroy()


@pytest.mark.parametrize("wide", [False, True])
def test_attention_training_step_twice(wide):
    import torch
    from paper_2309_03523_amd.runner import DysatDevice
    if wide:     # a window of more than 16 snapshots: one vertex per tile in the temporal kernels
        wl = synth.dysat_small(3, 24, 300, 128, 8, 5.0, [[0, 140, 0, 24], [140, 300, 0, 24]], hub=True)
        target = synth.round_bf16(synth.stream(3, "target").standard_normal(wl.X.shape).astype(np.float32))
    else:
        wl, target = synth.config5(seed=3, scale=0.004)
    dd = DysatDevice(wl, long_nnz=64, part_nnz=16)
    tgt = torch.from_numpy(target).cuda().to(torch.bfloat16)
    runs = []
    for _ in range(2):
        y = dd.forward().float().cpu().numpy().copy()
        dX = torch.full_like(dd.X, float("nan"))
        grads, loss = dd.backward(target=tgt, dX=dX)
        runs.append((y, loss, dX.float().cpu().numpy().copy(), {k: v.copy() for k, v in grads.items()}))
    (y1, l1, x1, g1), (y2, l2, x2, g2) = runs
    np.testing.assert_array_equal(y1, y2)
    assert l1 == l2
    np.testing.assert_array_equal(x1, x2)
    for k in g1:
        np.testing.assert_array_equal(g1[k], g2[k])
    dd.layer.destroy()
