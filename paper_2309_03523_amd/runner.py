"""Plumbing between a synthetic Workload (host NumPy arrays) and the HIP layer: upload with
torch, create the layer, load parameters, run.  No arithmetic of the method lives here."""
from __future__ import annotations

from typing import Optional

import numpy as np

from .binding import DgcLayer

# Optional progress sink for large uploads: a callable taking one string, None = silent.
progress = None


class DeviceWorkload:
    """Device copies of a Workload's graph and tensors plus a created layer."""

    def __init__(self, wl, *, gather_mode: str = "in_place", validate_level: int = 0, act_hidden: str = "relu",
                 act_out: str = "none", pitch: Optional[int] = None, struct_kind: str = "gcn", **layer_kw):
        import torch
        dev = torch.device("cuda:0")
        self.wl = wl
        on_device = bool(getattr(wl, "on_device", False))   # graph and tensors already in GPU memory
        if on_device:
            N, T = wl.N, wl.T
            self.rowptr, self.colidx = wl.rowptr, wl.col
        else:
            g = wl.graph
            N, T = g.N, g.T
            self.rowptr = [torch.from_numpy(s.rowptr).to(dev) for s in g.snaps]
            self.colidx = [torch.from_numpy(s.col).to(dev) for s in g.snaps]
        import time
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.layer = DgcLayer(self.rowptr, self.colidx, N, wl.chunks, F=wl.F, S=wl.S, H=wl.H,
                              time_kind=wl.time_kind, n_struct_layers=wl.n_struct_layers,
                              act_hidden=act_hidden, act_out=act_out, gather_mode=gather_mode,
                              validate_level=validate_level, struct_kind=struct_kind,
                              lstm_input_concat=bool(wl.notes.get("input_concat", False)), **layer_kw)
        self.create_s = time.perf_counter() - t0     # dgc_layer_create: validation, packing, workspace (it synchronises)
        self.layer.set_params(wl.params)

        def up(a, ld=None):
            """[T,N,F] -> device tensor with row pitch ld (a multiple of 4)."""
            if a is None:
                return None
            T, N, F = a.shape
            ld = ld or (F + 3) // 4 * 4
            buf = torch.full((T, N, ld), float("nan"), dtype=torch.float32, device=dev)
            for t in range(T):      # snapshot by snapshot: no second full-size device copy
                buf[t, :, :F] = torch.from_numpy(a[t]).to(dev)
                if a.nbytes >= (1 << 32) and (t + 1) % max(1, T // 4) == 0 and progress:
                    progress(f"  upload {tuple(a.shape)}: {t + 1}/{T} snapshots")
            return buf[:, :, :F] if ld != F else buf

        if on_device:
            self.X, self.C, self.C1, self.H0 = wl.X[:, :, :wl.F], wl.C[:, :, :wl.F], wl.C1, wl.H0
        else:
            self.X = up(wl.X, pitch)
            self.C = up(wl.C, pitch)
            self.C1 = up(wl.C1)
            self.H0 = torch.from_numpy(wl.H0).to(dev) if wl.H0 is not None else None
        self.Y = torch.full((T, N, self.layer.out_dim), float("nan"), dtype=torch.float32, device=dev)

    def forward(self, *, reset_mask=None, want_state: bool = False, use_h0: bool = True, C=None, C1=None):
        import torch
        rm = None
        if reset_mask is not None:
            rm = torch.from_numpy(np.ascontiguousarray(reset_mask, np.uint8)).to(self.Y.device)
        HN = None
        if want_state and self.wl.time_kind != "none":
            n_state = (2 if self.wl.time_kind == "lstm" else 1) * max(1, self.layer.n_time_layers)
            tot = int((self.wl.chunks[:, 1] - self.wl.chunks[:, 0]).sum())
            HN = torch.full((n_state * tot, self.wl.H), float("nan"), dtype=torch.float32, device=self.Y.device)
        self.layer.forward(self.X, self.C if C is None else C, self.Y, C1=self.C1 if C1 is None else C1,
                           H0=self.H0 if use_h0 else None, reset_mask=rm, HN=HN)
        torch.cuda.synchronize()
        return (self.Y, HN) if want_state else self.Y


def run_forward(wl, **kw) -> np.ndarray:
    """Upload, run one forward pass on cuda:0, return Y as a host array."""
    dw = DeviceWorkload(wl, **kw)
    Y = dw.forward().cpu().numpy()
    dw.layer.destroy()
    return Y


class DysatDevice:
    """Device copies (bfloat16) of a graph-attention workload plus a created layer."""

    def __init__(self, wl, *, validate_level: int = 0, **layer_kw):
        import time
        import torch
        dev = torch.device("cuda:0")
        self.wl = wl
        on_device = bool(getattr(wl, "on_device", False))   # graph and bfloat16 tensors already in GPU memory
        if on_device:
            N, T = wl.N, wl.T
            self.rowptr, self.colidx = wl.rowptr, wl.col
        else:
            N, T = wl.graph.N, wl.graph.T
            self.rowptr = [torch.from_numpy(s.rowptr).to(dev) for s in wl.graph.snaps]
            self.colidx = [torch.from_numpy(s.col).to(dev) for s in wl.graph.snaps]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.layer = DgcLayer(self.rowptr, self.colidx, N, wl.chunks, F=wl.F, S=wl.S, H=wl.H, time_kind="self_attn",
                              struct_kind="gat", dtype="bf16", heads=wl.notes["heads"],
                              validate_level=validate_level, **layer_kw)
        self.create_s = time.perf_counter() - t0
        self.layer.set_params(wl.params)
        if on_device:
            self.X, self.C = wl.X, wl.C
        else:
            self.X = torch.from_numpy(wl.X).to(dev).to(torch.bfloat16)
            self.C = torch.from_numpy(wl.C).to(dev).to(torch.bfloat16)
        self.Y = torch.full((T, N, wl.S), float("nan"), dtype=torch.bfloat16, device=dev)

    def forward(self, C=None):
        import torch
        self.layer.forward(self.X, self.C if C is None else C, self.Y)
        torch.cuda.synchronize()
        return self.Y

    def backward(self, *, target=None, dY=None, dX=None):
        """Gradients of the seven parameter tensors (dict of host arrays) and the loss (or None);
        dX: optional bfloat16 device tensor [T,N,F] that receives the input gradient."""
        import torch
        loss = torch.zeros(1, device=self.Y.device) if target is not None else None
        self.layer.backward(self.Y, dY=dY, target=target, loss_out=loss, dX=dX)
        torch.cuda.synchronize()
        grads = {k: self.layer.get_param(k + ".grad", v.shape) for k, v in self.wl.params.items()}
        return grads, (float(loss.item()) if loss is not None else None)
