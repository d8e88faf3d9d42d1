#!/usr/bin/env python3
"""Benchmark of the fused-chunk DGNN layer (GCN aggregation + transform + GRU) on one MI355X.

A step is one forward pass of the whole layer over the fused batch of chunks of the named
workload (default: configuration 2, the one the metric is quoted on: 32 snapshots x 100k vertices, F=S=H=128,
64 chunks).  Inputs are generated once, uploaded, and resident in HBM before timing starts.
Prints ONE JSON line: throughput in snapshot-vertex embeddings/s, the roofline of the dominant
kernel (the fused dense + recurrent kernel, measured live with HIP events on the launch
stream), and the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="config2", choices=["config1", "config2", "config2s", "config2tf", "config3", "config3w", "config3wc", "config3h", "config4s", "config4", "config5s", "config5", "config5w32", "stale", "fusion", "chunkgen", "config2lp"])
    ap.add_argument("--windows", default="0,1,2,3",
                    help="config3: which of its four 32-snapshot windows to run, one fused batch each (memory-capped fusion)")
    ap.add_argument("--mpnn-lstm", action="store_true",
                    help="config3: the paper's MPNN-LSTM in full (Section 6): the LSTM reads both GCN layers' outputs and "
                         "a second LSTM layer is stacked on the first")
    ap.add_argument("--presence", action="store_true",
                    help="config2lp: also set config2tf's presence matrix (temporal fusion over the generated chunks)")
    ap.add_argument("--no-configs", action="store_true",
                    help="config2 (the default): do not also run configs 1, 3, 4 and 5 for the line's `configs` object")
    ap.add_argument("--config-steps", type=int, default=5, help="timed steps of each extra configuration")
    ap.add_argument("--gather-mode", default="in_place", choices=["in_place", "staged"])
    ap.add_argument("--agg-kernel", default="table", choices=["table", "walk"],
                    help="aggregation kernels: the ones that read the edge table built at create (default) or the ones "
                         "that walk colidx")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--with-dx", action="store_true",
                    help="config4 / config5 workloads: the backward pass also computes the gradient of the input rows")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain device copy of X (a kernel of known size, to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


def make_workload(name: str, seed: int):
    from workloads import synth
    from paper_2309_03523_amd import runner
    synth.progress = runner.progress = lambda msg: print(msg, file=sys.stderr, flush=True)
    if name == "config1":
        return synth.config1(seed), "config1: 8 snapshots x 1000 vertices, ER avg deg 8, F=S=H=32, 4 chunks"
    if name == "config2s":
        return synth.config2(seed, scale=0.05), "config2 at 1/20 scale"
    if name == "config2tf":
        wl = synth.config2(seed)
        wl.notes["present"] = synth.presence(seed, wl.graph.T, wl.graph.N)
        return wl, ("config2 with temporal fusion: every vertex present in a snapshot with its own probability "
                    "U(0.15, 1); sequences concatenated into lanes of 8 (first-fit decreasing) instead of padded, each "
                    "starting from its own row of H0 as in config2")
    if name in ("config3w", "config3wc", "config3h"):
        cat = name == "config3wc"
        scale = 0.5 if name == "config3h" else 0.125
        return synth.config3(seed, scale=scale, input_concat=cat), (
            f"config3 at 1/{int(1 / scale)} of its vertex count, one 32-snapshot window: {int(2000 * scale)}k vertices, 2 GCN layers (172->128->128) + LSTM"
            + (" reading both GCN layers' outputs (256 wide)" if cat else "") + ", 64 uneven ranges")
    if name == "config4":
        from workloads import device_gen
        wl, target = device_gen.config4(seed, 1.0, say=synth.progress)
        wl.notes["target"] = target
        return wl, (f"config4: EvolveGCN-O, 64 snapshots x {wl.N} vertices, avg degree 16, F = S = 256, 32 chunks, "
                    "forward + backward (MSE); inputs drawn on the device")
    if name == "config4s":
        scale = 0.125
        wl, target = synth.config4(seed, scale=scale)
        wl.notes["target"] = target
        return wl, (("config4 at 1/8 of its vertex count" if name == "config4s" else "config4") +
                    f": EvolveGCN-O, 64 snapshots x {wl.graph.N} vertices, avg degree 16, "
                    "F = S = 256, 32 chunks, forward + backward (MSE)")
    return synth.config2(seed), ("config2: 32 snapshots x 100k vertices, lognormal edge counts, power-law "
                                 "degrees (tail 2.1), F=S=H=128, GCN+GRU, 64 chunks = 4 windows of 8 x 16 "
                                 "uneven vertex ranges")


def parity_numbers(got, want) -> dict:
    """Error figures of a device result against the oracle's: the relative error with its denominator
    floored at 1e-2 RMS and at 1e-1 RMS (fp32 paths assert the second, see the tests), at RMS (what the
    bf16 path asserts), the largest absolute error in units of RMS, and the 99.9th percentile of the
    unfloored relative error."""
    import numpy as np
    got = np.asarray(got, np.float64).ravel()
    want = np.asarray(want, np.float64).ravel()
    rms = max(float(np.sqrt(np.mean(want * want))), 1e-300)
    d, a = np.abs(got - want), np.abs(want)
    nz = a > 0
    return {"floor_1e-2_rms": float(np.max(d / np.maximum(a, 1e-2 * rms))),
            "floor_1e-1_rms": float(np.max(d / np.maximum(a, 1e-1 * rms))),
            "floor_rms": float(np.max(d / np.maximum(a, rms))),
            "max_abs_over_rms": float(d.max() / rms),
            "p999_unfloored": float(np.quantile(d[nz] / a[nz], 0.999)) if nz.any() else 0.0}


AGG_KERNELS = {"table": "k_agg_short + k_agg_long + k_spmm_long_reduce (edge-table kernels)",
               "walk": "k_spmm_short + k_spmm_long + k_spmm_long_reduce (column-walking kernels)"}


def flops_per_row(wl) -> dict:
    """Algorithmic flops per snapshot-vertex row of each step of the path."""
    g = {"gru": 3, "lstm": 4, "none": 0}[wl.time_kind]
    dense = 2 * wl.F * wl.S + (2 * wl.S * wl.S if wl.n_struct_layers == 2 else 0)
    s_in = 2 * wl.S if wl.notes.get("input_concat") else wl.S     # width of the time encoder's input
    rnn = 2 * s_in * g * wl.H + 2 * wl.H * g * wl.H
    return {"transform": dense, "rnn": rnn}


def measured_traffic(workload: str, gather_mode: str) -> dict:
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (two separate runs of
    this script, scaled by a plain copy of known size; figures and commands in profiles/).  They
    cannot be collected inside a timed run, so they are read from the committed summary."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(f"{workload}/{gather_mode}", {})
    except (OSError, ValueError):
        return {}


def with_traffic_rate(k: dict) -> dict:
    """Adds the rate of the measured HBM traffic (committed rocprofv3 counters) over the launch time
    measured in this run, next to the algorithmic figure."""
    if k.get("traffic") and k.get("ms_per_launch"):
        k["traffic_GBs"] = k["traffic"] / (k["ms_per_launch"] * 1e-3) / 1e9
        k["traffic_frac_of_hbm_peak"] = k["traffic_GBs"] / PEAK_HBM_GBS
    return k


def evolve_report(args, wl, desc, dw, rows, value, ms_per_step, stage, t_gen, t_create, loss, graph_ms=None, dX=None) -> dict:
    """JSON line for the EvolveGCN-O workload: a step is forward + backward."""
    import numpy as np
    import oracle
    F, S = wl.F, wl.S
    nnz = int(dw.layer.packing("seg_nnz_off")[-1])
    fwd_flops, bwd_flops = 2.0 * F * S * rows, 2.0 * F * S * rows
    kernels = {
        "dense_forward": {"kernel": "k_dense_wave<NONE> (Y = relu(M W_t), per-snapshot weights)", "bound": "mfma",
                          "achieved": fwd_flops / (stage[3] * 1e-3) / 1e12, "peak": PEAK_FP32_MFMA_TFLOPS,
                          "unit": "TFLOP/s", "ms_per_launch": float(stage[3])},
        "weight_gradient": {"kernel": "k_dw_partial + k_dw_reduce (dW_t = M_t^T dP_t)", "bound": "mfma",
                            "achieved": bwd_flops / (stage[5] * 1e-3) / 1e12, "peak": PEAK_FP32_MFMA_TFLOPS,
                            "unit": "TFLOP/s", "ms_per_launch": float(stage[5])},
    }
    traffic = measured_traffic(args.workload, args.gather_mode)
    for name, k in kernels.items():
        k["frac"] = k["achieved"] / k["peak"]
        k["traffic"] = traffic.get(name)
    dom = max(kernels.values(), key=lambda k: k["ms_per_launch"])
    out = {"metric": "snapshot-vertex embeddings/s per DGNN layer", "value": value, "unit": "embeddings/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": desc, "rows": rows, "nnz": nnz, "gather_mode": args.gather_mode,
                      "pass": "forward+backward" + (" incl. input gradient" if args.with_dx else "")},
           "roofline": dom, "kernels": kernels,
           "stage_ms": {"aggregate0": float(stage[0]), "dense_forward": float(stage[3]),
                        "weight_evolution": float(stage[4]), "weight_gradient": float(stage[5]),
                        "bptt": float(stage[6])},
           "loss": float(loss.item()), "setup_s": {"generate": t_gen, "upload_create_pack": t_create}}
    if graph_ms is not None:
        out["hip_graph_replay_ms_per_step"] = graph_ms
    if not args.no_cpu_baseline and getattr(wl, "on_device", False):
        out["parity"], out["cpu_baseline"] = evolve_sampled_baseline(wl, dw, dX, args.seed)
    elif not args.no_cpu_baseline:
        # the oracle on a few whole chunks of the first window (forward + gradients)
        import time as _t
        big = rows > 8_000_000        # the full configuration: one chunk, forward only, to stay within a minute or two
        sub = wl.chunks[:1] if big else wl.chunks[:2]
        print(f"oracle on {len(sub)} chunk(s) ...", file=sys.stderr, flush=True)
        t0 = _t.perf_counter()
        o = oracle.evolve(wl.graph, sub, wl.params, wl.X, wl.C, wl.notes["target"], want_grads=not big)
        dt = _t.perf_counter() - t0
        print(f"oracle done in {dt:.1f} s", file=sys.stderr, flush=True)
        n_rows = int(((sub[:, 1] - sub[:, 0]) * (sub[:, 3] - sub[:, 2])).sum())
        # only the sampled chunks' rows are copied back and compared (no pass over the whole tensors)
        want = np.concatenate([o["Y"][t0_:t1_, a_:b_].reshape(-1) for a_, b_, t0_, t1_ in sub.tolist()]).astype(np.float64)
        got = np.concatenate([dw.Y[t0_:t1_, a_:b_].cpu().numpy().reshape(-1) for a_, b_, t0_, t1_ in sub.tolist()])
        assert not np.isnan(want).any()
        par = parity_numbers(got, want)
        err = par["floor_1e-1_rms"]
        out["parity"] = par
        out["cpu_baseline"] = {"value": n_rows / dt, "unit": "embeddings/s", "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"the first {len(sub)} chunk(s) (of {len(wl.chunks)}), forward"
                                         f"{'' if big else ' + gradients'} = {n_rows} rows, "
                                         f"{dt:.1f} s (weight recurrence over all 64 snapshots included)",
                               "gpu_max_rel_err_on_sample": err}
    return out


def evolve_sampled_baseline(data, dw, dX, seed: int):
    """Config 4 at its stated size (inputs live on the device): the oracle on a seeded sample of vertices
    of every chunk (first, last and two random ones; stand-in problems built from copies of the rows
    they read), and, if the step computed it, input-gradient rows of one vertex per chunk."""
    import numpy as np
    from oracle import sampled
    from workloads import sampling, synth
    hg = data.host_graph()
    rng = synth.stream(seed, "bench-sample")
    chunks = data.chunks.tolist()
    gs, ws, gdx, wdx, dt_all, rows_eval = [], [], [], [], 0.0, 0
    for w in sorted({c[2] for c in chunks}):
        win = [c for c in chunks if c[2] == w]
        picks = []
        for ch in win:
            pick = {ch[0], ch[1] - 1} | set((rng.choice(ch[1] - ch[0], size=2, replace=False) + ch[0]).tolist())
            picks += [(v, ch) for v in sorted(pick)]
        want, dt = sampled.evolve_forward_reference(data, hg, picks, data.params)
        dt_all += dt
        rows_eval += sum(ch[3] - ch[2] for _, ch in picks)
        gs += [dw.Y[ch[2]:ch[3], v].cpu().numpy() for v, ch in picks]
        ws += want
        if dX is not None:
            gp = [(sampling.bounded_pick(hg, ch, rng, 600), ch) for ch in win]
            _, dxs, held, dt = sampled.evolve_input_gradient_reference(data, hg, gp, data.params, data.notes["target"], data.rows)
            dt_all += dt
            for i, ((v, ch), rows_i) in enumerate(zip(gp, held)):
                # a pick is set aside if a ReLU gate its gradient passes through lies within rounding of zero
                if all(((dw.Y[t, j].cpu().numpy() > 0) == (y_or > 0)).all() for t, j, y_or in rows_i):
                    gdx.append(dX[ch[2]:ch[3], v, :data.F].cpu().numpy())
                    wdx.append(dxs[i])
    par = parity_numbers(np.stack(gs), np.stack(ws))
    par["sampled_vertices"] = len(gs)
    if gdx:
        par["input_gradient"] = parity_numbers(np.stack(gdx), np.stack(wdx))
        par["input_gradient"]["sampled_vertices"] = len(gdx)
    base = {"value": rows_eval / dt_all, "unit": "embeddings/s", "cores": sampled.oracle.threads(),
            "kind": "oracle", "cpu": cpu_model(),
            "sample": f"{len(gs)} vertices, four of every one of the {len(chunks)} chunks over the chunk's window = {rows_eval} rows, "
                      f"{dt_all:.1f} s (each evaluation evolves the 64 weight matrices again)",
            "gpu_max_rel_err_on_sample": par["floor_1e-1_rms"]}
    return par, base


def cpu_model() -> str:
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, Y_gpu, target_seconds: float, seed: int) -> dict:
    """Time the CPU oracle on a seeded sample of vertices of every chunk (all snapshots of the
    chunk's window), sized from a short calibration run to about target_seconds.  Also returns
    the parity of the GPU result on those rows."""
    import numpy as np
    import oracle
    from workloads import synth

    rng = synth.stream(seed, "bench-sample")
    chunks = wl.chunks
    widths = chunks[:, 1] - chunks[:, 0]
    windows = chunks[:, 3] - chunks[:, 2]

    def sample(per_chunk):
        return [np.sort(rng.choice(int(w), size=min(int(w), per_chunk), replace=False)) + int(c[0])
                for c, w in zip(chunks, widths)]

    out_dim = wl.H if wl.time_kind != "none" else wl.S

    def run(sub):
        Y = np.full((wl.graph.T, wl.graph.N, out_dim), np.nan, np.float32)  # allocated outside the timed call
        t0 = time.perf_counter()
        oracle.forward(wl.graph, chunks, wl.params, wl.X, wl.C, time_kind=wl.time_kind,
                       n_struct_layers=wl.n_struct_layers, C1=wl.C1, H0=wl.H0, subset=sub, Y=Y,
                       act_hidden="relu", act_out="none", input_concat=bool(wl.notes.get("input_concat")))
        return Y, time.perf_counter() - t0

    # grow the sample until one run takes about target_seconds (at most three tries)
    per_chunk = 32
    for _ in range(3):
        sub = sample(per_chunk)
        Y, dt = run(sub)
        if dt >= 0.5 * target_seconds or per_chunk >= widths.max():
            break
        rows_now = sum(len(s) * int(w) for s, w in zip(sub, windows))
        rate = rows_now / max(dt, 1e-6)
        per_chunk = int(max(per_chunk + 1, min(widths.max(), target_seconds * rate / max(1, int(windows.sum())))))
    rows = sum(len(s) * int(w) for s, w in zip(sub, windows))
    mask = ~np.isnan(Y)
    want = Y[mask].astype(np.float64)
    got = Y_gpu[mask].astype(np.float64)
    par = parity_numbers(got, want)
    # the same oracle on one core, on a sample an eighth the size (the first vertices of the sample above)
    n_thr = oracle.threads()
    sub1 = [s_[:max(1, len(s_) // 8)] for s_ in sub]
    rows1 = sum(len(s_) * int(w) for s_, w in zip(sub1, windows))
    oracle.set_threads(1)
    try:
        _, dt1 = run(sub1)
    finally:
        oracle.set_threads(n_thr)
    return {"value": rows / dt, "unit": "embeddings/s", "cores": n_thr, "kind": "oracle",
            "sample": f"{per_chunk} seeded random vertices of each of the {len(chunks)} chunks over the chunk's "
                      f"whole window = {rows} rows, {dt:.1f} s",
            "single_thread": {"value": rows1 / dt1, "unit": "embeddings/s", "cores": 1,
                              "sample": f"{rows1} of those rows, {dt1:.1f} s"},
            "cpu": cpu_model(),
            "gpu_max_rel_err_on_sample": par["floor_1e-1_rms"], "parity": par}


# Algorithmic HBM bytes per snapshot-vertex row of each stage of the graph-attention +
# temporal-attention layer (kbar = stored non-zeros per row; the neighbour rows a stage gathers
# are cache-served re-reads and are reported separately as gather traffic):
def dysat_stage_bytes(kbar: float) -> dict:
    csr = 4.0 * kbar + 8.0
    return {
        "project": 256 + 256 + 256 + 256 + 64 + 32,            # X, C in; zX, zC, s out
        "edge_softmax": csr + 64 + 512 + 32,                    # CSR, own scalars; U (fp32), lse out
        "temporal_fwd": 512 + 256,                              # U in; Y out
        "temporal_bwd": 512 + 256 + 256 + 256 + 3 * 256 + 512 + 3 * 256,   # U, Y, target; dU, dQKV out; U, dQKV in (dW)
        "gat_bwd_rows": csr + 256 + 512 + 96 + 64,              # dU, U, scalars in; d s_dst, c out
        "gat_bwd_cols": csr + 4 * kbar + 4 + 512 + 96 + 512 + 512 + 512,    # CSR, owner; z, scalars; dz out; dz, X, C in (dW)
    }


def dysat_run(args) -> dict:
    """Workload of config 5: graph attention + causal temporal self-attention, bf16, forward +
    backward against MSE targets.  config5 (the stated 1,000,000 vertices) is drawn on the device,
    config5s (a quarter of the vertices) on the host."""
    import numpy as np
    import torch
    from workloads import synth
    from paper_2309_03523_amd.runner import DysatDevice

    scale = 0.25 if args.workload == "config5s" else 1.0
    window = 32 if args.workload == "config5w32" else 16     # config5w32: 32 snapshots x 500,000 vertices, one 32-snapshot window
    synth.progress = lambda msg: print(msg, file=sys.stderr, flush=True)
    on_device = args.workload != "config5s"
    t0 = time.perf_counter()
    if on_device:
        from workloads import device_gen
        wl, tgt = device_gen.config5(args.seed, scale, say=synth.progress, window=window)
        torch.cuda.synchronize()
        n_vertices = wl.N
    else:
        wl, target = synth.config5(args.seed, scale)
        n_vertices = wl.graph.N
    t_gen = time.perf_counter() - t0
    rows, nnz = wl.rows, (wl.nnz if on_device else wl.graph.nnz)
    t0 = time.perf_counter()
    dd = DysatDevice(wl)
    if not on_device:
        tgt = torch.from_numpy(target).cuda().to(torch.bfloat16)
    loss = torch.zeros(1, device="cuda")
    torch.cuda.synchronize()
    t_create = time.perf_counter() - t0
    layer, stream = dd.layer, torch.cuda.current_stream()

    dX = torch.empty_like(dd.X) if args.with_dx else None

    def step():
        layer.forward(dd.X, dd.C, dd.Y, stream=stream)
        layer.backward(dd.Y, target=tgt, loss_out=loss, dX=dX, stream=stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    layer.set_profiling(True)
    stage = np.zeros(13, np.float64)
    n_prof = max(3, min(args.steps, 10))
    for _ in range(n_prof):
        step()
        stage += layer.stage_times()
    stage /= n_prof
    layer.set_profiling(False)
    names = ["project", "edge_softmax", "temporal_fwd", "temporal_bwd", "gat_bwd_rows", "gat_bwd_cols"]
    per_row = dysat_stage_bytes(nnz / rows)
    try:      # HBM bytes per launch measured with rocprofv3 --pmc (profiles/), for the workload they were taken on
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as f:
            measured = json.load(f).get(args.workload, {})
    except (OSError, ValueError):
        measured = {}
    kernels = {}
    for i, nm in enumerate(names):
        ms = float(stage[7 + i])
        ach = per_row[nm] * rows / (ms * 1e-3) / 1e9
        kernels[nm] = {"bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                       "ms_per_launch": ms, "bytes_per_row": per_row[nm],
                       "traffic": measured.get(nm, {}).get("total")}
    for nm in ("edge_softmax", "gat_bwd_rows", "gat_bwd_cols"):
        gather = (nnz / rows) * (256 + 32 + (96 if nm == "gat_bwd_cols" else 0)) * rows
        kernels[nm]["gather_traffic_GBps"] = gather / (kernels[nm]["ms_per_launch"] * 1e-3) / 1e9
    dom_name = max(kernels, key=lambda k: kernels[k]["ms_per_launch"])
    dom = dict(kernels[dom_name], kernel=dom_name)
    out = {"metric": "snapshot-vertex embeddings/s per DGNN layer", "value": rows * args.steps / elapsed,
           "unit": "embeddings/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": 1e3 * elapsed / args.steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"config5{'' if scale == 1.0 else ' at 1/4 of its vertex count'}: graph attention (8 heads x 16) + "
                                  f"causal temporal self-attention, bf16, {window} snapshots x {n_vertices} vertices (one {window}-snapshot window), avg degree 12, "
                                  f"{len(wl.chunks)} uneven chunks, forward + backward (MSE)",
                      "rows": rows, "nnz": nnz,
                      "pass": "forward+backward" + (" incl. input gradient" if args.with_dx else "")},
           "roofline": dom, "kernels": kernels, "loss": float(loss.item()),
           "stage_ms": {nm: kernels[nm]["ms_per_launch"] for nm in names},
           "packing": {"create_ms": 1e3 * dd.create_s,
                       "step_plus_packing_over_one_epoch_ms": 1e3 * elapsed / args.steps + 1e3 * dd.create_s,
                       "step_plus_packing_over_100_epochs_ms": 1e3 * elapsed / args.steps + 10.0 * dd.create_s},
           "setup_s": {"generate": t_gen, "upload_create_pack": t_create}}
    if not args.no_cpu_baseline and on_device:
        # the oracle on sampled vertices of every chunk, each as a one-vertex problem built from copies of
        # the rows it reads (torch CPU, float64, forward)
        from oracle import dysat as odysat
        from workloads import sampling
        from workloads.device_gen import RowFetcher
        hg = wl.host_graph()
        rng = synth.stream(args.seed, "bench-sample")
        fx, fc = RowFetcher(wl.X, wl.F), RowFetcher(wl.C, wl.F)
        gs, ws, dt = [], [], 0.0
        for ch in wl.chunks.tolist():
            for v in sorted({ch[0], ch[1] - 1, int(rng.integers(ch[0], ch[1]))}):
                g1, c1, p1, X1, C1 = sampling.one_vertex_problem(hg, v, ch, fx, fc, wl.F, wl.params)
                t0 = time.perf_counter()
                ws.append(odysat.forward(g1, c1, p1, X1, C1, 8)["Y"][:, 0])
                dt += time.perf_counter() - t0
                gs.append(dd.Y[ch[2]:ch[3], v].float().cpu().numpy())
        out["parity"] = parity_numbers(np.stack(gs), np.stack(ws))
        out["parity"]["sampled_vertices"] = len(gs)
        n_rows = int(sum(len(g) for g in gs))
        out["cpu_baseline"] = {"value": n_rows / dt, "unit": "embeddings/s", "cores": torch.get_num_threads(), "kind": "oracle",
                               "cpu": cpu_model(),
                               "sample": f"{len(gs)} vertices, up to three of every one of the {len(wl.chunks)} chunks, forward = "
                                         f"{n_rows} rows, {dt:.1f} s",
                               "gpu_max_rel_err_on_sample": out["parity"]["floor_rms"]}
    elif not args.no_cpu_baseline:
        from oracle import dysat as odysat
        # the oracle (torch CPU, float64, forward + gradients) on the narrowest chunks
        order = np.argsort(wl.chunks[:, 1] - wl.chunks[:, 0])[:2]
        sub = wl.chunks[order]
        t0 = time.perf_counter()
        o = odysat.gradients(wl.graph, sub, wl.params, wl.X, wl.C, 8, target=target)
        dt = time.perf_counter() - t0
        n_rows = int(((sub[:, 1] - sub[:, 0]) * (sub[:, 3] - sub[:, 2])).sum())
        Yg = dd.Y.float().cpu().numpy()
        errs, pars = [], []
        for v_lo, v_hi, t_lo, t_hi in sub.tolist():
            pars.append(parity_numbers(Yg[t_lo:t_hi, v_lo:v_hi], o["Y"][t_lo:t_hi, v_lo:v_hi]))
            errs.append(pars[-1]["floor_rms"])
        out["parity"] = {k: max(p[k] for p in pars) for k in pars[0]}
        out["cpu_baseline"] = {"value": n_rows / dt, "unit": "embeddings/s", "cores": torch.get_num_threads(),
                               "kind": "oracle",
                               "sample": f"the 2 narrowest chunks (of {len(wl.chunks)}), forward + gradients = {n_rows} rows, {dt:.1f} s",
                               "gpu_max_rel_err_on_sample": max(errs)}
    dd.layer.destroy()
    if on_device:
        from workloads import device_gen
        device_gen.release(tgt, dX, dd.Y, wl)
    return out


def cpu_baseline_tfusion(wl, Y_gpu, seed: int) -> dict:
    """Oracle of the temporally fused layer on a seeded sample of vertices of every chunk:
    structure encoder by the C oracle, then every sampled vertex's own sequence."""
    import numpy as np
    import oracle
    from oracle import tfusion
    from workloads import synth
    rng = synth.stream(seed, "bench-sample")
    present = wl.notes["present"]
    sub = [np.sort(rng.choice(int(c[1] - c[0]), size=min(int(c[1] - c[0]), 48), replace=False)) + int(c[0])
           for c in wl.chunks]
    t0 = time.perf_counter()
    Z = oracle.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, time_kind="none", n_struct_layers=1,
                       act_hidden="relu", act_out="none", subset=sub)
    mask = np.zeros(present.shape, np.uint8)
    for c, s in zip(wl.chunks, sub):
        mask[c[2]:c[3], s] = present[c[2]:c[3], s]
    H0 = None if wl.H0 is None else wl.H0.astype(np.float64)
    want = tfusion.run_separate(np.nan_to_num(Z).astype(np.float64), mask, wl.chunks, wl.params, wl.time_kind, H0=H0)
    dt = time.perf_counter() - t0
    m = ~np.isnan(want)
    w = want[m]
    par = parity_numbers(Y_gpu[m], w)
    err = par["floor_1e-1_rms"]
    n_rows = int(m.any(axis=2).sum())
    return {"value": n_rows / dt, "unit": "embeddings/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"48 seeded random vertices of each of the {len(wl.chunks)} chunks, their present snapshots = "
                      f"{n_rows} rows, {dt:.1f} s (structure encoder in C with OpenMP, sequences in NumPy)",
            "gpu_max_rel_err_on_sample": err, "parity": par}


def stale_main(args):
    """The device stale filter (Section 5.2) over the embedding table of config 2: one step = one
    epoch's filter over every (snapshot, vertex) row.  Two embedding tables alternate as the current
    one, so that every step meets the same distances and sends the same rows."""
    import numpy as np
    import torch
    from paper_2309_03523_amd import binding
    from workloads import synth
    R, F = 32 * 100_000, 128
    l1, l_prev = 1.0, 0.5
    t0 = time.perf_counter()
    E, L0 = synth.drifted_copies(args.seed, R, F, kind="triangular")
    t_gen = time.perf_counter() - t0
    factor = binding.stale_theta_factor(l1, l_prev, "printed")
    Ed, Ld, Ad = torch.from_numpy(E).cuda(), torch.from_numpy(L0).cuda(), torch.from_numpy(L0).cuda()
    dist = torch.empty(R, device="cuda")
    send_idx = torch.empty(R, dtype=torch.int64, device="cuda")
    send_buf = torch.empty(R, F, device="cuda")
    result = torch.zeros(24, dtype=torch.uint8, device="cuda")
    ws = torch.empty(binding.stale_workspace_bytes(R), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    kw = dict(factor=factor, dist=dist, send_idx=send_idx, send_buf=send_buf, result=result, workspace=ws, stream=stream)

    binding.stale_filter(Ed, Ld, **kw)                       # first epoch, checked against the oracle below
    torch.cuda.synchronize()
    first = {"res": result.cpu().numpy().view(binding.STALE_RESULT_DTYPE)[0].copy(), "dist": dist.cpu().numpy(),
             "L_new": Ld.cpu().numpy()}
    first["send_idx"] = send_idx.cpu().numpy()[:int(first["res"]["n_send"])]
    tables = [Ad, Ed]                                        # the copies now swing between the two tables

    def step(i):
        binding.stale_filter(tables[i & 1], Ld, **kw)

    for i in range(2 * ((args.warmup + 1) // 2)):
        step(i)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record(stream)
    for i in range(args.steps):
        step(i)
    ev[1].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    dev_ms = ev[0].elapsed_time(ev[1]) / args.steps
    n_send = int(result.cpu().numpy().view(binding.STALE_RESULT_DTYPE)[0]["n_send"])
    assert n_send == int(first["res"]["n_send"]), "the alternating epochs do not send the same rows"
    bytes_per_step = R * (8 * F + 4) + n_send * (12 * F + 8)
    out = {"metric": "embedding rows filtered/s (stale filter)", "value": R * args.steps / elapsed, "unit": "rows/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "stale filter over config 2's embedding table: 3.2 M rows x 128, every row a "
                                  "candidate, drift lengths triangular on [0, 2], threshold factor of the printed "
                                  "equation at l_prev = l_1 / 2", "rows": R, "F": F, "sent_rows": n_send,
                      "theta_factor": factor},
           "roofline": {"kernel": "k_stale_dist + k_stale_count + scan + k_stale_compact (one filter call)",
                        "bound": "hbm", "achieved": bytes_per_step / (dev_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                        "unit": "GB/s", "frac": bytes_per_step / (dev_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                        "traffic": measured_traffic("stale", "in_place").get("filter"),
                        "bytes_per_launch": bytes_per_step, "ms_per_launch": dev_ms},
           "setup_s": {"generate": t_gen}}
    if not args.no_cpu_baseline:
        from oracle import stale
        t0 = time.perf_counter()
        want = stale.stale_filter(E, L0, factor=stale.theta_factor(l1, l_prev))
        t_cpu = time.perf_counter() - t0
        scale = want["D"]
        sure = np.abs(want["dist"] - want["theta"]) > 1e-5 * scale
        sent = np.zeros(R, bool)
        sent[first["send_idx"]] = True
        ok = bool((sent[sure] == (want["dist"] > want["theta"])[sure]).all()) and \
            bool((first["L_new"][first["send_idx"]] == E[first["send_idx"]]).all())
        out["cpu_baseline"] = {"value": R / t_cpu, "unit": "rows/s", "cores": 1, "kind": "oracle",
                               "sample": f"the whole table, first epoch, {t_cpu:.1f} s (NumPy float64)",
                               "gpu_max_rel_err_on_sample": float(np.abs(first["dist"] - want["dist"]).max() / scale),
                               "gpu_decisions_match": ok, "rows_in_rounding_band": int((~sure).sum())}
    print(json.dumps(out))


def fusion_main(args):
    """Spatial-fusion selection (Section 5.1.1) on config 2: one step = the device estimate of the rows
    every pair of the 64 chunks would load twice; the greedy selection under a memory cap follows."""
    import numpy as np
    import torch
    from paper_2309_03523_amd import binding
    from paper_2309_03523_amd.runner import DeviceWorkload
    t0 = time.perf_counter()
    wl, desc = make_workload("config2", args.seed)
    t_gen = time.perf_counter() - t0
    dw = DeviceWorkload(wl)
    layer = dw.layer
    stream = torch.cuda.current_stream()
    S = layer.shared_rows(stream)
    for _ in range(args.warmup):
        layer.shared_rows(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        layer.shared_rows(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = 1e3 * elapsed / args.steps
    rows = wl.graph.T * wl.graph.N
    halo = int(layer.packing("halo_ptr")[-1])
    own = wl.rows
    n = len(wl.chunks)
    pairs = int(np.triu(S).sum())                       # counter increments of the pair kernel
    marks = own + halo                                  # bits set by the marking kernel
    ch = np.asarray(wl.chunks)
    mem = ((ch[:, 1] - ch[:, 0]) * (ch[:, 3] - ch[:, 2])).astype(np.int64) * (wl.F + wl.S + wl.H) * 4
    seg_halo = np.diff(layer.packing("halo_ptr"))
    win = ch[:, 3] - ch[:, 2]
    mem += np.add.reduceat(seg_halo, np.concatenate([[0], np.cumsum(win)[:-1]])) * wl.F * 4
    cap = int(mem.sum() // 8)
    t0 = time.perf_counter()
    grp = binding.fusion_select(S, mem, cap)
    t_sel = time.perf_counter() - t0
    saved = int(sum(S[a, b] for a in range(n) for b in range(a + 1, n) if grp[a] == grp[b]))
    # LDS integer atomics: 32 banks x one atomic per clock x 256 CUs x 2.4 GHz
    peak = 256 * 32 * 2.4
    out = {"metric": "(snapshot, vertex) rows scanned/s (redundant-loading estimate between chunks)",
           "value": rows * args.steps / elapsed, "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64",
           "data": "synthetic",
           "config": {"workload": "spatial-fusion selection on " + desc, "chunks": n, "rows": rows,
                      "halo_entries": halo, "pair_increments": pairs},
           "roofline": {"kernel": "k_fs_pairs<true> (+ k_fs_zero, k_fs_mark; whole call incl. the 32 KB read-back)",
                        "bound": "alu", "achieved": pairs / (ms * 1e-3) / 1e9, "peak": peak, "unit": "Gatomic/s",
                        "frac": pairs / (ms * 1e-3) / 1e9 / peak, "traffic": None,
                        "ops_per_launch": pairs, "ms_per_launch": ms,
                        "hbm_bytes_algorithmic": marks * 8 + halo * 4 + rows * 8 * 2},
           "selection": {"cap_bytes": cap, "groups": int(grp.max()) + 1, "largest_group_bytes": int(np.bincount(grp, weights=mem).max()),
                         "rows_loaded_once_instead_of_twice": saved, "of_all_shared": pairs, "select_s": t_sel},
           "setup_s": {"generate": t_gen}}
    if not args.no_cpu_baseline:
        from oracle import fusion
        k = 16
        t0 = time.perf_counter()
        want = fusion.shared_rows(wl.graph, wl.chunks[:k])
        t_cpu = time.perf_counter() - t0
        sample_rows = int(sum((c[1] - c[0]) * (c[3] - c[2]) for c in ch[:k]))
        out["cpu_baseline"] = {"value": sample_rows / t_cpu, "unit": "rows/s", "cores": 1, "kind": "oracle",
                               "sample": f"load sets and pairwise intersections of the first {k} chunks ({sample_rows} "
                                         f"own rows), {t_cpu:.1f} s (Python sets)",
                               "gpu_matches_bit_exact": bool((S[:k, :k] == want).all())}
    print(json.dumps(out))


def labelled_main(args):
    """Config 2 with GENERATED chunks (Sections 4.1, 5.2): the device label propagation partitions
    the (snapshot, vertex) pairs, the layer runs over those chunks - a neighbour with another
    label is read from the cache, a vertex whose previous snapshot carries another label starts
    from the state cache, states that leave a chunk are written out.  One step = one forward."""
    import numpy as np
    import torch
    from paper_2309_03523_amd import binding
    from workloads import synth
    from paper_2309_03523_amd.runner import DeviceWorkload
    synth.progress = lambda msg: print(msg, file=sys.stderr, flush=True)
    w_s, w_t, cap, max_iters = 1, 1, 50_000, 1000        # one structure layer : one time layer; config 2's mean chunk size
    t0 = time.perf_counter()
    wl = synth.config2(args.seed)
    rect = wl.chunks
    g = wl.graph
    T, N = g.T, g.N
    wl.chunks = np.array([[0, N, 0, T]], np.int64)
    wl.H0 = None
    Hc_host = synth.stream(args.seed, "state-cache").standard_normal(size=(T * N, wl.H), dtype=np.float32) * np.float32(0.1)
    t_gen = time.perf_counter() - t0
    t0 = time.perf_counter()
    dw = DeviceWorkload(wl, gather_mode="in_place")
    layer = dw.layer
    torch.cuda.synchronize()
    t_create = time.perf_counter() - t0
    labels = torch.empty(T * N, dtype=torch.int32, device="cuda")
    t0 = time.perf_counter()
    iters, conv = binding.chunk_generate(dw.rowptr, dw.colidx, N, w_s=w_s, w_t=w_t, cap=cap, max_iters=max_iters, labels=labels)
    torch.cuda.synchronize()
    t_labels = time.perf_counter() - t0
    t0 = time.perf_counter()
    layer.set_labels(labels)
    t_tables = time.perf_counter() - t0
    present = None
    t_lanes = 0.0
    if getattr(args, "presence", False):
        present = synth.presence(args.seed, T, N)
        p_dev = torch.from_numpy(present).cuda()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        layer.set_presence(p_dev)
        t_lanes = time.perf_counter() - t0
        dw.Y.fill_(float("nan"))
    Hc = torch.from_numpy(Hc_host).cuda()
    HN = torch.full((T * N, wl.H), float("nan"), dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        layer.forward(dw.X, dw.C, dw.Y, H0=Hc, HN=HN, stream=stream)

    for _ in range(args.warmup):
        step()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(stream)
    for k in range(args.steps):
        step()
        marks[k + 1].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per = np.array([marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)])
    layer.set_profiling(True)
    stage = np.zeros(13, np.float64)
    for _ in range(3):
        step()
        stage += layer.stage_times()
    stage /= 3
    layer.set_profiling(False)
    rows = T * N if present is None else int(present.sum())
    ms = 1e3 * elapsed / args.steps
    # what the partition costs: neighbours and temporal neighbours read from the caches
    lab = labels.cpu().numpy().reshape(T, N)
    rect_lab = np.zeros((T, N), np.int32)
    for k, (a, b, t_lo, t_hi) in enumerate(rect.tolist()):
        rect_lab[t_lo:t_hi, a:b] = k

    def cut(l):
        stale_e = sum(int((l[t][np.repeat(np.arange(N), np.diff(sn.rowptr))] != l[t][sn.col]).sum()) for t, sn in enumerate(g.snaps))
        stale_t = N + int((l[1:] != l[:-1]).sum())
        return stale_e, stale_t

    se, st_ = cut(lab)
    re_, rt = cut(rect_lab)
    nnz = g.nnz
    sizes = np.bincount(lab.reshape(-1))
    sizes = sizes[sizes > 0]
    fl = flops_per_row(wl)
    n_lanes = int(layer.packing("lane_ptr")[-1]) if present is not None else 0
    dense_rows = rows if present is None else n_lanes * T           # the kernel computes every lane slot
    dense_flops = (fl["transform"] + fl["rnn"]) * dense_rows
    dense_ms, agg_ms = float(stage[3]), float(stage[0])
    achieved = dense_flops / (dense_ms * 1e-3) / 1e12
    if present is not None:
        deg = [np.diff(sn.rowptr) for sn in g.snaps]
        nnz = int(sum(int(d[present[t].astype(bool)].sum()) for t, d in enumerate(deg)))     # non-zeros of the rows computed
    agg_bytes = rows * (wl.F * 4) + nnz * 4 + rows * 8 + rows * (wl.F * 4)
    traffic = measured_traffic("config2lp", "in_place") if present is None else {}
    out = {"metric": "snapshot-vertex embeddings/s per DGNN layer", "value": rows * args.steps / elapsed, "unit": "embeddings/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": "config2 (32 snapshots x 100k vertices, F=S=H=128, GCN+GRU) over chunks generated by the "
                                  f"device label propagation (w_spatial = {w_s}, w_temporal = {w_t}, size limit {cap})" +
                                  ("" if present is None else
                                   f" with config2tf's presence matrix: temporal fusion over the generated chunks, {n_lanes} lanes of {T} "
                                   f"slots for {rows} present rows ({rows / max(1, n_lanes * T):.1%} of the slots filled); value counts present rows"),
                      "rows": rows, "nnz": nnz, "gather_mode": "in_place", "pass": "forward"},
           "roofline": {"kernel": "k_dense_wave<GRU, SEQ> (GCN transform + time encoder over every vertex's label runs)",
                        "bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                        "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic.get("dense"),
                        "flops_per_launch": dense_flops, "ms_per_launch": dense_ms},
           "roofline_aggregation": {"kernel": "k_spmm_short + k_spmm_long + k_spmm_long_reduce (pre-marked columns)",
                                    "bound": "hbm", "achieved": agg_bytes / (agg_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS,
                                    "unit": "GB/s", "frac": agg_bytes / (agg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                    "traffic": traffic.get("aggregation"), "bytes_per_launch": agg_bytes,
                                    "ms_per_launch": agg_ms, "gather_traffic_GBs": nnz * wl.F * 4 / (agg_ms * 1e-3) / 1e9},
           "stage_ms": {"aggregate0": agg_ms, "dense_rnn": dense_ms},
           "device_ms_per_step": {"median": float(np.median(per)), "min": float(per.min()), "max": float(per.max())},
           "chunks": {"count": int(sizes.size), "largest": int(sizes.max()), "median": float(np.median(sizes)),
                      "iterations": iters, "converged": bool(conv),
                      "stale_neighbour_reads": se, "stale_neighbour_fraction": se / nnz,
                      "stale_state_reads": st_, "stale_state_fraction": st_ / rows,
                      "rectangular_64_chunks": {"stale_neighbour_fraction": re_ / nnz, "stale_state_fraction": rt / rows}},
           "setup_s": {"generate": t_gen, "upload_create_pack": t_create, "label_propagation": t_labels,
                       "label_tables": t_tables, "lanes": t_lanes}}
    if not args.no_cpu_baseline:
        from oracle import labelled
        rng = synth.stream(args.seed, "bench-sample")
        Y_gpu = dw.Y.cpu().numpy()
        n_v, done, dt, errs, pars = 16, 0, 0.0, [], []
        while dt < 12.0 and done < 4096:      # growing seeded samples of vertices, all 32 snapshots each
            vs = np.sort(rng.choice(N, size=n_v, replace=False))
            t0 = time.perf_counter()
            want, _ = labelled.forward(g, lab, wl.params, wl.X, wl.C, time_kind=wl.time_kind, Hc=Hc_host, vertices=vs,
                                       present=present)
            dt += time.perf_counter() - t0
            done += n_v
            got = Y_gpu[:, vs]
            if present is not None:
                here = present[:, vs].astype(bool)
                assert np.array_equal(np.isnan(got).any(-1), ~here) and np.array_equal(np.isnan(want).any(-1), ~here)
                got, want = got[here], want[here]
            pars.append(parity_numbers(got, want))
            errs.append(pars[-1]["floor_1e-1_rms"])
            n_v = min(2 * n_v, 1024)
        out["cpu_baseline"] = {"value": done * T / dt, "unit": "embeddings/s", "cores": 1, "kind": "oracle",
                               "sample": f"{done} seeded random vertices, all {T} snapshots = {done * T} rows, {dt:.1f} s "
                                         "(plain Python / NumPy loops over rows and edges)",
                               "gpu_max_rel_err_on_sample": max(errs),
                               "parity": {k: max(p[k] for p in pars) for k in pars[0]}}
    print(json.dumps(out))


def chunkgen_main(args):
    """Chunk generation by weighted label propagation (Section 4.1) on config 2's graph: one step =
    one whole generation (all iterations until no label changes)."""
    import numpy as np
    import torch
    from paper_2309_03523_amd import binding
    from workloads import synth
    synth.progress = lambda msg: print(msg, file=sys.stderr, flush=True)
    w_s, w_t, cap, max_iters = 2, 1, 25_000 * 8, 1000     # two structure layers : one time layer; chunks of config 2's size
    t0 = time.perf_counter()
    g = synth.config2_graph(args.seed)
    t_gen = time.perf_counter() - t0
    rp = [torch.from_numpy(s.rowptr).cuda() for s in g.snaps]
    ci = [torch.from_numpy(s.col).cuda() for s in g.snaps]
    n = g.T * g.N
    labels = torch.empty(n, dtype=torch.int32, device="cuda")
    kw = dict(w_s=w_s, w_t=w_t, cap=cap, max_iters=max_iters, labels=labels)
    for _ in range(min(args.warmup, 1)):
        binding.chunk_generate(rp, ci, g.N, **kw)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        iters, conv = binding.chunk_generate(rp, ci, g.N, **kw)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms = 1e3 * elapsed / args.steps
    edges = g.nnz - n + 2 * (g.T - 1) * g.N               # directed super-graph edges
    lab = labels.cpu().numpy()
    sizes = np.bincount(lab, minlength=n)
    sizes = sizes[sizes > 0]
    # weight inside chunks / total weight (each undirected edge once), on the host from the labels
    inside = 0
    for t, sn in enumerate(g.snaps):
        row = np.repeat(np.arange(g.N, dtype=np.int64), np.diff(sn.rowptr))
        l = lab[t * g.N:(t + 1) * g.N]
        inside += w_s * (int((l[row] == l[sn.col]).sum()) - g.N) // 2
        if t + 1 < g.T:
            inside += w_t * int((l == lab[(t + 1) * g.N:(t + 2) * g.N]).sum())
    total = w_s * (g.nnz - n) // 2 + w_t * (g.T - 1) * g.N
    bytes_iter = 4 * g.nnz + 24 * n
    out = {"metric": "super-graph edge visits/s (label propagation, all iterations of one chunk generation)",
           "value": edges * iters * args.steps / elapsed, "unit": "edges/s", "n_gpus": 1, "steps": args.steps,
           "warmup": min(args.warmup, 1), "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "i32", "data": "synthetic",
           "config": {"workload": "chunk generation on config 2's graph: 32 snapshots x 100k vertices, "
                                  f"w_spatial = {w_s}, w_temporal = {w_t}, size limit {cap}", "super_vertices": n,
                      "directed_edges": edges, "iterations": iters, "converged": conv},
           "roofline": {"kernel": "k_cg_propose_short + k_cg_propose_long + k_cg_decide_short + k_cg_decide_long, per iteration",
                        "bound": "hbm", "achieved": bytes_iter * iters / (ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": bytes_iter * iters / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                        "traffic": measured_traffic("chunkgen", "in_place").get("iteration"),
                        "bytes_per_launch": bytes_iter, "ms_per_launch": ms / iters},
           "chunks": {"count": int(sizes.size), "largest": int(sizes.max()), "median": float(np.median(sizes)),
                      "weight_inside_chunks": inside, "total_weight": total, "inside_fraction": inside / total},
           "setup_s": {"generate": t_gen}}
    if not args.no_cpu_baseline:
        from oracle import chunkgen
        small = synth.config2_graph(args.seed, scale=0.003)
        srp = [torch.from_numpy(s.rowptr).cuda() for s in small.snaps]
        sci = [torch.from_numpy(s.col).cuda() for s in small.snaps]
        slab = torch.empty(small.T * small.N, dtype=torch.int32, device="cuda")
        s_it, s_conv = binding.chunk_generate(srp, sci, small.N, w_s=w_s, w_t=w_t, cap=cap // 333, max_iters=max_iters, labels=slab)
        t0 = time.perf_counter()
        want = chunkgen.propagate(small, w_s, w_t, cap // 333, max_iters)
        t_cpu = time.perf_counter() - t0
        s_edges = small.nnz - small.T * small.N + 2 * (small.T - 1) * small.N
        out["cpu_baseline"] = {"value": s_edges * want["iterations"] / t_cpu, "unit": "edges/s", "cores": 1, "kind": "oracle",
                               "sample": f"the same generator at 3/1000 of the vertex count ({small.T * small.N} super-vertices, "
                                         f"{want['iterations']} iterations), {t_cpu:.1f} s (Python loops)",
                               "gpu_matches_bit_exact": bool((slab.cpu().numpy() == want["labels"]).all()
                                                             and s_it == want["iterations"] and s_conv == want["converged"])}
    print(json.dumps(out))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (chunks would shard across GPUs by chunk "
              "assignment; no collective is built). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    own_line = {"chunkgen": chunkgen_main, "config2lp": labelled_main, "stale": stale_main, "fusion": fusion_main}
    if args.workload in own_line:
        own_line[args.workload](args)
        return
    if args.workload.startswith("config5"):
        out = dysat_run(args)
    elif args.workload == "config3":
        out = config3_run(args)
    else:
        out = gcn_run(args)
        if args.workload == "config2" and not args.no_configs:
            out["configs"] = other_configs(args)
    print(json.dumps(out))


def gcn_run(args) -> dict:
    """One workload of the GCN + recurrent (or EvolveGCN-O) layer: generate, create, time, report."""
    import numpy as np
    import torch
    from paper_2309_03523_amd.runner import DeviceWorkload

    t0 = time.perf_counter()
    wl, desc = make_workload(args.workload, args.seed)
    t_gen = time.perf_counter() - t0
    rows = wl.rows
    on_device = bool(getattr(wl, "on_device", False))

    t0 = time.perf_counter()
    evolve = "evolve.W_init" in wl.params
    dw = DeviceWorkload(wl, gather_mode=args.gather_mode, act_hidden="relu", agg_kernel=args.agg_kernel,
                        act_out="relu" if evolve else "none", struct_kind="evolve_gcn_o" if evolve else "gcn")
    if evolve:
        print("upload target ...", file=sys.stderr, flush=True)
    target = None
    if evolve:
        target = wl.notes["target"] if on_device else torch.from_numpy(wl.notes["target"]).cuda()
    loss = torch.zeros(1, device="cuda") if evolve else None
    torch.cuda.synchronize()
    t_create = time.perf_counter() - t0
    layer = dw.layer
    stream = torch.cuda.current_stream()
    tfuse = None
    if "present" in wl.notes:
        present = wl.notes["present"]
        t0 = time.perf_counter()
        layer.set_presence(torch.from_numpy(present).cuda())
        cov = np.zeros(present.shape, bool)
        for v_lo, v_hi, t_lo, t_hi in wl.chunks.tolist():
            cov[t_lo:t_hi, v_lo:v_hi] = True
        padded_rows = rows
        rows = int((present.astype(bool) & cov).sum())       # embeddings actually produced
        n_lanes = int(layer.packing("lane_ptr")[-1])
        window = int((wl.chunks[:, 3] - wl.chunks[:, 2]).max())
        live = present.astype(bool) & cov
        nnz_present = int(sum(int(np.diff(sn.rowptr)[live[t]].sum()) for t, sn in enumerate(wl.graph.snaps)))
        tfuse = {"present_rows": rows, "padded_rows": padded_rows, "nnz_present_rows": nnz_present, "lanes": n_lanes,
                 "lane_slots": n_lanes * window, "lane_fill": rows / max(1, n_lanes * window),
                 "pack_s": time.perf_counter() - t0}

    dX = torch.empty_like(dw.X) if (evolve and args.with_dx) else None

    def step():
        layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=dw.H0, stream=stream)
        if evolve:
            layer.backward(dw.Y, target=target, loss_out=loss, dX=dX, stream=stream)

    if args.calib_copy:
        scratch = torch.empty_like(dw.X)
        scratch.copy_(dw.X)
        torch.cuda.synchronize()
        print(f"calib-copy: {dw.X.numel() * 4} bytes read and as many written", file=sys.stderr)
        del scratch
    # measured HBM ceiling next to the published one: a plain device copy of X (read + write)
    copy_GBs = None
    if dw.X.numel() * dw.X.element_size() >= (1 << 28) and not evolve and not on_device:
        scratch = torch.empty_like(dw.X)
        scratch.copy_(dw.X)
        cm = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        cm[0].record(stream)
        for _ in range(5):
            scratch.copy_(dw.X)
        cm[1].record(stream)
        torch.cuda.synchronize()
        copy_GBs = 5 * 2 * dw.X.numel() * dw.X.element_size() / (cm[0].elapsed_time(cm[1]) * 1e-3) / 1e9
        del scratch
    for _ in range(args.warmup):
        step()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # per-step device times
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record(stream)
    for k in range(args.steps):
        step()
        marks[k + 1].record(stream)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    value = rows * args.steps / elapsed
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    step_stats = {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1]}

    # the launch-bound small configuration also as a captured HIP graph: forward only enqueues kernels,
    # so the caller can record it once and replay it
    graph_ms = None
    if args.workload in ("config1", "config4s"):
        # (config4s: its weight recurrence is some 330 small dependent launches per step)
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        hip_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(hip_graph, stream=side):
            layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=dw.H0)
            if evolve:
                layer.backward(dw.Y, target=target, loss_out=loss, dX=dX)
        for _ in range(args.warmup):
            hip_graph.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            hip_graph.replay()
        torch.cuda.synchronize()
        graph_ms = 1e3 * (time.perf_counter() - tg) / args.steps

    # per-stage device times of the same launches, HIP events on the launch stream
    layer.set_profiling(True)
    stage = np.zeros(13, np.float64)
    n_prof = max(3, min(args.steps, 10))
    for _ in range(n_prof):
        step()
        stage += layer.stage_times()
    stage /= n_prof
    layer.set_profiling(False)

    packing = {"create_ms": 1e3 * dw.create_s,
               "step_plus_packing_over_one_epoch_ms": ms_per_step + 1e3 * dw.create_s,
               "step_plus_packing_over_100_epochs_ms": ms_per_step + 10.0 * dw.create_s,
               "note": "wall time of dgc_layer_create (validation, chunk-fusion packing kernels, workspace allocation; "
                       "it synchronises); the paper partitions once per job and trains 100 epochs"}
    if evolve:
        out = evolve_report(args, wl, desc, dw, rows, value, ms_per_step, stage, t_gen, t_create, loss, graph_ms, dX)
        out["packing"] = packing
        if on_device:
            from workloads import device_gen
            device_gen.release(dw, dX, wl)
        return out
    fl = flops_per_row(wl)
    # the last dense launch: last GCN layer's transform + time encoder
    dense_rows = tfuse["lane_slots"] if tfuse else rows     # the kernel also computes the empty slots
    dense_flops = (fl["transform"] + fl["rnn"]) * dense_rows if wl.n_struct_layers == 1 else \
        (2 * wl.S * wl.S + fl["rnn"]) * dense_rows
    dense_ms = float(stage[3])
    achieved = dense_flops / (dense_ms * 1e-3) / 1e12
    traffic = measured_traffic(args.workload, args.gather_mode)
    roofline = {"kernel": "k_dense_wave / k_dense (GCN transform + time encoder, fused over the window)",
                "bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic.get("dense"),
                "flops_per_launch": dense_flops, "ms_per_launch": dense_ms}
    # aggregation kernels: algorithmic (compulsory) bytes = X rows once + CSR + M written once
    nnz = int(layer.packing("seg_nnz_off")[-1])
    if tfuse:
        # only the rows of present vertices are aggregated (and written, in lane order); every
        # row of X can still be somebody's neighbour
        nnz_agg = tfuse["nnz_present_rows"]
        agg_bytes = tfuse["padded_rows"] * (wl.F * 4) + nnz_agg * 4 + rows * 8 + rows * (wl.F * 4)
    else:
        nnz_agg = nnz
        agg_bytes = rows * (wl.F * 4) + nnz * 4 + rows * 8 + rows * (wl.F * 4)
    agg_ms = float(stage[0])
    agg = {"kernel": AGG_KERNELS[args.agg_kernel], "bound": "hbm",
           "achieved": agg_bytes / (agg_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
           "frac": agg_bytes / (agg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
           "traffic": traffic.get("aggregation") if args.agg_kernel == "table" else None,     # the counters were taken on the default kernels
           "bytes_per_launch": agg_bytes, "ms_per_launch": agg_ms,
           "gather_traffic_GBs": nnz_agg * wl.F * 4 / (agg_ms * 1e-3) / 1e9, "nnz": nnz_agg}

    out = {"metric": "snapshot-vertex embeddings/s per DGNN layer", "value": value, "unit": "embeddings/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
           "data": "synthetic",
           "config": {"workload": desc, "rows": rows, "nnz": nnz, "gather_mode": args.gather_mode,
                      "agg_kernel": args.agg_kernel, "pass": "forward"},
           "roofline": with_traffic_rate(roofline), "roofline_aggregation": with_traffic_rate(agg),
           "stage_ms": ({"aggregate0": float(stage[0]), "dense_rnn": float(stage[3])} if wl.n_struct_layers == 1 else
                        {"aggregate0": float(stage[0]), "dense0": float(stage[1]), "aggregate1": float(stage[2]),
                         "dense_rnn": float(stage[3])}),
           "device_ms_per_step": step_stats, "measured_hbm_copy_GBs": copy_GBs, "packing": packing,
           "setup_s": {"generate": t_gen, "upload_create_pack": t_create}}
    if graph_ms is not None:
        out["hip_graph_replay_ms_per_step"] = graph_ms
    if tfuse:
        out["temporal_fusion"] = tfuse
        out["roofline"]["kernel"] += " over the lanes, every slot's output stored straight to its row"
    if not args.no_cpu_baseline:
        Y_gpu = dw.Y.cpu().numpy()
        if tfuse:
            out["cpu_baseline"] = cpu_baseline_tfusion(wl, Y_gpu, args.seed)
        else:
            out["cpu_baseline"] = cpu_baseline(wl, Y_gpu, args.cpu_seconds, args.seed)
        out["parity"] = out["cpu_baseline"].get("parity")
    dw.layer.destroy()
    return out


def config3_run(args) -> dict:
    """Config 3 at its stated size: 2,000,000 vertices x 128 snapshots do not fit the GPU at once, so
    the 256 chunks run as four fused batches of 64, one per 32-snapshot window (the memory-capped
    fusion of Section 5.1.1), each drawn on the device, run, sampled against the oracle and released.
    A step = one forward over every listed window; times are summed over the windows."""
    import numpy as np
    import torch
    from oracle import sampled
    from paper_2309_03523_amd.runner import DeviceWorkload
    from workloads import device_gen, sampling, synth

    def say(msg):
        print(msg, file=sys.stderr, flush=True)

    windows = [int(x) for x in args.windows.split(",") if x != ""]
    stream = torch.cuda.current_stream()
    tot = {"rows": 0, "nnz": 0, "elapsed": 0.0, "gen": 0.0, "create": 0.0}
    stage_sum = np.zeros(13, np.float64)
    per_window, pars, base_rows, base_dt = [], [], 0, 0.0
    for w in windows:
        device_gen.release()
        t0 = time.perf_counter()
        full = bool(getattr(args, "mpnn_lstm", False))
        data = device_gen.config3_window(args.seed, 1.0, window=w, say=say, input_concat=full, n_time_layers=2 if full else 1)
        torch.cuda.synchronize()
        t_gen = time.perf_counter() - t0
        dw = DeviceWorkload(data, gather_mode=args.gather_mode, act_hidden="relu", act_out="none", agg_kernel=args.agg_kernel,
                            n_time_layers=2 if full else 1)
        layer = dw.layer

        def step():
            layer.forward(dw.X, dw.C, dw.Y, C1=dw.C1, H0=dw.H0, stream=stream)

        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        layer.set_profiling(True)
        stage = np.zeros(13, np.float64)
        n_prof = max(2, min(args.steps, 5))
        for _ in range(n_prof):
            step()
            stage += layer.stage_times()
        stage /= n_prof
        layer.set_profiling(False)
        rows, nnz = data.rows, data.nnz
        win = {"window": w, "rows": rows, "nnz": nnz, "ms_per_step": 1e3 * elapsed / args.steps,
               "generate_s": t_gen, "create_ms": 1e3 * dw.create_s,
               "stage_ms": {"aggregate0": float(stage[0]), "dense0": float(stage[1]), "aggregate1": float(stage[2]),
                            "dense_rnn": float(stage[3])}}
        if not args.no_cpu_baseline:
            say(f"window {w}: oracle on sampled vertices ...")
            hg = data.host_graph()
            rng = synth.stream(args.seed, f"bench-sample-{w}")
            ids = sampling.pick_chunks(hg, data.chunks, 4, rng)
            subsets = [sampling.pick_vertices(hg, data.chunks[k], 5, rng) for k in ids]
            want, where, dt = sampled.two_layer_reference(data, hg, ids, subsets, input_concat=full,
                                                          n_time_layers=2 if full else 1)
            got = sampled.device_rows(dw.Y, data.chunks, where, data.H)
            win["parity"] = parity_numbers(got, want)
            win["parity"]["sampled_vertices"] = int(len(where))
            win["parity"]["sampled_chunks"] = ids
            pars.append(win["parity"])
            base_rows += int(len(where)) * 32
            base_dt += dt
            del hg
        per_window.append(win)
        tot["rows"] += rows
        tot["nnz"] += nnz
        tot["elapsed"] += elapsed
        tot["gen"] += t_gen
        tot["create"] += dw.create_s
        stage_sum += stage
        device_gen.release(dw, data)
    F, S, H = 172, 128, 128
    rows = tot["rows"]
    full = bool(getattr(args, "mpnn_lstm", False))
    dense_flops = (2 * S * S + 2 * (2 * S if full else S) * 4 * H + 2 * H * 4 * H + (4 * H * 4 * H if full else 0)) * rows
    dense_ms = float(stage_sum[3])
    ach = dense_flops / (dense_ms * 1e-3) / 1e12
    traffic = measured_traffic("config3_mpnn_lstm" if full else "config3", args.gather_mode)     # per window
    roofline = {"kernel": "k_dense_wave<LSTM> (second GCN transform + LSTM, fused over the window" +
                          (", and the second LSTM layer's launch)" if full else ")"), "bound": "mfma",
                "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s", "frac": ach / PEAK_FP32_MFMA_TFLOPS,
                "traffic": traffic.get("dense"), "flops_per_launch": dense_flops / len(windows),
                "ms_per_launch": dense_ms / len(windows)}
    first_flops = 2 * F * S * rows
    agg_bytes = rows * (F * 4) * 2 + rows * (S * 4) * 2 + 2 * (tot["nnz"] * 4 + rows * 8)
    agg_ms = float(stage_sum[0] + stage_sum[2])
    ms_per_step = 1e3 * tot["elapsed"] / args.steps
    out = {"metric": "snapshot-vertex embeddings/s per DGNN layer", "value": rows * args.steps / tot["elapsed"],
           "unit": "embeddings/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": f"config3 at its stated size: 2,000,000 vertices, windows {windows} of the four 32-snapshot "
                                  "windows, each one fused batch of 64 uneven chunks; 2 GCN layers (172->128->128) + " +
                                  ("2 stacked LSTM layers, the first reading both GCN outputs (the paper's MPNN-LSTM); " if full else "LSTM; ") +
                                  "inputs drawn on the device" +
                                  ("" if len(windows) == 4 else f"; the whole config is 4 windows: x {4 / len(windows):g}"),
                      "rows": rows, "nnz": tot["nnz"], "gather_mode": args.gather_mode, "pass": "forward"},
           "roofline": roofline,
           "kernels": {"first_transform": {"kernel": "k_dense_wave<NONE> (first GCN layer, 172 -> 128)", "bound": "mfma",
                                           "achieved": first_flops / (float(stage_sum[1]) * 1e-3) / 1e12,
                                           "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                                           "frac": first_flops / (float(stage_sum[1]) * 1e-3) / 1e12 / PEAK_FP32_MFMA_TFLOPS,
                                           "ms": float(stage_sum[1])}},
           "roofline_aggregation": {"kernel": AGG_KERNELS[args.agg_kernel] + " of both GCN layers, all windows of the step", "bound": "hbm",
                                    "achieved": agg_bytes / (agg_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                    "frac": agg_bytes / (agg_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                    "traffic": (len(windows) * (traffic["aggregation"] + traffic["aggregation_second_layer"])
                                                if "aggregation" in traffic and args.agg_kernel == "table" else None),
                                    "bytes_per_step": agg_bytes, "ms": agg_ms,
                                    "gather_traffic_GBs": tot["nnz"] * (F + S) * 4 / (agg_ms * 1e-3) / 1e9},
           "stage_ms": {"aggregate0": float(stage_sum[0]), "dense0": float(stage_sum[1]),
                        "aggregate1": float(stage_sum[2]), "dense_rnn": float(stage_sum[3])},
           "windows": per_window,
           "packing": {"create_ms": 1e3 * tot["create"],
                       "step_plus_packing_over_one_epoch_ms": ms_per_step + 1e3 * tot["create"],
                       "step_plus_packing_over_100_epochs_ms": ms_per_step + 10.0 * tot["create"]},
           "setup_s": {"generate": tot["gen"], "upload_create_pack": tot["create"]}}
    if pars:
        import oracle
        out["parity"] = {k: max(p[k] for p in pars) for k in pars[0] if k not in ("sampled_chunks",)}
        out["parity"]["sampled_vertices"] = sum(p["sampled_vertices"] for p in pars)
        out["cpu_baseline"] = {"value": base_rows / base_dt, "unit": "embeddings/s", "cores": oracle.threads(),
                               "kind": "oracle", "cpu": cpu_model(),
                               "sample": f"8 vertices of each of 8 chunks per window (first, last, densest, the hub's, four "
                                         f"random) = {base_rows} rows, {base_dt:.1f} s; a sampled row also evaluates the "
                                         "first-layer rows of all its neighbours",
                               "gpu_max_rel_err_on_sample": out["parity"]["floor_1e-1_rms"]}
    return out


def other_configs(args) -> dict:
    """Configurations 1, 3 (one window), 4 and 5 at their stated sizes, a few steps each, for the
    `configs` object of the default line: step time, throughput, dominant kernel, sampled parity."""
    import argparse as _ap
    out = {}
    plan = [("config1", gcn_run, {}), ("config3", config3_run, {"windows": "1"}), ("config4", gcn_run, {"with_dx": False}),
            ("config5", dysat_run, {})]
    for name, fn, extra in plan:
        a = _ap.Namespace(**{**vars(args), "workload": name, "steps": args.config_steps, "warmup": 2,
                             "cpu_seconds": 5.0, "no_configs": True, **extra})
        t0 = time.perf_counter()
        try:
            from workloads import device_gen
            device_gen.release()
            r = fn(a)
            dom = r.get("roofline", {})
            out[name] = {"workload": r["config"]["workload"], "pass": r["config"].get("pass"), "rows": r["config"]["rows"],
                         "ms_per_step": r["ms_per_step"], "value": r["value"], "unit": r["unit"], "dtype": r["dtype"],
                         "dominant_kernel": {k: dom.get(k) for k in ("kernel", "bound", "achieved", "peak", "unit", "frac")},
                         "stage_ms": r.get("stage_ms"), "parity": r.get("parity"),
                         "cpu_baseline": {k: v for k, v in (r.get("cpu_baseline") or {}).items() if k != "parity"},
                         "wall_s": time.perf_counter() - t0}
        except Exception as e:      # an extra configuration must never take the headline line down
            out[name] = {"error": f"{type(e).__name__}: {e}"[:400], "wall_s": time.perf_counter() - t0}
            print(f"configs[{name}] failed: {e}", file=sys.stderr, flush=True)
    return out


if __name__ == "__main__":
    main()
