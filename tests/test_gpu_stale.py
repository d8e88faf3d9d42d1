"""The device stale filter (Section 5.2) against the oracle: distances and the threshold within
fp32 rounding, the decision exact for every row whose distance is not within rounding of the
threshold, the send list ascending, the message and the updated copies bit for bit."""
import numpy as np
import pytest

from oracle import stale
from workloads import synth

pytestmark = pytest.mark.gpu

DIST_TOL = 2e-6     # relative, fp32 sum of F <= 512 squared differences against float64
BAND = 1e-5         # rows this close (relative) to the threshold may fall either way


def _device_filter(E, L, ld, rows, factor, theta, with_buf=True, bf16=False):
    import torch
    from paper_2309_03523_amd import binding
    R, F = E.shape
    dt = torch.bfloat16 if bf16 else torch.float32      # bf16: E and L hold bf16-representable values already
    Ed = torch.full((R, ld), float("nan"), device="cuda", dtype=dt)
    Ld = torch.full((R, ld), float("nan"), device="cuda", dtype=dt)
    Ed[:, :F] = torch.from_numpy(E).cuda().to(dt)
    Ld[:, :F] = torch.from_numpy(L).cuda().to(dt)
    rd = None if rows is None else torch.from_numpy(rows).cuda()
    if rows is not None and rows.size == 0:     # an empty list is still a list: keep its pointer non-NULL
        rd = torch.zeros(1, dtype=torch.int64, device="cuda")
    n = R if rows is None else rows.size
    dist = torch.full((max(n, 1),), -1.0, device="cuda")
    send_idx = torch.full((max(n, 1),), -7, dtype=torch.int64, device="cuda")
    send_buf = torch.full((max(n, 1), ld), float("nan"), device="cuda", dtype=dt) if with_buf else None
    result = torch.zeros(24, dtype=torch.uint8, device="cuda")
    ws = torch.empty(binding.stale_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    binding.stale_filter(Ed, Ld, F=F, rows=rd, n_rows=None if rows is None else rows.size, factor=factor, theta=theta, dist=dist, send_idx=send_idx,
                         send_buf=send_buf, result=result, workspace=ws)
    torch.cuda.synchronize()
    res = result.cpu().numpy().view(binding.STALE_RESULT_DTYPE)[0]
    k = int(res["n_send"])
    return {"dist": dist.cpu().numpy()[:n], "send_idx": send_idx.cpu().numpy()[:k],
            "send_buf": None if send_buf is None else send_buf.float().cpu().numpy()[:k, :F],
            "L_new": Ld.float().cpu().numpy()[:, :F], "pad": Ld.float().cpu().numpy()[:, F:], "res": res,
            "tail_idx": send_idx.cpu().numpy()[k:n]}


def _check(E, L, rows, factor, theta, got):
    want = stale.stale_filter(E, L, factor=factor, theta=theta, rows=rows)
    cand = np.arange(E.shape[0]) if rows is None else rows
    scale = max(want["D"], 1e-30)
    assert np.abs(got["dist"] - want["dist"]).max() <= DIST_TOL * scale
    assert abs(float(got["res"]["D"]) - want["D"]) <= DIST_TOL * scale
    th = float(got["res"]["theta"])
    assert abs(th - want["theta"]) <= DIST_TOL * max(want["theta"], scale)
    assert int(got["res"]["n_invalid"]) == 0
    # the decision: exact outside the rounding band around the threshold, valid inside it
    sure = np.abs(want["dist"] - want["theta"]) > BAND * scale
    sent = np.isin(cand, got["send_idx"])
    np.testing.assert_array_equal(sent[sure], (want["dist"] > want["theta"])[sure])
    assert (got["dist"][sent] > th).all() and (got["dist"][~sent] <= th).all()
    assert (np.diff(got["send_idx"]) > 0).all()                    # candidate (ascending) order
    assert (got["tail_idx"] == -7).all()                           # nothing written past the count
    idx = got["send_idx"]
    if got["send_buf"] is not None:
        np.testing.assert_array_equal(got["send_buf"], E[idx])     # the message: bit for bit
    keep = np.setdiff1d(np.arange(E.shape[0]), idx)
    np.testing.assert_array_equal(got["L_new"][idx], E[idx])
    np.testing.assert_array_equal(got["L_new"][keep], L[keep])
    assert np.isnan(got["pad"]).all()                              # pitch padding untouched
    return want, sure


CASES = {
    "f128_all": dict(R=5000, F=128, ld=128, frac=None, factor=0.3),
    "f32_ragged_tile": dict(R=4097, F=32, ld=36, frac=None, factor=stale.theta_factor(1.0, 0.4)),
    "f100_subset_abs": dict(R=3000, F=100, ld=104, frac=0.4, theta=0.8),
    "f6_tail_columns": dict(R=1000, F=6, ld=8, frac=None, factor=0.25),
    "f256_subset": dict(R=2500, F=256, ld=256, frac=0.2, factor=stale.theta_factor(2.0, 0.1, "sigmoid")),
    "f300_two_sweeps": dict(R=700, F=300, ld=300, frac=None, factor=0.5),
    "f16_small": dict(R=70, F=16, ld=16, frac=None, factor=0.1),
    "theta_zero": dict(R=3000, F=64, ld=64, frac=None, theta=0.0),
    "one_row_one_column": dict(R=1, F=1, ld=4, frac=None, factor=0.5),
    "two_rows_bf16": dict(R=2, F=3, ld=8, frac=None, theta=0.0, bf16=True),
    "widest": dict(R=40, F=4096, ld=4096, frac=None, factor=0.3),
    "bf16_f128": dict(R=5000, F=128, ld=128, frac=None, factor=0.3, bf16=True),
    "bf16_f100_subset_tail": dict(R=3000, F=100, ld=104, frac=0.4, theta=0.8, bf16=True),
    "bf16_f520_two_sweeps": dict(R=600, F=520, ld=520, frac=None, factor=0.5, bf16=True),
    "factor_one": dict(R=3000, F=64, ld=64, frac=0.5, factor=1.0),
}


@pytest.mark.parametrize("name", list(CASES))
def test_filter_matches_oracle(name):
    c = CASES[name]
    E, L = synth.drifted_copies(11, c["R"], c["F"])
    if c.get("bf16"):
        E, L = synth.round_bf16(E), synth.round_bf16(L)
    rows = None if c["frac"] is None else synth.boundary_rows(11, c["R"], c["frac"])
    got = _device_filter(E, L, c["ld"], rows, c.get("factor"), c.get("theta"), bf16=bool(c.get("bf16")))
    want, sure = _check(E, L, rows, c.get("factor"), c.get("theta"), got)
    print(f"{name}: {got['send_idx'].size} of {want['dist'].size} candidates sent, D {want['D']:.4f}, theta "
          f"{want['theta']:.4f}, {int((~sure).sum())} rows inside the rounding band", flush=True)
    if name == "theta_zero":
        assert got["send_idx"].size == int((want["dist"] > 0).sum()) < c["R"]
    if name == "factor_one":
        assert got["send_idx"].size == 0


def test_two_epochs_and_no_message_buffer():
    # second epoch on the updated copies: rows sent in the first have distance exactly 0
    E, L = synth.drifted_copies(12, 6000, 128)
    got = _device_filter(E, L, 128, None, 0.2, None, with_buf=False)
    _check(E, L, None, 0.2, None, got)
    first = got["send_idx"]
    E2 = (E + synth.drifted_copies(13, 6000, 128)[0] * np.float32(0.01)).astype(np.float32)
    got2 = _device_filter(E2, got["L_new"].copy(), 128, None, 0.6, None)
    _check(E2, got["L_new"], None, 0.6, None, got2)
    again = _device_filter(E, got["L_new"].copy(), 128, None, None, 0.0)
    assert (again["dist"][first] == 0).all() and not np.isin(first, again["send_idx"]).any()


def test_empty_candidates_and_invalid_rows():
    import torch
    from paper_2309_03523_amd import binding
    E, L = synth.drifted_copies(14, 300, 32)
    got = _device_filter(E, L, 32, np.zeros(0, np.int64), 0.5, None)
    assert int(got["res"]["n_send"]) == 0 and float(got["res"]["D"]) == 0.0
    np.testing.assert_array_equal(got["L_new"], L)
    # listed rows outside the tensor are skipped and counted, the others are handled as usual
    rows = np.array([-3, 0, 5, 17, 300, 10 ** 12], np.int64)
    Ed, Ld = torch.from_numpy(E).cuda(), torch.from_numpy(L).cuda()
    dist = torch.zeros(8, device="cuda")
    send_idx = torch.zeros(8, dtype=torch.int64, device="cuda")
    result = torch.zeros(24, dtype=torch.uint8, device="cuda")
    ws = torch.empty(binding.stale_workspace_bytes(6), dtype=torch.uint8, device="cuda")
    binding.stale_filter(Ed, Ld, rows=torch.from_numpy(rows).cuda(), theta=0.0, dist=dist, send_idx=send_idx,
                         result=result, workspace=ws)
    torch.cuda.synchronize()
    res = result.cpu().numpy().view(binding.STALE_RESULT_DTYPE)[0]
    assert int(res["n_invalid"]) == 3
    want = stale.stale_filter(E, L, theta=0.0, rows=np.array([0, 5, 17]))
    assert send_idx.cpu().numpy()[:int(res["n_send"])].tolist() == want["send_idx"].tolist()


def test_argument_errors():
    import torch
    from paper_2309_03523_amd import binding
    E = torch.zeros(64, 32, device="cuda")
    L = torch.zeros(64, 32, device="cuda")
    dist = torch.zeros(64, device="cuda")
    idx = torch.zeros(64, dtype=torch.int64, device="cuda")
    res = torch.zeros(24, dtype=torch.uint8, device="cuda")
    ws = torch.empty(binding.stale_workspace_bytes(64), dtype=torch.uint8, device="cuda")
    ok = dict(dist=dist, send_idx=idx, result=res, workspace=ws, factor=0.5)
    binding.stale_filter(E, L, **ok)
    with pytest.raises(binding.DgcError, match="overlap"):
        binding.stale_filter(E, E, **ok)
    with pytest.raises(binding.DgcError, match="workspace"):
        binding.stale_filter(E, L, **{**ok, "workspace": ws[:8]})
    with pytest.raises(binding.DgcError, match="pitch"):
        binding.stale_filter(torch.zeros(64, 30, device="cuda"), torch.zeros(64, 30, device="cuda"), **ok)
    with pytest.raises(binding.DgcError, match="theta"):
        binding.stale_filter(E, L, **{**ok, "factor": None, "theta": -0.5})
    torch.cuda.synchronize()
