"""dgc_stale_filter_static (the entry point that allocates nothing: its block counts and scan
temporaries live in a fixed device array inside the library) against dgc_stale_filter with a
caller workspace: same distances, D, threshold, send list, message and updated copies, bit for
bit, on two calls in a row of which the second is smaller (the array still holds the first
call's contents then)."""
import numpy as np
import pytest

from workloads import synth

pytestmark = pytest.mark.gpu


def _run(E, L, ld, rows, factor, static):
    import torch
    from paper_2309_03523_amd import binding
    R, F = E.shape
    Ed = torch.full((R, ld), float("nan"), device="cuda")
    Ld = torch.full((R, ld), float("nan"), device="cuda")
    Ed[:, :F] = torch.from_numpy(E).cuda()
    Ld[:, :F] = torch.from_numpy(L).cuda()
    rd = None if rows is None else torch.from_numpy(rows).cuda()
    n = R if rows is None else rows.size
    dist = torch.full((n,), -1.0, device="cuda")
    send_idx = torch.full((n,), -7, dtype=torch.int64, device="cuda")
    send_buf = torch.full((n, ld), float("nan"), device="cuda")
    result = torch.zeros(24, dtype=torch.uint8, device="cuda")
    ws = None if static else torch.empty(binding.stale_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    binding.stale_filter(Ed, Ld, F=F, rows=rd, factor=factor, dist=dist, send_idx=send_idx, send_buf=send_buf,
                         result=result, workspace=ws)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    res = result.cpu().numpy().view(binding.STALE_RESULT_DTYPE)[0]
    return {"dist": dist.cpu().numpy(), "send_idx": send_idx.cpu().numpy(), "send_buf": send_buf.cpu().numpy(),
            "L": Ld.cpu().numpy(), "res": res}


def _same(a, b):
    for k in ("dist", "send_idx", "send_buf", "L"):
        np.testing.assert_array_equal(a[k], b[k], err_msg=k)
    for f in ("n_send", "D", "theta", "n_invalid"):
        assert a["res"][f] == b["res"][f], f


def test_static_scratch_matches_workspace_twice_second_smaller():
    from paper_2309_03523_amd import binding
    assert binding.stale_static_max_candidates() == 1 << 26
    # first call: 150 000 candidates = 74 selection blocks; second: a row list of 3 000 = 2 blocks
    E1, L1 = synth.drifted_copies(11, 150_000, 64)
    E2, L2 = synth.drifted_copies(12, 9_000, 100)
    rows2 = synth.boundary_rows(13, 9_000, 1 / 3)
    for E, L, ld, rows, factor in ((E1, L1, 64, None, 0.3), (E2, L2, 104, rows2, 0.45)):
        got = _run(E, L, ld, rows, factor, static=True)
        want = _run(E, L, ld, rows, factor, static=False)
        assert 0 < int(want["res"]["n_send"]) < (E.shape[0] if rows is None else rows.size)
        _same(got, want)


def test_static_scratch_rejects_too_many_candidates():
    import torch
    from paper_2309_03523_amd import binding
    lib = binding.load()
    cap = binding.stale_static_max_candidates()
    t = torch.zeros(64, device="cuda")
    # R beyond the limit with rows = NULL: refused before anything is enqueued or dereferenced
    rc = lib.dgc_stale_filter_static(t.data_ptr(), 4, t.data_ptr() + 128, 4, cap + 1, 4, 0, None, 0, 0.5, 0.0,
                                     t.data_ptr(), t.data_ptr(), None, 0, t.data_ptr(), None)
    assert rc == 4 and b"candidates" in lib.dgc_last_error(None)
