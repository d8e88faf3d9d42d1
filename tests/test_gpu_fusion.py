"""The device estimate of redundant loading between chunks (Section 5.1.1) against the oracle's
set definition, bit for bit, and the selection that follows from it."""
import numpy as np
import pytest

from oracle import fusion
from workloads import synth

pytestmark = pytest.mark.gpu


def _layer(wl):
    from paper_2309_03523_amd.runner import DeviceWorkload
    return DeviceWorkload(wl).layer


def _strips(N, T, width):
    return [[v, min(N, v + width), 0, T] for v in range(0, N, width)]


CASES = {
    "ragged_4_chunks_hub": lambda: synth.random_small(
        5, 8, 260, 8, 32, 32, 4.0, [[0, 70, 0, 8], [70, 201, 0, 5], [70, 201, 5, 8], [201, 260, 2, 8]], "gru", hub=True),
    "70_chunks_two_words": lambda: synth.random_small(6, 3, 280, 8, 32, 32, 6.0, _strips(280, 3, 4), "gru", hub=True),
    "130_chunks_global_counters": lambda: synth.random_small(7, 2, 260, 8, 32, 32, 5.0, _strips(260, 2, 2), "gru"),
    "single_chunk": lambda: synth.random_small(8, 2, 100, 8, 32, 32, 5.0, [[0, 100, 0, 2]], "gru"),
    "partial_cover": lambda: synth.random_small(9, 4, 200, 8, 32, 32, 5.0, [[10, 60, 1, 3], [100, 180, 0, 4]], "gru"),
    "one_vertex_chunks": lambda: synth.random_small(10, 2, 5, 8, 32, 32, 3.0, _strips(5, 2, 1), "gru", hub=True),
    "no_edges": lambda: synth.random_small(11, 3, 50, 8, 32, 32, 0.0, _strips(50, 3, 10), "gru"),
    "exactly_128_chunks": lambda: synth.random_small(12, 1, 256, 8, 32, 32, 6.0, _strips(256, 1, 2), "gru", hub=True),
    "129_chunks": lambda: synth.random_small(13, 1, 258, 8, 32, 32, 6.0, _strips(258, 1, 2), "gru", hub=True),
}


@pytest.mark.parametrize("name", list(CASES))
def test_shared_rows_bit_exact(name):
    wl = CASES[name]()
    got = _layer(wl).shared_rows()
    want = fusion.shared_rows(wl.graph, wl.chunks)
    print(f"{name}: {len(wl.chunks)} chunks, {int(np.triu(want).sum())} shared rows in {int((np.triu(want) > 0).sum())} pairs",
          flush=True)
    np.testing.assert_array_equal(got, want)


def test_config2_scaled_selection_end_to_end():
    from paper_2309_03523_amd import binding
    wl = synth.config2(0, scale=0.02)                   # 2 000 vertices x 32 snapshots, 64 chunks in 4 windows
    layer = _layer(wl)
    got = layer.shared_rows()
    want = fusion.shared_rows(wl.graph, wl.chunks)
    np.testing.assert_array_equal(got, want)
    ch = np.asarray(wl.chunks)
    for a in range(len(ch)):                            # different windows share nothing
        for b in range(len(ch)):
            if ch[a, 2] != ch[b, 2]:
                assert got[a, b] == 0
    mem = (ch[:, 1] - ch[:, 0]) * (ch[:, 3] - ch[:, 2])   # stand-in for the measured memory: own rows
    cap = int(mem.sum() // 6)
    grp = binding.fusion_select(got, mem, cap)
    np.testing.assert_array_equal(grp, fusion.select_fusion(want, mem, cap))
    gm = np.bincount(grp, weights=mem)
    assert gm.max() <= cap and grp.max() + 1 < len(ch)
