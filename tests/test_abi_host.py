"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments with the documented status codes before touching
the device."""
import ctypes as ct
import os
import re

import numpy as np
import pytest

from paper_2309_03523_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return binding.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "dgc.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dgc_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert binding.version().startswith("dgc ")


def _create(lib, desc_kw=None, chunks=((0, 4, 0, 2),), T=2, N=4, null_snapshot=False):
    d = dict(struct_kind=0, n_struct_layers=1, time_kind=1, dtype=0, F=8, S=32, H=32, act_hidden=0, act_out=0,
             gather_mode=0, validate_level=0, rows_per_group=0, long_nnz=0, part_nnz=0, dense_kernel=0, heads=0,
             lstm_input_concat=0, agg_kernel=0, n_time_layers=0)
    d.update(desc_kw or {})
    desc = binding.DescT(*[d[n] for n, _ in binding.DescT._fields_])
    fake = 0x1000  # never dereferenced: every check below fails before the device is used
    rp = (ct.c_void_p * T)(*[fake] * T)
    cj = (ct.c_void_p * T)(*([fake] * (T - 1) + [None if null_snapshot else fake]))
    graph = binding.GraphT(T, N, rp, cj)
    carr = (binding.ChunkT * len(chunks))(*[binding.ChunkT(*c) for c in chunks])
    h = ct.c_void_p(None)
    rc = lib.dgc_layer_create(ct.byref(desc), ct.byref(graph), carr, len(chunks), None, ct.byref(h))
    assert rc != 0 and not h.value
    return rc, lib.dgc_last_error(None).decode()


def test_create_rejects_bad_descriptors(lib):
    assert _create(lib, dict(S=48))[0] == 1
    assert _create(lib, dict(H=31))[0] == 1
    assert _create(lib, dict(F=0))[0] == 1
    assert _create(lib, dict(n_struct_layers=3))[0] == 1
    assert _create(lib, dict(time_kind=9))[0] == 1
    assert _create(lib, dict(dtype=7))[0] == 1
    assert _create(lib, dict(struct_kind=5))[0] == 1
    # graph attention, temporal self-attention and bf16 only come together, in one shape
    assert _create(lib, dict(dtype=1))[0] == 4
    assert _create(lib, dict(struct_kind=2))[0] == 4
    assert _create(lib, dict(time_kind=3))[0] == 4
    gat = dict(struct_kind=2, time_kind=3, dtype=1, F=128, S=128, H=128, heads=8)
    assert _create(lib, dict(gat, heads=4))[0] == 4
    assert _create(lib, dict(gat, F=64))[0] == 4
    assert _create(lib, dict(gat), chunks=((0, 5, 0, 2),))[0] == 3
    assert _create(lib, dict(rows_per_group=64))[0] == 1
    assert _create(lib, null_snapshot=True)[0] == 1
    # the LSTM reading both GCN layers' outputs: two layers, LSTM, the wave-private kernel's sizes
    cat = dict(lstm_input_concat=1, n_struct_layers=2, time_kind=2)
    assert _create(lib, dict(cat, time_kind=1))[0] == 1
    assert _create(lib, dict(cat, n_struct_layers=1))[0] == 1
    assert _create(lib, dict(cat, lstm_input_concat=2))[0] == 1
    assert _create(lib, dict(cat, S=96, H=96))[0] == 4
    assert _create(lib, dict(cat, dense_kernel=1))[0] == 4
    assert _create(lib, dict(gat, lstm_input_concat=1))[0] == 1


def test_create_rejects_bad_chunks(lib):
    rc, msg = _create(lib, chunks=((0, 5, 0, 2),))
    assert rc == 3 and "outside" in msg
    assert _create(lib, chunks=((2, 2, 0, 2),))[0] == 3          # empty vertex range
    assert _create(lib, chunks=((0, 4, 1, 1),))[0] == 3          # empty window
    assert _create(lib, chunks=((0, 4, 0, 3),))[0] == 3          # window past T
    rc, msg = _create(lib, chunks=((0, 3, 0, 2), (2, 4, 1, 2)))
    assert rc == 3 and "overlap" in msg
    # touching but disjoint chunks pass the chunk check; without a GPU the next failure is the
    # device.  (With a GPU the fake CSR pointers would be followed, so the case is CPU-only.)
    import torch
    if not torch.cuda.is_available():
        rc, msg = _create(lib, chunks=((0, 2, 0, 2), (2, 4, 0, 1), (2, 4, 1, 2)))
        assert rc == 6


def test_null_arguments(lib):
    h = ct.c_void_p(None)
    assert lib.dgc_layer_create(None, None, None, 0, None, ct.byref(h)) == 1
    assert lib.dgc_layer_destroy(None) == 0
    assert lib.dgc_layer_forward(None, None, 0, None, 0, None, 0, None, None, None, 0, None, None) == 1
    assert lib.dgc_layer_packing(None, b"halo_ptr", None, 0, None) == 1
    assert isinstance(lib.dgc_last_error(None), bytes)


def test_product_does_not_import_the_oracle():
    """The product path never routes through the oracle (or any CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2309_03523_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "dgc_oracle" not in text, f
    assert "paper_2309_03523_amd" not in open(os.path.join(ROOT, "oracle", "__init__.py")).read()
    # the input generators hold no arithmetic of the method and import neither side
    for f in os.listdir(os.path.join(ROOT, "workloads")):
        if f.endswith(".py"):
            text = open(os.path.join(ROOT, "workloads", f)).read()
            assert "import oracle" not in text and "from oracle" not in text and "paper_2309_03523_amd" not in text, f


def test_stale_threshold_factor_and_host_checks(lib):
    import math
    lib.dgc_stale_theta_factor.restype = ct.c_double
    lib.dgc_stale_theta_factor.argtypes = [ct.c_double, ct.c_double, ct.c_int32]
    lib.dgc_stale_workspace_bytes.restype = ct.c_int64
    lib.dgc_stale_workspace_bytes.argtypes = [ct.c_int64]
    f = lib.dgc_stale_theta_factor
    assert f(2.0, 2.0, 0) == 0.5 and f(2.0, 2.0, 1) == 0.5               # no loss decrease yet
    assert abs(f(3.0, 0.0, 0) - 1.0 / (1.0 + math.e)) < 1e-15            # the equation as printed, norm = 1
    assert abs(f(3.0, 0.0, 1) - math.e / (1.0 + math.e)) < 1e-15
    assert abs(f(1.0, 0.3, 0) + f(1.0, 0.3, 1) - 1.0) < 1e-15
    assert f(0.0, 1.0, 0) < 0 and f(1.0, 1.0, 7) < 0 and f(1.0, float("nan"), 0) < 0
    w = [lib.dgc_stale_workspace_bytes(n) for n in (0, 1, 2048, 2049, 10 ** 7)]
    assert w[0] > 0 and all(a <= b for a, b in zip(w, w[1:])) and lib.dgc_stale_workspace_bytes(-1) < 0
    lib.dgc_stale_filter.restype = ct.c_int
    lib.dgc_stale_filter.argtypes = [ct.c_void_p, ct.c_int64, ct.c_void_p, ct.c_int64, ct.c_int64, ct.c_int32, ct.c_int32,
                                     ct.c_void_p, ct.c_int64, ct.c_double, ct.c_double, ct.c_void_p, ct.c_void_p,
                                     ct.c_void_p, ct.c_int64, ct.c_void_p, ct.c_void_p, ct.c_int64, ct.c_void_p]
    assert lib.dgc_stale_filter(None, 0, None, 0, 0, 0, 0, None, 0, 0.5, 0.0, None, None, None, 0, None, None, 0, None) == 1
    assert b"stale filter" in lib.dgc_last_error(None)


def test_fusion_select_and_chunk_assign_match_the_oracle():
    # host arithmetic behind the C ABI: no GPU needed
    from oracle import fusion
    from paper_2309_03523_amd import binding
    rng = np.random.default_rng(0)
    for trial in range(25):
        n = int(rng.integers(1, 24))
        sh = rng.integers(0, 40, (n, n))
        sh = np.triu(sh, 1) + np.triu(sh, 1).T
        sh[rng.random((n, n)) < 0.3] = 0
        sh = np.minimum(sh, sh.T)
        mem = rng.integers(0, 20, n)
        cap = int(rng.integers(5, 70))
        np.testing.assert_array_equal(binding.fusion_select(sh, mem, cap), fusion.select_fusion(sh, mem, cap))
        g = rng.integers(1, 50, n).astype(float)          # integer-valued: sums are exact in any order
        h = rng.integers(0, 9, (n, n)).astype(float)
        h = np.triu(h, 1) + np.triu(h, 1).T
        for n_gpus in (1, 2, 3, 8):
            np.testing.assert_array_equal(binding.chunk_assign(g, h, n_gpus), fusion.assign_chunks(g, h, n_gpus))
    with pytest.raises(binding.DgcError, match="symmetric"):
        binding.fusion_select(np.array([[0, 1], [2, 0]]), np.array([1, 1]), 5)
    with pytest.raises(binding.DgcError, match="negative memory"):
        binding.fusion_select(np.zeros((2, 2), np.int64), np.array([1, -1]), 5)
    with pytest.raises(binding.DgcError, match="n_gpus"):
        binding.chunk_assign(np.ones(2), np.zeros((2, 2)), 0)
