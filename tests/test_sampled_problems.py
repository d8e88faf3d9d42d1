"""The small problems that the full-size GPU parity tests hand to the oracle vertex by vertex must
give what the oracle gives for those vertices inside the whole problem: checked here on problems
small enough to run whole (CPU only; both sides are the oracle)."""
import numpy as np

import oracle
from oracle import dysat
from workloads import synth


def test_sampled_problem_of_the_evolving_gcn_equals_the_whole():
    import test_gpu_evolve as te
    chunks = [[0, 40, 0, 6], [40, 97, 0, 3], [40, 97, 3, 6], [97, 150, 0, 6]]
    wl = te._workload(5, 6, 150, 32, chunks)
    whole = oracle.evolve(wl.graph, wl.chunks, wl.params, wl.X, wl.C)["Y"]
    picks = [(v, ch) for ch in wl.chunks.tolist() for v in range(ch[0], ch[1], 7)]
    hub = int(np.argmax(np.diff(wl.graph.snaps[0].rowptr)))
    picks += [(hub, ch) for ch in wl.chunks.tolist() if ch[0] <= hub < ch[1]]
    g1, c1, X1, C1 = te._sampled_problem(wl, picks)
    part = oracle.evolve(g1, c1, wl.params, X1, C1)["Y"]
    for i, (v, ch) in enumerate(picks):
        np.testing.assert_allclose(part[ch[2]:ch[3], i], whole[ch[2]:ch[3], v], rtol=0, atol=1e-6)
        assert np.abs(whole[ch[2]:ch[3], v]).max() > 0


def test_one_vertex_problem_of_the_attention_layer_equals_the_whole():
    import test_gpu_dysat as td
    c = td.CASES["ragged"]
    wl = synth.dysat_small(46, c["T"], c["N"], 128, 8, c["deg"], c["chunks"], hub=True)
    whole = dysat.forward(wl.graph, wl.chunks, wl.params, wl.X, wl.C, 8)["Y"]
    for ch in wl.chunks.tolist():
        for v in range(ch[0], ch[1], 9):
            g1, c1, p1, X1, C1 = td._one_vertex_problem(wl, v, ch)
            part = dysat.forward(g1, c1, p1, X1, C1, 8)["Y"][:, 0]
            np.testing.assert_allclose(part, whole[ch[2]:ch[3], v], rtol=0, atol=1e-12)


def test_two_hop_problem_gives_the_input_gradient_of_the_whole():
    """The stand-in that carries a sampled vertex together with its neighbours of the same chunk:
    its output and the gradient of its input row (rescaled by the ratio of the covered element
    counts, the only thing the mean in the loss sees of the rest) equal the whole problem's."""
    import test_gpu_evolve as te
    from workloads import sampling
    chunks = [[0, 40, 0, 6], [40, 97, 0, 3], [40, 97, 3, 6], [97, 150, 0, 6]]
    wl = te._workload(7, 6, 150, 32, chunks)
    target = synth.stream(7, "target").standard_normal((6, 150, 32)).astype(np.float32)
    whole = oracle.evolve(wl.graph, wl.chunks, wl.params, wl.X, wl.C, target, want_dx=True)
    picks = [(v, ch) for ch in wl.chunks.tolist() for v in range(ch[0], ch[1], 11)]
    hub = int(np.argmax(np.diff(wl.graph.snaps[3].rowptr)))
    picks += [(hub, ch) for ch in wl.chunks.tolist() if ch[0] <= hub < ch[1]]
    g1, c1, X1, C1, T1, where, _ = sampling.two_hop_problem(
        wl.graph, picks, lambda t, ids: wl.X[t, ids], lambda t, ids: wl.C[t, ids], lambda t, ids: target[t, ids], 32)
    part = oracle.evolve(g1, c1, wl.params, X1, C1, T1, want_dx=True)
    n_whole = sum((b - a) * (t1 - t0) for a, b, t0, t1 in chunks)
    n_part = int(((c1[:, 1] - c1[:, 0]) * (c1[:, 3] - c1[:, 2])).sum())
    seen = 0.0
    for (v, ch), loc in zip(picks, where.tolist()):
        np.testing.assert_allclose(part["Y"][ch[2]:ch[3], loc], whole["Y"][ch[2]:ch[3], v], rtol=0, atol=1e-6)
        want = whole["dX"][ch[2]:ch[3], v]
        got = part["dX"][ch[2]:ch[3], loc] * (n_part / n_whole)
        np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-12 * np.abs(want).max())
        seen = max(seen, float(np.abs(want).max()))
    assert seen > 0
