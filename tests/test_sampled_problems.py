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
