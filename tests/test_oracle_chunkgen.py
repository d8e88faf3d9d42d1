"""Pins of the label-propagation oracle (oracle/chunkgen.py): the paper's closed form for the
initial labels, textbook outcomes on graphs whose communities are obvious, the role of the two
edge weights, the size limit, and the invariants the paper's argument rests on."""
import numpy as np
import pytest

from oracle import chunkgen
from workloads import synth


def _graph(N, edge_lists):
    return synth.DynamicGraph(N=N, snaps=[synth.csr_from_undirected(N, np.array([e[0] for e in el], np.int64),
                                                                    np.array([e[1] for e in el], np.int64))
                                          for el in edge_lists])


def _clique(vs):
    return [(a, b) for k, a in enumerate(vs) for b in vs[k + 1:]]


def test_initial_labels_closed_form():
    # c(v_{i,t}) = (vertices of the earlier snapshots) + i: all different, snapshot-major
    lab = chunkgen.initial_labels(3, 5)
    assert lab.tolist() == list(range(15))
    assert lab.reshape(3, 5)[2, 1] == 2 * 5 + 1
    assert np.unique(chunkgen.initial_labels(7, 11)).size == 77


def test_two_cliques_and_a_bridge_become_two_chunks():
    g = _graph(10, [_clique([0, 1, 2, 3, 4]) + _clique([5, 6, 7, 8, 9]) + [(4, 5)]])
    out = chunkgen.propagate(g, 1, 1, cap=100, max_iters=50)
    lab = out["labels"]
    assert out["converged"]
    assert len(set(lab[:5])) == 1 and len(set(lab[5:])) == 1 and lab[0] != lab[5]
    # every edge but the bridge is inside a chunk
    assert chunkgen.inside_weight(g, lab, 1, 1) == chunkgen.total_weight(g, 1, 1) - 1


def test_temporal_edges_carry_labels_across_snapshots():
    # no spatial edges at all: each vertex's copies form a path over the snapshots
    g = _graph(3, [[], [], [], []])
    out = chunkgen.propagate(g, 1, 1, cap=100, max_iters=50)
    lab = out["labels"].reshape(4, 3)
    assert out["converged"]
    for i in range(3):
        # a path of 4 settles into chunks of adjacent copies; nothing crosses to another vertex
        assert set(lab[:, i]) <= {t * 3 + i for t in range(4)}
    assert chunkgen.inside_weight(g, out["labels"], 1, 1) >= 3 * 2
    # with temporal weight 0 nothing propagates: every label stays as initialised
    still = chunkgen.propagate(g, 1, 0, cap=100, max_iters=50)
    assert still["labels"].tolist() == list(range(12)) and still["iterations"] == 1


def test_edge_weights_decide_between_spatial_and_temporal_neighbours():
    # two snapshots; vertex 0 at t=1 has two spatial neighbours {1, 2} that already share a label
    # (they form a triangle with 3 in both snapshots) and one temporal neighbour (its own copy at t=0,
    # which sits in a clique {0, 4, 5} at t=0 only).
    snap0 = _clique([0, 4, 5]) + _clique([1, 2, 3])
    snap1 = _clique([1, 2, 3]) + [(0, 1), (0, 2)]
    g = _graph(6, [snap0, snap1])
    x = 1 * 6 + 0
    heavy_t = chunkgen.propagate(g, 1, 5, cap=100, max_iters=50)["labels"]
    heavy_s = chunkgen.propagate(g, 5, 1, cap=100, max_iters=50)["labels"]
    assert heavy_t[x] == heavy_t[0 * 6 + 0]            # temporal edge outweighs the two spatial ones (5 > 2)
    assert heavy_s[x] == heavy_s[1 * 6 + 1]            # spatial edges outweigh it (10 > 1)
    assert heavy_t[x] != heavy_t[1 * 6 + 1] and heavy_s[x] != heavy_s[0 * 6 + 0]


def test_one_iteration_by_hand():
    # path 0 - 1 - 2, one snapshot, all weights 1, labels 0, 1, 2.
    # candidates: 0 -> 1, 1 -> 0 (tie between 0 and 2, smaller label), 2 -> 1; all want to change
    # (own score 0).  The order of iteration 0 is 0, 1, 2 (h(0) = 0 < h(1) < h(2)): 0 changes (no
    # earlier neighbour wants); 1 is blocked by 0; 2 is blocked by 1.
    g = _graph(3, [[(0, 1), (1, 2)]])
    assert sorted(range(3), key=lambda x: chunkgen.order_key(x, 0)) == [0, 1, 2]
    lab, changed = chunkgen.iteration(g, chunkgen.initial_labels(1, 3), 1, 1, cap=10, r=0)
    assert lab.tolist() == [1, 1, 2] and changed == 1
    # next: 0 has label 1 with score 1 (stays); 1 has own score 1, candidate 2 scores 1: not strictly more;
    # 2 -> 1 scores 1 > 0: changes.
    lab, changed = chunkgen.iteration(g, lab, 1, 1, cap=10, r=1)
    assert lab.tolist() == [1, 1, 1] and changed == 1
    assert chunkgen.iteration(g, lab, 1, 1, cap=10, r=2)[1] == 0


def test_order_of_an_iteration_decides_between_adjacent_vertices():
    # two vertices, one edge: both want the other's label; exactly the one that comes first in the
    # iteration's order changes, and the order is not the index order in every iteration
    g = _graph(2, [[(0, 1)]])
    firsts = set()
    for r in range(40):
        lab, changed = chunkgen.iteration(g, chunkgen.initial_labels(1, 2), 1, 1, cap=10, r=r)
        first = min(range(2), key=lambda x: chunkgen.order_key(x, r))
        assert changed == 1 and lab[first] == 1 - first and lab[1 - first] == 1 - first
        firsts.add(first)
    assert firsts == {0, 1}
    # the mixing function is a bijection on a sample and spreads consecutive inputs
    hs = [chunkgen._h(v) for v in range(5000)]
    assert len(set(hs)) == 5000 and chunkgen._h(0) == 0 and max(hs) > 2 ** 31 > min(hs[1:])


def test_size_limit_holds_labels_back():
    g = _graph(8, [_clique(list(range(8)))])
    free = chunkgen.propagate(g, 1, 1, cap=100, max_iters=50)["labels"]
    assert len(set(free)) == 1                          # one clique, one chunk
    assert chunkgen.propagate(g, 1, 1, cap=1, max_iters=50)["labels"].tolist() == list(range(8))   # nothing admissible
    capped = chunkgen.propagate(g, 1, 1, cap=3, max_iters=50)
    sizes = np.bincount(capped["labels"])
    assert capped["converged"] and sizes.max() <= 3 + 1 and (sizes > 0).sum() >= 2
    # a label that had reached the limit when an iteration started gains no vertex in it
    lab = chunkgen.initial_labels(1, 8)
    for r in range(10):
        before = np.bincount(lab, minlength=8)
        lab, changed = chunkgen.iteration(g, lab, 1, 1, cap=3, r=r)
        after = np.bincount(lab, minlength=8)
        assert (after[before >= 3] <= before[before >= 3]).all()
        if not changed:
            break


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_every_iteration_raises_the_weight_inside_chunks(seed):
    wl = synth.random_small(seed, 3, 40, 4, 32, 32, 3.0, [[0, 40, 0, 3]], "gru", hub=True)
    g, ws, wt = wl.graph, 2, 1
    lab = chunkgen.initial_labels(g.T, g.N)
    total = chunkgen.total_weight(g, ws, wt)
    prev = chunkgen.inside_weight(g, lab, ws, wt)
    assert prev == 0
    for it in range(200):
        lab, changed = chunkgen.iteration(g, lab, ws, wt, cap=10 ** 9, r=it)
        cur = chunkgen.inside_weight(g, lab, ws, wt)
        if changed == 0:
            assert cur == prev
            break
        assert cur >= prev + changed                    # every change gains at least one unit of weight
        prev = cur
    else:
        raise AssertionError("did not converge")
    assert 0 < prev <= total                            # inside + between = total: maximising one minimises the other
    # fixed point: no vertex has a neighbour label that scores strictly more than its own
    for x in range(lab.size):
        sc = {}
        for u, w in chunkgen.neighbours(g, x, ws, wt):
            sc[lab[u]] = sc.get(lab[u], 0) + w
        assert all(s <= sc.get(lab[x], 0) for s in sc.values())
    out = chunkgen.propagate(g, ws, wt, cap=10 ** 9, max_iters=200)
    np.testing.assert_array_equal(out["labels"], lab)
    assert out["converged"] and out["iterations"] == it + 1
