"""Pins of the stale-filter oracle (oracle/stale.py) against closed forms, brute force and the
argument the paper makes for comparing with the copy sent last (Section 5.2)."""
import math

import numpy as np
import pytest

from oracle import stale
from workloads import synth


def test_theta_closed_forms():
    # no loss decrease yet: norm = 0, both signs give half of D
    assert stale.theta_factor(2.0, 2.0, "printed") == 0.5
    assert stale.theta_factor(2.0, 2.0, "sigmoid") == 0.5
    # loss fallen to zero: norm = 1
    assert stale.theta_factor(3.0, 0.0, "printed") == pytest.approx(1.0 / (1.0 + math.e), rel=1e-15)
    assert stale.theta_factor(3.0, 0.0, "sigmoid") == pytest.approx(math.e / (1.0 + math.e), rel=1e-15)
    # loss halved: norm = 1/2, whatever the scale of the loss
    for l1 in (0.7, 5.0, 120.0):
        assert stale.theta_factor(l1, l1 / 2, "printed") == pytest.approx(1.0 / (1.0 + math.sqrt(math.e)), rel=1e-15)


def test_theta_direction_of_each_variant():
    losses = [1.0, 0.8, 0.5, 0.2, 0.05]
    printed = [stale.theta_factor(1.0, l, "printed") for l in losses]
    sigmoid = [stale.theta_factor(1.0, l, "sigmoid") for l in losses]
    assert all(a > b for a, b in zip(printed, printed[1:]))       # the equation as printed falls
    assert all(a < b for a, b in zip(sigmoid, sigmoid[1:]))       # the prose wants it to grow
    for p, s in zip(printed, sigmoid):
        assert p + s == pytest.approx(1.0, abs=1e-15)            # 1/(1+e^x) + 1/(1+e^-x) = 1


def test_distance_known_triangles():
    E = np.zeros((3, 6))
    L = np.zeros((3, 6))
    E[0, 1], E[0, 4] = 3.0, 4.0                 # 3-4-5
    E[1, 0], L[1, 0] = 1.0, -1.0                # one coordinate, difference 2
    E[2], L[2] = 1.5, -0.5                      # every coordinate differs by 2: 2*sqrt(6)
    np.testing.assert_allclose(stale.distances(E, L), [5.0, 2.0, 2.0 * math.sqrt(6.0)], rtol=1e-15)
    # symmetric in its arguments, zero on identical rows
    np.testing.assert_array_equal(stale.distances(E, L), stale.distances(L, E))
    assert (stale.distances(E, E) == 0).all()


def test_distance_brute_force():
    E, L = synth.drifted_copies(3, 37, 19)
    want = [math.sqrt(math.fsum((float(E[r, f]) - float(L[r, f])) ** 2 for f in range(19))) for r in range(37)]
    np.testing.assert_allclose(stale.distances(E, L), want, rtol=1e-14)
    rows = np.array([0, 5, 6, 36])
    np.testing.assert_allclose(stale.distances(E, L, rows), [want[r] for r in rows], rtol=1e-14)


def test_filter_brute_force_and_update():
    E, L = synth.drifted_copies(4, 200, 16)
    out = stale.stale_filter(E, L, factor=0.3)
    dist = [math.sqrt(math.fsum((float(E[r, f]) - float(L[r, f])) ** 2 for f in range(16))) for r in range(200)]
    D = max(dist)
    assert out["D"] == pytest.approx(D, rel=1e-14)
    assert out["theta"] == pytest.approx(0.3 * D, rel=1e-14)
    want = [r for r in range(200) if dist[r] > 0.3 * D]
    assert out["send_idx"].tolist() == want and 0 < len(want) < 200
    np.testing.assert_array_equal(out["send_buf"], E[want].astype(np.float64))
    keep = np.setdiff1d(np.arange(200), want)
    np.testing.assert_array_equal(out["L_new"][want], E[want].astype(np.float64))
    np.testing.assert_array_equal(out["L_new"][keep], L[keep].astype(np.float64))
    # inputs untouched; filtering again with the same threshold sends nothing new
    again = stale.stale_filter(E, out["L_new"], theta=out["theta"])
    assert again["send_idx"].size == 0
    np.testing.assert_array_equal(again["dist"][want], 0.0)


def test_static_thresholds_are_monotone_and_bounded():
    # the multiples of D of the paper's accuracy table
    E, L = synth.drifted_copies(5, 5000, 32)
    D = stale.distances(E, L).max()
    changed = int((stale.distances(E, L) > 0).sum())
    sent = [stale.stale_filter(E, L, theta=f * D)["send_idx"].size for f in (0.0, 0.1, 0.3, 0.5, 0.7, 0.9, 1.0)]
    assert sent[0] == changed < 5000           # theta = 0: everything that moved, nothing that did not
    assert all(a >= b for a, b in zip(sent, sent[1:]))
    assert sent[-2] >= 1 and sent[-1] == 0      # the farthest row passes 0.9 D; nothing exceeds D itself
    # the generator's distance mix: most rows well below 1, a tail above (the shape the paper plots)
    d = stale.distances(E, L)
    assert 0.75 < (d < 1.0).mean() < 0.95 and d.max() > 3.0


def test_candidates_restrict_distance_maximum_and_selection():
    E, L = synth.drifted_copies(6, 300, 8)
    L[17] = E[17] + 100.0                        # a huge drift on a row that is not a candidate
    rows = np.array([r for r in range(300) if r % 3 == 0 and r != 17], np.int64)
    out = stale.stale_filter(E, L, factor=0.5, rows=rows)
    assert out["D"] < 50 and out["dist"].shape == rows.shape
    assert set(out["send_idx"].tolist()) <= set(rows.tolist())
    np.testing.assert_array_equal(out["L_new"][17], L[17].astype(np.float64))
    assert stale.stale_filter(E, L, factor=0.5, rows=np.zeros(0, np.int64))["D"] == 0.0


def test_slow_drift_is_sent_eventually_but_never_against_the_previous_epoch():
    # the paper's argument for keeping the copy sent last: steps of 1 in a fixed direction, theta 2.5
    F, epochs, theta = 4, 10, 2.5
    direction = np.array([[1.0, 0.0, 0.0, 0.0]])
    L_last = np.zeros((1, F))
    L_prev = np.zeros((1, F))
    sent_last, sent_prev = [], []
    for r in range(1, epochs + 1):
        E = r * direction
        out = stale.stale_filter(E, L_last, theta=theta)
        if out["send_idx"].size:
            sent_last.append(r)
        L_last = out["L_new"]
        if stale.stale_filter(E, L_prev, theta=theta)["send_idx"].size:
            sent_prev.append(r)
        L_prev = E.copy()                        # the alternative design: refresh every epoch
    assert sent_last == [3, 6, 9]
    assert sent_prev == []
    # the error against what the peers hold never exceeds theta under the method
    assert np.abs(epochs * direction - L_last).max() <= theta


def test_static_threshold_traffic_against_the_printed_table():
    # The paper prints, per data set, the share of traffic a static threshold x*D saves.  The data
    # are not available; the triangular drift generator was chosen so that the oracle's filter on it
    # saves what the table prints for Amazon and Epinion at x >= 0.3 within 5 points.  (A filter
    # that compared with >=, used the squared distance, or took D over the wrong set would not.)
    import os
    table = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "stale_threshold_table.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, *vals = line.split()
                table[name] = [float(v) for v in vals]
    E, L = synth.drifted_copies(7, 40000, 16, kind="triangular", unchanged=0.0)
    D = stale.distances(E, L).max()
    saved = [100.0 * (1.0 - stale.stale_filter(E, L, theta=x * D)["send_idx"].size / 40000) for x in (0.3, 0.5, 0.7, 0.9)]
    for name in ("Amazon", "Epinion"):
        for got, want in zip(saved, table[name][1:]):
            assert abs(got - want) < 5.0, (name, saved, table[name])
    # every data set in the table saves more traffic at a larger threshold; so does the oracle
    assert all(a < b for a, b in zip(saved, saved[1:]))
    for vals in table.values():
        assert all(a < b for a, b in zip(vals, vals[1:]))
