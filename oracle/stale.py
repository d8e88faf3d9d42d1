"""CPU oracle of the adaptive stale-embedding filter (Section 5.2 of the paper): an embedding is
(re)transmitted only if its L2 distance to the copy transmitted last exceeds a threshold that
follows the training loss.

TEST INFRASTRUCTURE ONLY: plain NumPy, float64.  Nothing in the product path may import this
module.

Definitions (the paper's, with the points it leaves open decided here):
  * candidates: the rows that can be transmitted at all (`rows`, ascending; None = every row);
  * dist[r] = || E[r] - L[r] ||_2, E the current embeddings, L the copies transmitted last;
  * D = max dist over the candidates (the paper's D_r; 0 if there are none);
  * theta = factor(l_1, l_{r-1}) * D with the threshold equation of Section 5.2, or a given value
    (the static thresholds of the paper's accuracy table are multiples of D);
  * a candidate is transmitted iff dist[r] > theta (strictly: with theta = 0 an unchanged
    embedding is not sent); the transmitted rows, ascending, are `send_idx`; their current values
    are the message (`send_buf`) and replace the stored copies (L[r] <- E[r]); all other copies
    stay as they are, so slow drift adds up against the copy sent last and is sent eventually.

The threshold equation as printed gives a factor that falls from 1/2 towards 1/(1+e) while the
loss falls; the prose around it asks for a threshold that grows.  `variant="printed"` is the
equation, `variant="sigmoid"` the sign under which the prose holds (factor = 1/(1+exp(-norm))).
"""
from __future__ import annotations

import math
from typing import Optional

import numpy as np


def theta_factor(l1: float, l_prev: float, variant: str = "printed") -> float:
    """theta_r / D_r from the initial loss l_1 and the loss of the epoch before (Section 5.2)."""
    norm = (l1 - l_prev) / l1
    if variant == "printed":
        return 1.0 / (1.0 + math.exp(norm))
    if variant == "sigmoid":
        return 1.0 / (1.0 + math.exp(-norm))
    raise ValueError(variant)


def distances(E: np.ndarray, L: np.ndarray, rows: Optional[np.ndarray] = None) -> np.ndarray:
    """dist[r] for every row (rows=None) or for the listed rows, float64."""
    E = np.asarray(E, np.float64)
    L = np.asarray(L, np.float64)
    if rows is not None:
        E, L = E[rows], L[rows]
    d = E - L
    return np.sqrt((d * d).sum(axis=1))


def stale_filter(E: np.ndarray, L: np.ndarray, *, factor: Optional[float] = None,
                 theta: Optional[float] = None, rows: Optional[np.ndarray] = None) -> dict:
    """One epoch of the filter.  Exactly one of `factor` (theta = factor * D) and `theta` is given.
    Returns dist (per candidate), D, theta, send_idx (row numbers, ascending), send_buf and the
    updated copies L_new; E and L are not modified."""
    assert (factor is None) != (theta is None)
    cand = np.arange(E.shape[0], dtype=np.int64) if rows is None else np.asarray(rows, np.int64)
    dist = distances(E, L, cand)
    D = float(dist.max()) if dist.size else 0.0
    th = factor * D if theta is None else float(theta)
    send_idx = cand[dist > th]
    L_new = np.array(L, np.float64, copy=True)
    L_new[send_idx] = np.asarray(E, np.float64)[send_idx]
    return {"dist": dist, "D": D, "theta": th, "send_idx": send_idx,
            "send_buf": np.asarray(E, np.float64)[send_idx].copy(), "L_new": L_new}
