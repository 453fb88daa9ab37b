"""Comparison rules shared by the GPU parity tests.

Integer / bit results are compared exactly when both sides are given the same
floating-point inputs (staged tests).  End to end, the GPU rotates in fp32 and
the oracle in fp64, so a coordinate that lies within rounding of a cell
boundary may fall on the other side; the rules below accept exactly that and
nothing else.
"""
from __future__ import annotations

import math

import numpy as np

BOUNDARY_TOL = 1e-5   # |y - boundary| allowed for an index mismatch
MIN_AGREEMENT = 0.9999
REL_TOL = 1e-4        # floating-point outputs, relative to the natural scale


def _allowed_mismatches(size):
    """99.99 % agreement is a rate: below 10^4 decisions a single mismatch (which must still lie inside the
    band, checked separately) is under its resolution and is allowed."""
    return max(1, int(math.floor((1.0 - MIN_AGREEMENT) * size + 1e-9)))


def check_indices(idx_gpu, idx_or, y_or32, bounds32):
    """idx agreement >= 99.99 %; every mismatch is one bucket off and the
    oracle's y is within BOUNDARY_TOL of the boundary between the two."""
    idx_gpu = np.asarray(idx_gpu)
    idx_or = np.asarray(idx_or)
    bad = idx_gpu != idx_or
    frac = 1.0 - bad.mean() if bad.size else 1.0
    assert bad.sum() <= _allowed_mismatches(bad.size), f"index agreement {frac:.6f}"
    if bad.any():
        g, o_, y = idx_gpu[bad], idx_or[bad], np.asarray(y_or32, dtype=np.float64)[bad]
        assert np.all(np.abs(g - o_) == 1), "index mismatch by more than one bucket"
        b = np.asarray(bounds32, dtype=np.float64)[np.minimum(g, o_)]
        assert np.all(np.abs(y - b) <= BOUNDARY_TOL), f"mismatch away from a boundary: {np.max(np.abs(y - b))}"
    return frac


def check_signs(qjl_gpu, u_or, scale):
    """sign agreement >= 99.99 %; mismatches only where |u| <= 1e-5 * scale
    (scale = ||S_i|| * ||r|| per entry, broadcastable)."""
    qjl_gpu = np.asarray(qjl_gpu, dtype=bool)
    want = np.asarray(u_or) >= 0.0
    bad = qjl_gpu != want
    frac = 1.0 - bad.mean() if bad.size else 1.0
    assert bad.sum() <= _allowed_mismatches(bad.size), f"sign agreement {frac:.6f}"
    if bad.any():
        lim = 1e-5 * np.broadcast_to(scale, np.asarray(u_or).shape)[bad]
        assert np.all(np.abs(np.asarray(u_or)[bad]) <= lim), "sign mismatch away from zero"
    return frac


def check_close(got, want, scale, what="value", rel=REL_TOL):
    """|got - want| <= rel * (|want| + scale) elementwise."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    err = np.abs(got - want)
    lim = rel * (np.abs(want) + np.broadcast_to(scale, want.shape))
    worst = float(np.max(err / np.maximum(lim, 1e-300))) if err.size else 0.0
    assert worst <= 1.0, f"{what}: error {worst:.3f}x the tolerance (max abs err {err.max():.3e})"
    return worst


def check_topk(topk_gpu, scores_ref, k, scale):
    """Set equality after removing candidates whose reference score is within
    2e-4*scale of the cut between rank k and rank k+1; exact order where the
    neighbouring gaps exceed that."""
    scores_ref = np.asarray(scores_ref, dtype=np.float64)
    topk_gpu = np.asarray(topk_gpu)
    for r in range(scores_ref.shape[0]):
        s = scores_ref[r]
        tol = 2e-4 * float(np.broadcast_to(scale, (scores_ref.shape[0],))[r])
        order = np.argsort(-s, kind="stable")
        cut_hi, cut_lo = s[order[k - 1]], s[order[k]] if s.size > k else -math.inf
        sure = {int(i) for i in order[:k] if s[i] > cut_lo + tol}
        maybe = {int(i) for i in np.nonzero(s >= cut_hi - tol)[0]}
        got = [int(i) for i in topk_gpu[r]]
        assert len(set(got)) == k, "duplicate index in top-k"
        assert sure.issubset(set(got)), f"row {r}: a clear top-{k} member is missing"
        assert set(got).issubset(maybe | sure), f"row {r}: an index outside the candidates was returned"
        gs = s[got]
        assert np.all(gs[:-1] >= gs[1:] - tol), f"row {r}: top-k not in descending order"
