"""Parity rule between the GPU result and the oracle (shared by the GPU tests and bench).

The paper does not say which of several near-equal neighbours is "the" answer, so what is
unique is compared exactly and the rest is checked for validity:
  set rule       where the oracle's relative gap behind the k-th neighbour exceeds 1e-4 (or
                 k == n) the index SET of the row must equal the oracle's;
  position rule  position p must hold the oracle's index wherever the gaps on both sides of
                 the oracle's p-th distance exceed 1e-4 relative;
  always         distances agree position by position within 1e-4 relative + 1e-5 absolute;
                 every reported (index, distance) pair is consistent with the oracle's fp64
                 distance of that pair; indices of a row are distinct and in range.
"""
from __future__ import annotations

import numpy as np

REL = 1e-4
ABS = 1e-5
TINY = 1e-30


def check(idx_gpu, dist_gpu, o_idx, o_dist, o_next, n, pair_dist=None):
    """Arrays are [r, k] for the same rows.  Returns a dict of counts; raises on violation.

    pair_dist: optional callable (rows_local, cols) -> fp64 oracle distance of the GPU's own
    (row, idx) pairs, used for the consistency check.
    """
    idx_gpu = np.asarray(idx_gpu).astype(np.int64)
    dist_gpu = np.asarray(dist_gpu).astype(np.float64)
    r, k = o_idx.shape
    assert idx_gpu.shape == (r, k) and dist_gpu.shape == (r, k)
    assert idx_gpu.min(initial=0) >= 0 and idx_gpu.max(initial=0) < n, "index out of range"
    srt = np.sort(idx_gpu, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1]), "duplicate index inside a row"
    assert np.all(dist_gpu >= 0), "negative distance"
    assert np.all(np.diff(dist_gpu, axis=1) >= 0), "row not ascending"
    tol = REL * o_dist + ABS
    bad = np.abs(dist_gpu - o_dist) > tol
    assert not bad.any(), f"distance mismatch at {np.argwhere(bad)[:5].tolist()}"
    if pair_dist is not None:
        own = pair_dist(idx_gpu)
        bad = np.abs(dist_gpu - own) > REL * own + ABS
        assert not bad.any(), "reported distance inconsistent with its own index"

    gap_k = (o_next - o_dist[:, -1]) / np.maximum(o_dist[:, -1], TINY)
    set_rows = (gap_k > REL) | np.isinf(o_next)
    set_ok = np.array([set(a) == set(b) for a, b in zip(idx_gpu[set_rows], o_idx[set_rows])],
                      dtype=bool)
    assert set_ok.all(), f"index set differs on {int((~set_ok).sum())} rows with a clear k-th gap"

    # gaps between consecutive oracle distances, with the (k+1)-th appended
    ext = np.concatenate([o_dist, o_next[:, None]], axis=1)
    gap_after = (ext[:, 1:] - ext[:, :-1]) / np.maximum(ext[:, :-1], TINY)  # [r, k]
    gap_after = np.where(np.isinf(ext[:, 1:]), np.inf, gap_after)
    clear_after = gap_after > REL
    clear_before = np.concatenate([np.ones((r, 1), dtype=bool), clear_after[:, :-1]], axis=1)
    must_match = clear_after & clear_before
    pos_bad = must_match & (idx_gpu != o_idx)
    assert not pos_bad.any(), f"position rule violated at {np.argwhere(pos_bad)[:5].tolist()}"

    strict = np.all(idx_gpu == o_idx, axis=1)
    return {
        "rows": int(r),
        "set_rule_rows": int(set_rows.sum()),
        "position_rule_entries": int(must_match.sum()),
        "strict_rows": int(strict.sum()),
        "max_rel_dist_err": float(np.max(np.abs(dist_gpu - o_dist) / np.maximum(o_dist, 1e-12)))
        if r * k else 0.0,
    }
