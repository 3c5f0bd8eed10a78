"""Exact brute-force kNN (the ground truth of the paper's accuracy measure), the
accuracy measure itself (eqs. (2)-(3)) and graph invariants.  Test infrastructure."""
from __future__ import annotations

import numpy as np


def exact_knn_definition(X, K: int):
    """The definition written out: all pairwise squared distances in float64 by
    direct differences, self excluded, ordered by (distance, id).  O(n^2 d)
    memory-light loops over rows; only for small n."""
    X = np.asarray(X, dtype=np.float64)
    n = X.shape[0]
    ids = np.empty((n, K), dtype=np.int64)
    dists = np.empty((n, K), dtype=np.float64)
    for i in range(n):
        diff = X - X[i]
        dd = np.einsum("ij,ij->i", diff, diff)
        dd[i] = np.inf
        order = np.lexsort((np.arange(n), dd))[:K]
        ids[i] = order
        dists[i] = dd[order]
    return ids, dists


def exact_knn(X, rows, K: int, block: int = 256, slack: int = 32):
    """Exact K nearest neighbours of the given rows among all rows of X.

    Candidates are shortlisted with a float64 Gram-matrix form, then their
    distances are recomputed by direct differences in float64 and ordered by
    (distance, id), so the result does not carry the cancellation error of the
    shortlist step."""
    X32 = np.asarray(X)
    n, d = X32.shape
    rows = np.asarray(rows, dtype=np.int64)
    Xd = X32.astype(np.float64)
    norms = np.einsum("ij,ij->i", Xd, Xd)
    m = min(n - 1, K + slack)
    out_ids = np.empty((rows.shape[0], K), dtype=np.int64)
    out_d = np.empty((rows.shape[0], K), dtype=np.float64)
    for r0 in range(0, rows.shape[0], block):
        rr = rows[r0:r0 + block]
        G = Xd[rr] @ Xd.T
        G *= -2.0
        G += norms[None, :]
        G += norms[rr][:, None]
        G[np.arange(rr.shape[0]), rr] = np.inf
        short = np.argpartition(G, m - 1, axis=1)[:, :m]
        for a, i in enumerate(rr):
            c = np.sort(short[a])
            diff = Xd[c] - Xd[i]
            dd = np.einsum("ij,ij->i", diff, diff)
            order = np.lexsort((c, dd))[:K]
            out_ids[r0 + a] = c[order]
            out_d[r0 + a] = dd[order]
    return out_ids, out_d


def recall(approx_ids, true_ids) -> float:
    """Eq. (3): sum_i |R'_i n R_i| / (N K).  Empty slots (-1) count as misses."""
    approx_ids = np.asarray(approx_ids)
    true_ids = np.asarray(true_ids)
    assert approx_ids.shape == true_ids.shape
    hit = 0
    for a, t in zip(approx_ids, true_ids):
        hit += np.intersect1d(a[a >= 0], t).shape[0]
    return hit / float(true_ids.size)


def check_graph_invariants(X, ids, dists, rows=None, rtol: float = 1e-5):
    """Raise AssertionError unless every list is sorted by (dist, id), has no
    self loop, no duplicate id, empties (-1, +inf) only at the tail, and every
    stored distance equals the float64 squared L2 distance to relative rtol."""
    X = np.asarray(X)
    ids = np.asarray(ids)
    dists = np.asarray(dists)
    n_rows, K = ids.shape
    rows = np.arange(n_rows) if rows is None else np.asarray(rows)
    live = ids >= 0
    assert np.all(live[:, :-1] >= live[:, 1:]), "empty slot before a live one"
    assert np.all(np.isinf(dists[~live])), "empty slot without +inf"
    assert np.all(ids[live] < X.shape[0])
    assert not np.any(ids == rows[:, None]), "self loop"
    srt = np.sort(np.where(live, ids, -1 - np.arange(K)[None, :]), axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1]), "duplicate id"
    d0, d1 = dists[:, :-1], dists[:, 1:]
    i0, i1 = ids[:, :-1], ids[:, 1:]
    both = live[:, :-1] & live[:, 1:]
    ok = (d0 < d1) | ((d0 == d1) & (i0 < i1))
    assert np.all(ok | ~both), "list not sorted by (dist, id)"
    Xd = X.astype(np.float64)
    for r0 in range(0, n_rows, 4096):
        sl = slice(r0, min(n_rows, r0 + 4096))
        nb = np.where(live[sl], ids[sl], 0)
        diff = Xd[nb] - Xd[rows[sl]][:, None, :]
        ref = np.einsum("rkj,rkj->rk", diff, diff)
        got = dists[sl].astype(np.float64)
        err = np.abs(got - ref) <= rtol * ref
        assert np.all(err | ~live[sl]), "stored distance differs from float64 recomputation"
