"""Exact filtered kNN straight from the problem definition (Section 3, Def. 1),
written in numpy fp64 independently of the oracle.  Used to pin the oracle and to
spot-check ground truth."""
import numpy as np


def membership(label_offsets, label_ids, n_labels):
    """bool [n, n_labels]: point i carries label l."""
    n = len(label_offsets) - 1
    m = np.zeros((n, n_labels), dtype=bool)
    owner = np.repeat(np.arange(n), np.diff(label_offsets))
    m[owner, label_ids] = True
    return m


def filtered_knn(vectors, member, q, qlabels, k, restrict=None):
    """Top-k (ids ascending by (distance, id), distances) among points carrying
    every label in qlabels.  restrict: optional array of candidate ids."""
    ok = np.ones(member.shape[0], dtype=bool)
    for l in qlabels:
        ok &= member[:, l]
    cand = np.flatnonzero(ok)
    if restrict is not None:
        cand = np.intersect1d(cand, restrict)
    d = ((vectors[cand].astype(np.float64) - q.astype(np.float64)[None, :]) ** 2).sum(axis=1)
    order = np.lexsort((cand, d))[:k]
    ids = np.full(k, -1, dtype=np.int64)
    dist = np.full(k, np.inf, dtype=np.float64)
    ids[:len(order)] = cand[order]
    dist[:len(order)] = d[order]
    return ids, dist


def recall_at_k(found_ids, true_ids):
    """Eq. (1): |A ∩ GT| / K with K replaced by |GT| when fewer than K points
    match; queries with no match are skipped."""
    num = den = 0
    for f, t in zip(found_ids, true_ids):
        t = t[t >= 0]
        if len(t) == 0:
            continue
        num += len(np.intersect1d(f[f >= 0], t))
        den += len(t)
    return num / max(den, 1)
