"""Exact k-nearest neighbours and recall (TEST INFRASTRUCTURE ONLY).

Recall@K is the fraction of true nearest neighbours found among the K returned
results (Section 4.2.1).  Parity status: pinned by a pure-Python double loop on
tiny inputs (tests/test_oracle_search.py)."""
from __future__ import annotations

import numpy as np


def exact_knn(X: np.ndarray, Q: np.ndarray, k: int, metric: str = "l2", chunk: int = 256):
    """ids [nq,k] i64 and scores [nq,k] f64 (squared L2 ascending, or inner
    product descending); ties go to the lower id."""
    X64 = np.asarray(X, np.float64)
    xn = np.einsum("ij,ij->i", X64, X64)
    ids = np.empty((Q.shape[0], k), np.int64)
    sc = np.empty((Q.shape[0], k), np.float64)
    for s in range(0, Q.shape[0], chunk):
        q = np.asarray(Q[s:s + chunk], np.float64)
        dot = q @ X64.T
        if metric == "l2":
            key = np.einsum("ij,ij->i", q, q)[:, None] + xn[None, :] - 2.0 * dot
        else:
            key = -dot
        part = np.argpartition(key, min(k, key.shape[1] - 1), axis=1)[:, :k] if k < key.shape[1] else \
            np.tile(np.arange(key.shape[1]), (key.shape[0], 1))
        for r in range(key.shape[0]):
            kk = key[r]
            kth = np.max(kk[part[r]])
            cand = np.nonzero(kk <= kth)[0]  # includes every tie of the k-th value
            o = cand[np.lexsort((cand, kk[cand]))][:k]
            ids[s + r] = o
            sc[s + r] = kk[o] if metric == "l2" else -kk[o]
    return ids, sc


def recall_at_k(found: np.ndarray, truth: np.ndarray) -> float:
    """Mean over queries of |found ∩ truth| / K."""
    k = truth.shape[1]
    hit = 0
    for f, t in zip(found, truth):
        hit += np.intersect1d(f[f >= 0], t).shape[0]
    return hit / (truth.shape[0] * k)
