"""Exact k-nearest-neighbour search by brute force in numpy -- independent of the oracle.

Used only to pin the oracle (with nprobe = nlist an IVF search is exact kNN) and as recall
ground truth.  Scores come from one matrix product on fp64 copies (L2 through the expanded
form, which on integer-valued or small inputs is exact in fp64) and rows are ordered with
numpy's lexsort on (id, score): a different formula, a different sort and a different
language from the oracle's C loops.
"""
import numpy as np

METRIC_L2 = 0
METRIC_IP = 1


def knn(base: np.ndarray, queries: np.ndarray, k: int, metric: int):
    """(ids [nq, k] int64, scores [nq, k] float64), best first, ties -> smaller id."""
    x = base.astype(np.float64)
    q = queries.astype(np.float64)
    dots = q @ x.T
    if metric == METRIC_L2:
        sc = (q * q).sum(1)[:, None] + (x * x).sum(1)[None, :] - 2.0 * dots
        key = sc
    else:
        sc = dots
        key = -dots
    n = x.shape[0]
    kk = min(k, n)
    ids = np.empty((q.shape[0], kk), dtype=np.int64)
    out = np.empty((q.shape[0], kk), dtype=np.float64)
    row_ids = np.arange(n)
    for i in range(q.shape[0]):
        order = np.lexsort((row_ids, key[i]))[:kk]
        ids[i] = order
        out[i] = sc[i, order]
    return ids, out


def recall_at_k(found_ids: np.ndarray, true_ids: np.ndarray) -> float:
    """Mean over queries of |found ∩ true| / |true| (ids < 0 in ``found`` are padding)."""
    hits = 0
    total = 0
    for f, t in zip(found_ids, true_ids):
        hits += len(set(int(v) for v in f if v >= 0) & set(int(v) for v in t))
        total += len(t)
    return hits / max(total, 1)
