"""CPU oracle of IVF search over product-quantised lists -- TEST INFRASTRUCTURE ONLY.

The paper (Sec. 1) names IVF with PQ-compressed lists beside IVF-Flat as the index family a vector pool serves; it
defines neither, so this is the textbook definition (product quantisation with asymmetric distance computation):

  * the d coordinates are cut into M consecutive sub-vectors of d/M coordinates; sub-space m has a codebook of
    `ksub` entries (rows of d/M values);
  * the code of a stored vector is, per sub-space, the number of the codebook entry nearest (squared L2) to its
    sub-vector, ties to the smaller number; its *reconstruction* is the concatenation of those entries;
  * the score of a query against a stored vector is the metric -- squared L2, ascending, or inner product,
    descending -- between the QUERY ITSELF (not quantised: "asymmetric") and the reconstruction;
  * which vectors are candidates is decided as in IVF-Flat: the nprobe best centroids by the query's metric, every
    vector of their lists; the answer is the k best candidates by (score, id).

Readings where the definition leaves a choice: the sub-vectors are those of the stored vector itself, not of its
residual to the list's centroid (both are in use; this one makes the query's per-sub-space tables independent of the
list); codebook training is Lloyd's algorithm per sub-space on the sub-vectors, an empty cell keeps its entry.

Everything here is written as the definition reads: reconstruct, then take the metric, in fp64.  No tables, no
blocking.  Candidate enumeration and the probe set come from the IVF-Flat oracle (same package).
"""
from __future__ import annotations

import numpy as np

import oracle

METRIC_L2 = 0
METRIC_IP = 1


def _sub(x: np.ndarray, m: int, M: int) -> np.ndarray:
    d = x.shape[-1]
    assert d % M == 0
    w = d // M
    return x[..., m * w:(m + 1) * w]


def encode(X: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """codes[i, m] = number of the entry of codebooks[m] nearest to sub-vector m of X[i] (ties: the smaller number).
    codebooks: [M, ksub, d/M]."""
    M, ksub, w = codebooks.shape
    X = np.asarray(X, dtype=np.float64)
    assert X.shape[1] == M * w
    codes = np.zeros((X.shape[0], M), dtype=np.uint8 if ksub <= 256 else np.uint16)
    for m in range(M):
        sub = _sub(X, m, M)                                                   # [n, w]
        d2 = ((sub[:, None, :] - codebooks[m].astype(np.float64)[None, :, :]) ** 2).sum(axis=2)
        codes[:, m] = np.argmin(d2, axis=1)                                   # (argmin returns the first minimum)
    return codes


def decode(codes: np.ndarray, codebooks: np.ndarray) -> np.ndarray:
    """The reconstructions, fp64 [n, d]."""
    M = codebooks.shape[0]
    return np.concatenate([codebooks[m].astype(np.float64)[codes[:, m].astype(np.int64)] for m in range(M)], axis=1)


def scores(q: np.ndarray, codes: np.ndarray, codebooks: np.ndarray, metric: int) -> np.ndarray:
    """Score of the query against every coded vector: the metric between q and the reconstruction."""
    xhat = decode(codes, codebooks)
    qq = np.asarray(q, dtype=np.float64)
    if metric == METRIC_L2:
        return ((xhat - qq[None, :]) ** 2).sum(axis=1)
    return (xhat * qq[None, :]).sum(axis=1)


def train(X: np.ndarray, init: np.ndarray, iters: int) -> np.ndarray:
    """Lloyd's algorithm per sub-space from the given initial codebooks [M, ksub, d/M]; an empty cell keeps its entry."""
    cb = np.array(init, dtype=np.float64)
    M = cb.shape[0]
    X = np.asarray(X, dtype=np.float64)
    for _ in range(iters):
        codes = encode(X, cb)
        for m in range(M):
            sub = _sub(X, m, M)
            for c in range(cb.shape[1]):
                members = sub[codes[:, m] == c]
                if members.shape[0]:
                    cb[m, c] = members.mean(axis=0)
    return cb


def quantisation_error(X: np.ndarray, codes: np.ndarray, codebooks: np.ndarray) -> float:
    """Mean squared distance between the vectors and their reconstructions."""
    return float(((np.asarray(X, dtype=np.float64) - decode(codes, codebooks)) ** 2).sum(axis=1).mean())


def candidates(index: "oracle.Index", probe: np.ndarray):
    """Stored positions (list-major) and ids of every vector of the probed lists, list after list."""
    pos = np.concatenate([np.arange(int(index.list_off[l]), int(index.list_off[l + 1]), dtype=np.int64) for l in probe]
                         + [np.zeros(0, dtype=np.int64)])
    return pos, index.list_ids[pos]


def search(index: "oracle.Index", codes_listmajor: np.ndarray, codebooks: np.ndarray, q: np.ndarray, k: int, nprobe: int,
           metric: int, probe: np.ndarray = None, all_candidates: bool = False):
    """One query.  codes_listmajor[p] is the code of the vector stored at position p (its id is index.list_ids[p]).
    Returns (probe, ids[k] int64 (-1 padded), dist[k] fp64 (+inf / -inf padded), n_out[, cand_ids, cand_scores])."""
    if probe is None:
        probe = oracle.probe_set(oracle.coarse_scores(index, q, metric), nprobe, metric)
    pos, ids = candidates(index, probe)
    sc = scores(q, codes_listmajor[pos], codebooks, metric) if pos.shape[0] else np.zeros(0)
    order = np.lexsort((ids, sc if metric == METRIC_L2 else -sc))
    n = min(k, order.shape[0])
    out_ids = np.full(k, -1, dtype=np.int64)
    out_dist = np.full(k, np.inf if metric == METRIC_L2 else -np.inf, dtype=np.float64)
    out_ids[:n] = ids[order[:n]]
    out_dist[:n] = sc[order[:n]]
    if all_candidates:
        return probe, out_ids, out_dist, n, ids[order], sc[order]
    return probe, out_ids, out_dist, n


def search_reranked(index: "oracle.Index", codes_listmajor: np.ndarray, codebooks: np.ndarray, q: np.ndarray, k: int, k_adc: int,
                    nprobe: int, metric: int, probe: np.ndarray = None):
    """Two stages, as a deployment runs them: the k_adc best by reconstruction score (above), then those are scored
    exactly against the stored vectors themselves (fp64) and the k best by (exact score, id) are the answer.
    Returns (probe, ids[k], dist[k], n_out, stage1_ids, stage1_scores) -- the last two for every candidate, in stage-1
    order, so that a checker can tell what was clearly in, clearly out, or at the boundary of the short list."""
    probe, _, _, _, cand_ids, cand_sc = search(index, codes_listmajor, codebooks, q, k_adc, nprobe, metric, probe=probe,
                                               all_candidates=True)
    short = cand_ids[:k_adc]
    x = index.base[short].astype(np.float64)
    qq = np.asarray(q, dtype=np.float64)
    exact = ((x - qq[None, :]) ** 2).sum(axis=1) if metric == METRIC_L2 else (x * qq[None, :]).sum(axis=1)
    order = np.lexsort((short, exact if metric == METRIC_L2 else -exact))
    n = min(k, order.shape[0])
    out_ids = np.full(k, -1, dtype=np.int64)
    out_dist = np.full(k, np.inf if metric == METRIC_L2 else -np.inf, dtype=np.float64)
    out_ids[:n] = short[order[:n]]
    out_dist[:n] = exact[order[:n]]
    return probe, out_ids, out_dist, n, cand_ids, cand_sc
