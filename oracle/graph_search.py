"""CPU oracle of the paper's own engine: best-first search over a fixed-degree neighbour graph,
advanced one "extend" at a time -- TEST INFRASTRUCTURE ONLY.

Paper Sec. 3.2: the database X (N x d) and a fixed-degree neighbour list G (N x D) are resident; a
request keeps a candidate list topM (ids and distances) and a visited table that admits only
first-seen candidates to the distance computation.  One extend of a request: select up to p
non-expanded parents from its topM, read the D neighbours of each, filter by visited, compute the
distances of the survivors, merge them into topM, mark the consumed parents expanded.  A request
stops on its own when an extend leaves the candidates of topM unchanged.

The paper is silent on the following; the readings taken here (and by the HIP path) are:
  * how a request starts: from a list of entry points given with the index (`seeds`); they are scored
    and form the first topM before the first extend (this is not counted as an extend);
  * which parents: the first p non-expanded entries of topM in its order (best first);
  * order of topM and ties: by (score, id), L2 ascending, inner product descending;
  * L2 is the squared distance; scores are the sums over the stored values in fp64, as the definition has
    them (on integer-valued data that is exact, and equals what fp32 arithmetic in any order gives);
  * a search is a chain of decisions -- which candidates enter topM, in which order, hence which parents are
    expanded next -- each taken on scores.  search() also reports `min_gap`, the smallest relative difference
    between two neighbouring scores at any of those decisions (among the first topM + 1 candidates of every
    merge): an implementation whose scores are within a relative error well below min_gap of these must take
    every decision the same way and arrive at the same trajectory; below that, near-ties may legitimately be
    ordered differently;
  * a request also stops when topM holds no non-expanded entry, or after max_iters extends;
  * neighbour entries >= N are padding and skipped;
  * the answer is the first k entries of topM.

Written as the steps above, one request at a time, no batching.  Plain numpy; fp64 sums.
"""
from __future__ import annotations

import numpy as np

METRIC_L2 = 0
METRIC_IP = 1


def scores(X: np.ndarray, ids, q: np.ndarray, metric: int) -> np.ndarray:
    """Score of q against the rows `ids` of X: fp64 sum over the stored values."""
    x = X[np.asarray(ids, dtype=np.int64)].astype(np.float64)
    qq = q.astype(np.float64)
    if metric == METRIC_L2:
        return ((x - qq[None, :]) ** 2).sum(axis=1)
    return (x * qq[None, :]).sum(axis=1)


def _decision_gap(ids, sc, order, topm):
    """Smallest relative difference between neighbouring scores among the first topm + 1 candidates in
    `order` (what decides membership of topM and the order inside it).  Equal scores of different rows count
    as a gap of zero."""
    head = [int(i) for i in order[:topm + 1]]
    gap = np.inf
    for a, b in zip(head[:-1], head[1:]):
        sa, sb = float(sc[a]), float(sc[b])
        gap = min(gap, abs(sa - sb) / max(abs(sa), abs(sb), 1e-300))
    return gap


def _order(ids, sc, metric):
    """Indices that sort candidates best first, ties by ascending id."""
    key = np.asarray(sc, dtype=np.float64)
    if metric == METRIC_IP:
        key = -key
    return np.lexsort((np.asarray(ids, dtype=np.int64), key))


def search(X: np.ndarray, G: np.ndarray, seeds, q: np.ndarray, k: int, topm: int, p: int, max_iters: int,
           metric: int, trace: bool = False):
    """One request.  Returns dict(ids[k] int64 (-1 padded), dist[k] fp64, n, iters, evals, min_gap[, trace])."""
    n, D = G.shape
    assert 1 <= k <= topm and p >= 1
    visited = np.zeros(n, dtype=bool)
    # start: the entry points, first-seen only
    cand = []
    for s in seeds:
        s = int(s)
        if s < n and not visited[s]:
            visited[s] = True
            cand.append(s)
    evals = len(cand)
    sc = scores(X, cand, q, metric) if cand else np.zeros(0, dtype=np.float64)
    o = _order(cand, sc, metric)
    min_gap = _decision_gap(cand, sc, o, topm)
    o = o[:topm]
    top_ids = [cand[i] for i in o]
    top_sc = [sc[i] for i in o]
    top_exp = [False] * len(top_ids)
    steps = [dict(ids=list(top_ids), dist=[float(v) for v in top_sc])] if trace else None
    iters = 0
    while iters < max_iters:
        parents = [i for i, e in enumerate(top_exp) if not e][:p]
        if not parents:
            break
        iters += 1
        cand = []
        for i in parents:
            top_exp[i] = True
            for v in G[top_ids[i]]:
                v = int(v)
                if v < n and not visited[v]:
                    visited[v] = True
                    cand.append(v)
        evals += len(cand)
        sc = scores(X, cand, q, metric) if cand else np.zeros(0, dtype=np.float64)
        all_ids = top_ids + cand
        all_sc = list(top_sc) + list(sc)
        all_exp = top_exp + [False] * len(cand)
        o = _order(all_ids, all_sc, metric)
        min_gap = min(min_gap, _decision_gap(all_ids, all_sc, o, topm))
        o = o[:topm]
        new_ids = [all_ids[i] for i in o]
        changed = set(new_ids) != set(top_ids)
        top_ids, top_sc, top_exp = new_ids, [all_sc[i] for i in o], [all_exp[i] for i in o]
        if trace:
            steps.append(dict(ids=list(top_ids), dist=[float(v) for v in top_sc]))
        if not changed:
            break
    m = min(k, len(top_ids))
    ids = np.full(k, -1, dtype=np.int64)
    dist = np.full(k, np.inf if metric == METRIC_L2 else -np.inf, dtype=np.float64)
    ids[:m] = top_ids[:m]
    dist[:m] = top_sc[:m]
    out = dict(ids=ids, dist=dist, n=m, iters=iters, evals=evals, min_gap=float(min_gap))
    if trace:
        out["trace"] = steps
    return out
