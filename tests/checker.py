"""Tie-aware comparison of a search result with the oracle's.

Top-k id sets must equal the oracle's except among ties, where scores agree within the
tolerance; returned scores must agree with the oracle's score of the same id.

Tolerance model (relative ``tol`` = 1e-4 for fp32 indexes, 2e-3 for fp16 indexes):
* returned scores: |g - o| <= tol * |o| for squared L2 -- the library hands back distances computed in the
  difference form, whose fp32 error is relative to the distance itself, so a distance of exactly zero must
  come back as zero --, and tol * |o| + ABS_EPS * |q| |x| for the inner product (fp32 accumulation of d
  products of either sign: the error is relative to sum |q_i x_i|, not to the possibly cancelling sum);
* which candidates make the list: the scan ranks squared L2 in the expanded form |x|^2 + |q|^2 - 2 q.x, whose
  fp32 error is proportional to the norms, not to the distance, so the tie band around the k-th score keeps
  an absolute term ABS_EPS * (|q|^2 + |x|^2) beside tol * |tau| (inner product: ABS_EPS * |q| |x|).
ABS_EPS = 4e-6 = 64 * 2^-24.

``strict`` mode: tolerance zero -- ids must equal the oracle's list exactly (same order,
ties by id) and scores must be equal as fp32 values (used where the arithmetic is exact).
"""
import numpy as np

METRIC_L2 = 0
METRIC_IP = 1
ABS_EPS = 4e-6


def tolerance_for(dtype_code: int) -> float:
    return 1e-4 if dtype_code == 0 else 2e-3


def score_allowance(metric, tol, oracle_scores, scale):
    """How far a returned score may be from the oracle's: purely relative for squared L2, relative plus the
    absolute term for the inner product (scale = |q| |x| per returned row)."""
    rel = tol * np.abs(oracle_scores)
    return rel if metric == METRIC_L2 else rel + ABS_EPS * scale


def _norm2(v):
    v = np.asarray(v, dtype=np.float64)
    return float((v * v).sum())


def check_result(q, base, metric, k, got_ids, got_dist, got_n, cand_ids, cand_scores,
                 tol, strict=False):
    """Raise AssertionError unless (got_ids, got_dist, got_n) is a valid answer.

    cand_ids / cand_scores: ALL candidates of the probed lists with their oracle scores, in
    the oracle's final order (best first, ties by id).  Returns the number of positions at
    which the returned id differs from the oracle's (all inside the tie band).
    """
    m = cand_ids.shape[0]
    want_n = min(k, m)
    assert got_n == want_n, f"n_out {got_n} != {want_n}"
    ids = np.asarray(got_ids[:got_n], dtype=np.int64)
    dist = np.asarray(got_dist[:got_n], dtype=np.float64)
    # padding of the tail
    pad = np.inf if metric == METRIC_L2 else -np.inf
    assert np.all(np.asarray(got_ids[got_n:k]) == -1), "tail ids must be -1"
    assert np.all(np.asarray(got_dist[got_n:k], dtype=np.float64) == pad), "tail scores must be +/-inf"
    if want_n == 0:
        return 0
    assert len(set(ids.tolist())) == got_n, "duplicate ids"
    order = np.argsort(cand_ids, kind="stable")
    sorted_ids = cand_ids[order]
    pos = np.searchsorted(sorted_ids, ids)
    assert np.all(pos < m) and np.all(sorted_ids[np.minimum(pos, m - 1)] == ids), \
        "returned id is not in a probed list"
    o_of_id = cand_scores[order][pos]

    if strict:
        assert np.array_equal(ids, cand_ids[:want_n]), "strict: ids differ from the oracle's"
        assert np.array_equal(dist.astype(np.float32), cand_scores[:want_n].astype(np.float32)), \
            "strict: scores differ from the oracle's"
        return 0

    qn2 = _norm2(q)
    xn2 = (base[ids].astype(np.float64) ** 2).sum(axis=1)
    scale = qn2 + xn2 if metric == METRIC_L2 else np.sqrt(qn2 * xn2)
    allowed = score_allowance(metric, tol, o_of_id, scale)
    err = np.abs(dist - o_of_id)
    assert np.all(err <= allowed), \
        f"score off by {err.max():.3e} (allowed {allowed[np.argmax(err)]:.3e}) for id {ids[np.argmax(err)]}"
    # returned order monotone (equal allowed)
    if metric == METRIC_L2:
        assert np.all(np.diff(dist) >= 0), "scores not ascending"
    else:
        assert np.all(np.diff(dist) <= 0), "scores not descending"
    # band around the oracle's k-th score
    tau = float(cand_scores[want_n - 1])
    band = tol * abs(tau) + ABS_EPS * float(np.max(scale))
    sign = 1.0 if metric == METRIC_L2 else -1.0
    # every candidate better than tau by more than the band must be present
    better = sign * (tau - cand_scores) > band
    must = set(cand_ids[better].tolist())
    missing = must - set(ids.tolist())
    assert not missing, f"{len(missing)} clearly-better candidates missing, e.g. id {next(iter(missing))}"
    # no returned id may be worse than tau by more than the band
    worse = sign * (o_of_id - tau) > band
    assert not worse.any(), f"id {ids[np.argmax(worse)]} is worse than the k-th score by more than the tie band"
    return int((ids != cand_ids[:want_n]).sum())


def probe_sets_equivalent(got_probe, want_probe, coarse_scores, metric, tol, scale_eps=0.0):
    """True if the probe sets are equal, or differ only by centroids whose fp64 coarse score
    lies within the tolerance band of the boundary (rank nprobe) score."""
    g, w = set(int(v) for v in got_probe), set(int(v) for v in want_probe)
    if g == w:
        return True
    if len(g) != len(w):
        return False
    boundary = float(coarse_scores[int(want_probe[-1])])
    band = tol * abs(boundary) + scale_eps
    for j in (g ^ w):
        if abs(float(coarse_scores[j]) - boundary) > band:
            return False
    return True
