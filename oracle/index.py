"""Oracle-side index handling -- TEST INFRASTRUCTURE ONLY (see package docstring).

* ``build_index``: the oracle's own plain IVF-Flat construction from given centroids
  (assignment to the best centroid in fp64, lists in ascending row order), optionally
  preceded by Lloyd iterations.  Used to search without any GPU and to compare the
  clustering objective of an index built elsewhere.  k-means amplifies rounding, so an
  index built elsewhere is never compared bit by bit: parity of the build is UNPINNED
  beyond ``check_index`` and the objective comparison.
* ``check_index``: validates an exported index (partition of the rows, monotone offsets,
  every checked row stored in the list of its best centroid or of one within tolerance).

Pins (tests/test_index_oracle_pins.py, tests/golden/index_examples.json): ``lloyd`` and
``inertia`` against hand-worked iterations (an empty cluster, the spherical variant) and
against scipy's k-means on separated blobs; ``assign_rows`` against hand cases with tied
centroids and an enumeration in Python integers; ``partition`` against counted lists;
``build_index`` against the lists of the hand-worked search examples; ``check_index`` against
planted faults (wrong list, worst list, duplicated id, broken offsets, a near-tie on either
side of the tolerance); and mutated copies of this file, which must fail those pins.
"""
from __future__ import annotations

import numpy as np

from . import Index, METRIC_IP, METRIC_L2


def _scores_fp64(rows: np.ndarray, centroids: np.ndarray, metric: int) -> np.ndarray:
    """[m, nlist] fp64 scores.  L2 by the difference form, IP by the dot product."""
    r = rows.astype(np.float64)
    c = centroids.astype(np.float64)
    if metric == METRIC_IP:
        return r @ c.T
    out = np.empty((r.shape[0], c.shape[0]), dtype=np.float64)
    for j in range(c.shape[0]):
        diff = r - c[j]
        out[:, j] = np.einsum("ij,ij->i", diff, diff)
    return out


def assign_rows(base: np.ndarray, centroids: np.ndarray, metric: int, chunk: int = 4096) -> np.ndarray:
    """Best centroid per row (L2 smallest / IP largest), ties -> smaller centroid number."""
    n = base.shape[0]
    out = np.empty(n, dtype=np.int64)
    for s in range(0, n, chunk):
        sc = _scores_fp64(base[s:s + chunk], centroids, metric)
        out[s:s + chunk] = np.argmin(sc, axis=1) if metric == METRIC_L2 else np.argmax(sc, axis=1)
    return out


def lloyd(base: np.ndarray, init_centroids: np.ndarray, iters: int, metric: int) -> np.ndarray:
    """Plain Lloyd iterations in fp64.  L2: centroid = mean of its rows.  IP: spherical
    k-means (centroid = mean, then normalised).  An empty cluster keeps its centroid."""
    c = init_centroids.astype(np.float64).copy()
    x = base.astype(np.float64)
    for _ in range(iters):
        a = assign_rows(base, c, metric)
        for j in range(c.shape[0]):
            members = x[a == j]
            if members.shape[0] == 0:
                continue
            m = members.mean(axis=0)
            if metric == METRIC_IP:
                nrm = np.sqrt((m * m).sum())
                if nrm > 0:
                    m = m / nrm
            c[j] = m
    return c


def partition(assignment: np.ndarray, nlist: int):
    """(list_off uint64[nlist+1], list_ids int64[n]); rows of a list in ascending order."""
    order = np.argsort(assignment, kind="stable").astype(np.int64)
    counts = np.bincount(assignment, minlength=nlist).astype(np.uint64)
    off = np.zeros(nlist + 1, dtype=np.uint64)
    off[1:] = np.cumsum(counts)
    return off, order


def build_index(base: np.ndarray, centroids: np.ndarray, metric: int, train_iters: int = 0) -> Index:
    """The oracle's own index: optional Lloyd from the given centroids, centroids rounded
    to the storage precision of the base (so they are values an fp16 index can hold),
    then assignment and partition."""
    c = lloyd(base, centroids, train_iters, metric) if train_iters else centroids.astype(np.float64)
    c_stored = c.astype(base.dtype).astype(np.float32)
    a = assign_rows(base, c_stored, metric)
    off, ids = partition(a, c_stored.shape[0])
    return Index(base, c_stored, off, ids)


def inertia(base: np.ndarray, index: Index, metric: int) -> float:
    """Clustering objective of the partition: L2 -> sum of squared distances of each row to
    its list's centroid; IP -> sum of (1 - dot) (both smaller = better)."""
    total = 0.0
    c = index.centroids.astype(np.float64)
    for j in range(index.nlist):
        rows = index.list_ids[int(index.list_off[j]):int(index.list_off[j + 1])]
        if rows.size == 0:
            continue
        x = base[rows].astype(np.float64)
        if metric == METRIC_L2:
            diff = x - c[j]
            total += float((diff * diff).sum())
        else:
            total += float((1.0 - x @ c[j]).sum())
    return total


def check_index(index: Index, build_metric: int, tol: float, sample: int = 0, seed: int = 0) -> dict:
    """Validate an exported index.  Raises AssertionError on a structural fault.

    Structural (always, all rows): offsets start at 0, are non-decreasing and end at n; the id
    array is a permutation of 0..n-1.  Assignment (all rows, or ``sample`` seeded rows): the
    list a row is stored in has the best fp64 score among all centroids under the build
    metric, or one within ``tol`` relative (scale max(|best|, |own|)) of the best.
    Returns counts: rows checked, exact-best rows, near-tie rows.
    """
    n, nlist = index.n, index.nlist
    off = index.list_off
    assert int(off[0]) == 0, "list_off[0] != 0"
    assert int(off[-1]) == n, "list_off[nlist] != n"
    assert np.all(off[1:] >= off[:-1]), "list_off not monotone"
    seen = np.zeros(n, dtype=np.uint8)
    ids = index.list_ids
    assert ids.min(initial=0) >= 0 and ids.max(initial=0) < n, "id out of range"
    np.add.at(seen, ids, 1)
    assert np.all(seen == 1), "ids are not a permutation of the rows"
    list_of_row = np.empty(n, dtype=np.int64)
    list_of_row[ids] = np.repeat(np.arange(nlist, dtype=np.int64), np.diff(off).astype(np.int64))

    rows = np.arange(n, dtype=np.int64)
    if sample and sample < n:
        rows = np.sort(np.random.default_rng(seed).choice(n, size=sample, replace=False))
    exact = near = 0
    for s in range(0, rows.size, 2048):
        r = rows[s:s + 2048]
        sc = _scores_fp64(index.base[r], index.centroids, build_metric)
        own = sc[np.arange(r.size), list_of_row[r]]
        best = sc.min(axis=1) if build_metric == METRIC_L2 else sc.max(axis=1)
        gap = np.abs(own - best)
        scale = np.maximum(np.maximum(np.abs(best), np.abs(own)), 1e-30)
        is_exact = gap == 0
        is_near = (~is_exact) & (gap <= tol * scale)
        bad = ~(is_exact | is_near)
        assert not bad.any(), (f"{int(bad.sum())} rows stored in a list that is not their best centroid "
                               f"(first row {int(r[np.argmax(bad)])})")
        exact += int(is_exact.sum())
        near += int(is_near.sum())
    return dict(checked=int(rows.size), exact=exact, near_tie=near)
