"""Pins of the product-quantisation oracle (oracle/pq.py) against things that are not that oracle: a hand-worked
example, the table-sum route to the same scores written out here, a lossless case in which the IVF-Flat oracle (pinned
on its own) must give the same answers, brute force over all codes, and planted mistakes that must fail a pin."""
import itertools
import json
import os

import numpy as np
import pytest

import oracle
from oracle import pq as opq

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "pq_examples.json")))["example"]


def _gold():
    cb = np.array(GOLD["codebooks"], dtype=np.float64)
    X = np.array(GOLD["vectors"], dtype=np.float64)
    q = np.array(GOLD["query"], dtype=np.float64)
    return cb, X, q


def _check_gold(mod):
    cb, X, q = _gold()
    codes = mod.encode(X, cb)
    assert codes.tolist() == GOLD["codes"]
    assert np.array_equal(mod.decode(codes, cb), np.array(GOLD["reconstructions"], dtype=np.float64))
    assert np.allclose(mod.scores(q, codes, cb, 0), GOLD["l2"], rtol=0, atol=1e-12)
    assert np.allclose(mod.scores(q, codes, cb, 1), GOLD["ip"], rtol=0, atol=1e-12)
    assert abs(mod.quantisation_error(X, codes, cb) - GOLD["quantisation_error"]) < 1e-12
    assert np.allclose(mod.train(X, cb, 1), np.array(GOLD["after_one_lloyd_iteration"]), rtol=0, atol=1e-12)
    idx = oracle.Index(X.astype(np.float32), np.zeros((1, 4), dtype=np.float32), [0, 5], np.arange(5))
    for metric, want in ((0, GOLD["top3_l2_ids"]), (1, GOLD["top3_ip_ids"])):
        _, ids, dist, n = mod.search(idx, codes, cb, q.astype(np.float32), 3, 1, metric)
        assert n == 3 and ids.tolist() == want
    _, ids, dist, n = mod.search(idx, codes, cb, q.astype(np.float32), 8, 1, 0)
    assert n == 5 and ids[5:].tolist() == [-1, -1, -1] and np.all(np.isinf(dist[5:]))


def test_hand_worked_example():
    _check_gold(opq)


def test_scores_equal_the_sum_of_per_subspace_table_entries():
    """The route every implementation takes -- one table per sub-space of the query's partial scores against the
    codebook entries, summed over the code -- written out here, against the oracle's reconstruct-then-score."""
    rng = np.random.default_rng(5)
    M, ksub, w, n = 6, 16, 3, 200
    cb = rng.normal(size=(M, ksub, w))
    codes = rng.integers(0, ksub, size=(n, M)).astype(np.uint8)
    q = rng.normal(size=M * w)
    for metric in (0, 1):
        table = np.zeros((M, ksub))
        for m in range(M):
            qm = q[m * w:(m + 1) * w]
            for c in range(ksub):
                table[m, c] = ((qm - cb[m, c]) ** 2).sum() if metric == 0 else (qm * cb[m, c]).sum()
        by_table = np.array([sum(table[m, codes[i, m]] for m in range(M)) for i in range(n)])
        assert np.allclose(opq.scores(q, codes, cb, metric), by_table, rtol=1e-12, atol=1e-12)


def test_encode_is_the_best_code_by_brute_force():
    """On a tiny case every one of the ksub^M codes is tried: none reconstructs a vector better than the oracle's,
    and among equally good ones the oracle's is the smallest in every sub-space."""
    rng = np.random.default_rng(6)
    M, ksub, w = 3, 4, 2
    cb = rng.integers(-2, 3, size=(M, ksub, w)).astype(np.float64)          # small integers: ties happen
    X = rng.integers(-2, 3, size=(40, M * w)).astype(np.float64)
    codes = opq.encode(X, cb)
    all_codes = np.array(list(itertools.product(range(ksub), repeat=M)), dtype=np.uint8)
    recon = opq.decode(all_codes, cb)
    for i in range(X.shape[0]):
        err = ((recon - X[i][None, :]) ** 2).sum(axis=1)
        best = np.flatnonzero(err == err.min())
        assert tuple(codes[i]) == tuple(all_codes[best].min(axis=0))       # per sub-space independent: the minima combine
        assert abs(((opq.decode(codes[i:i + 1], cb)[0] - X[i]) ** 2).sum() - err.min()) < 1e-12


def test_lossless_codebooks_give_the_flat_index_answers():
    """Vectors assembled from codebook entries are their own reconstructions, so searching the codes must return
    exactly what the IVF-Flat oracle returns on the vectors (ids and order; scores to rounding)."""
    rng = np.random.default_rng(7)
    M, ksub, w, n, nlist = 4, 8, 4, 600, 6
    cb = rng.integers(-8, 9, size=(M, ksub, w)).astype(np.float32)
    codes = rng.integers(0, ksub, size=(n, M)).astype(np.uint8)
    X = opq.decode(codes, cb).astype(np.float32)
    assert np.array_equal(opq.encode(X, cb), opq.encode(opq.decode(codes, cb), cb))
    assert np.array_equal(opq.decode(opq.encode(X, cb), cb), X.astype(np.float64))   # (duplicate entries may renumber a code, never change the vector)
    from oracle import index as oindex
    cent = X[rng.choice(n, nlist, replace=False)]
    idx = oindex.build_index(X, cent, 0, train_iters=2)
    codes_lm = opq.encode(X[idx.list_ids], cb)
    for metric in (0, 1):
        for t in range(20):
            q = rng.integers(-8, 9, size=M * w).astype(np.float32)
            probe, ids, dist, n_out = opq.search(idx, codes_lm, cb, q, 10, 3, metric)
            fp, fids, fdist, fn = oracle.search(idx, q, 10, 3, metric)
            assert np.array_equal(probe, fp) and n_out == fn
            assert np.array_equal(ids, fids)                                   # integer data: exact scores, exact order
            assert np.array_equal(dist[:n_out], fdist[:fn])


def test_training_never_increases_the_quantisation_error():
    rng = np.random.default_rng(8)
    X = rng.normal(size=(500, 8))
    cb = X[rng.choice(500, 8, replace=False)].reshape(8, 4, 2).transpose(1, 0, 2).copy()      # [M=4, ksub=8, w=2]
    prev = opq.quantisation_error(X, opq.encode(X, cb), cb)
    for _ in range(4):
        cb = opq.train(X, cb, 1)
        err = opq.quantisation_error(X, opq.encode(X, cb), cb)
        assert err <= prev + 1e-12
        prev = err


class _Mutant:
    """The oracle with one function replaced by a plausibly wrong one."""

    def __init__(self, **repl):
        self.__dict__.update({k: getattr(opq, k) for k in ("encode", "decode", "scores", "train", "quantisation_error", "search")})
        self.__dict__.update(repl)
        if "scores" in repl or "decode" in repl:                               # search must see the replaced pieces
            mod = self

            def search(index, codes, cb, q, k, nprobe, metric, probe=None, all_candidates=False):
                pos, ids = opq.candidates(index, np.arange(index.nlist) if probe is None else probe)
                sc = mod.scores(q, codes[pos], cb, metric)
                order = np.lexsort((ids, sc if metric == 0 else -sc))
                n = min(k, order.shape[0])
                out_ids = np.full(k, -1, dtype=np.int64)
                out_dist = np.full(k, np.inf if metric == 0 else -np.inf)
                out_ids[:n] = ids[order[:n]]
                out_dist[:n] = sc[order[:n]]
                return probe, out_ids, out_dist, n
            self.search = search


def _decode_subspaces_reversed(codes, cb):
    M = cb.shape[0]
    return np.concatenate([cb[M - 1 - m].astype(np.float64)[codes[:, m].astype(np.int64)] for m in range(M)], axis=1)


def _encode_last_minimum(X, cb):
    M, ksub, w = cb.shape
    X = np.asarray(X, dtype=np.float64)
    codes = np.zeros((X.shape[0], M), dtype=np.uint8)
    for m in range(M):
        d2 = ((X[:, None, m * w:(m + 1) * w] - cb[m][None, :, :]) ** 2).sum(axis=2)
        codes[:, m] = ksub - 1 - np.argmin(d2[:, ::-1], axis=1)               # ties to the LARGER number
    return codes


def _scores_quantised_query(q, codes, cb, metric):
    qhat = opq.decode(opq.encode(np.asarray(q, dtype=np.float64)[None, :], cb), cb)[0]       # symmetric, not asymmetric
    return opq.scores(qhat, codes, cb, metric)


def _scores_ip_as_distance(q, codes, cb, metric):
    return opq.scores(q, codes, cb, 0)


def _train_empty_cell_to_zero(X, init, iters):
    cb = np.array(init, dtype=np.float64)
    for _ in range(iters):
        codes = opq.encode(X, cb)
        for m in range(cb.shape[0]):
            w = cb.shape[2]
            for c in range(cb.shape[1]):
                members = np.asarray(X, dtype=np.float64)[codes[:, m] == c][:, m * w:(m + 1) * w]
                cb[m, c] = members.mean(axis=0) if members.shape[0] else 0.0
    return cb


@pytest.mark.parametrize("name,repl", [
    ("sub-spaces in reverse order", dict(decode=_decode_subspaces_reversed,
                                         scores=lambda q, c, cb, m: ((_decode_subspaces_reversed(c, cb) - np.asarray(q, dtype=np.float64)) ** 2).sum(axis=1)
                                         if m == 0 else (_decode_subspaces_reversed(c, cb) * np.asarray(q, dtype=np.float64)).sum(axis=1))),
    ("ties to the larger code", dict(encode=_encode_last_minimum)),
    ("query quantised too", dict(scores=_scores_quantised_query)),
    ("inner product scored as a distance", dict(scores=_scores_ip_as_distance)),
])
def test_planted_mistakes_fail_the_hand_worked_example(name, repl):
    with pytest.raises(AssertionError):
        _check_gold(_Mutant(**repl))


def test_the_empty_cell_rule_is_pinned():
    """A codebook entry no sub-vector is nearest to keeps its value (the hand-worked example has none, so here)."""
    X = np.array([[0.0, 0.0], [1.0, 0.0], [0.0, 1.0]])
    init = np.array([[[0.0, 0.0], [5.0, 5.0]]])                                # M = 1, entry 1 attracts nothing
    got = opq.train(X, init, 1)
    assert np.allclose(got[0, 0], [1 / 3, 1 / 3]) and np.array_equal(got[0, 1], [5.0, 5.0])
    assert not np.array_equal(_train_empty_cell_to_zero(X, init, 1)[0, 1], [5.0, 5.0])


def test_reranking_pins():
    """The two-stage search: with a short list as long as the candidate set the second stage decides alone, so the
    answer must be the IVF-Flat oracle's; with lossless codebooks both stages score alike, so it must be the
    one-stage answer; and a short list of exactly k returns the one-stage ids, re-ordered by their exact scores."""
    rng = np.random.default_rng(11)
    M, ksub, w, n, nlist = 4, 16, 3, 500, 5
    X = rng.normal(size=(n, M * w)).astype(np.float32)
    cb = opq.train(X, X[rng.choice(n, ksub, replace=False)].reshape(ksub, M, w).transpose(1, 0, 2), 3)
    from oracle import index as oindex
    idx = oindex.build_index(X, X[rng.choice(n, nlist, replace=False)], 0, train_iters=2)
    codes_lm = opq.encode(X[idx.list_ids], cb)
    for metric in (0, 1):
        for t in range(10):
            q = rng.normal(size=M * w).astype(np.float32)
            probe, ids, dist, n_out, _, _ = opq.search_reranked(idx, codes_lm, cb, q, 7, n, 3, metric)
            fp, fids, fdist, fn = oracle.search(idx, q, 7, 3, metric)
            assert np.array_equal(ids, fids) and np.allclose(dist[:n_out], fdist[:fn], rtol=1e-12, atol=1e-12)
            _, ids1, _, n1 = opq.search(idx, codes_lm, cb, q, 7, 3, metric)
            _, ids2, dist2, n2, _, _ = opq.search_reranked(idx, codes_lm, cb, q, 7, 7, 3, metric)
            assert n1 == n2 and sorted(ids1.tolist()) == sorted(ids2.tolist())
            exact = ((X[ids2[:n2]].astype(np.float64) - q.astype(np.float64)) ** 2).sum(axis=1) if metric == 0 else \
                (X[ids2[:n2]].astype(np.float64) * q.astype(np.float64)).sum(axis=1)
            assert np.allclose(dist2[:n2], exact, rtol=1e-12, atol=1e-12)
            assert np.all(np.diff(dist2[:n2]) >= 0) if metric == 0 else np.all(np.diff(dist2[:n2]) <= 0)
