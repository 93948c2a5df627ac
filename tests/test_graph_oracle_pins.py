"""Pins for the CPU oracle of the graph engine (oracle/graph_search.py): hand-worked trajectories,
special cases that reduce to exact kNN by brute force, and the invariants of the extend loop."""
import json
import os

import numpy as np
import pytest

from oracle import graph_search as gs
from tests import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "graph_examples.json")


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_hand_worked_trajectories(dtype):
    data = json.load(open(GOLDEN))
    X = np.asarray(data["base"], dtype=dtype)
    G = np.asarray(data["graph"], dtype=np.uint32)
    q = np.asarray(data["q"], dtype=dtype)
    for c in data["cases"]:
        r = gs.search(X, G, c["seeds"], q, c["k"], c["topm"], c["p"], c["max_iters"], gs.METRIC_L2, trace=True)
        assert r["trace"] == c["trace"], c["name"]
        assert (r["iters"], r["evals"], r["n"]) == (c["iters"], c["evals"], len(c["ids"])), c["name"]
        assert list(r["ids"]) == c["ids"] and list(r["dist"]) == c["dist"], c["name"]


def _random_instance(rng, n, dim, D, dtype, connected=True):
    X = rng.integers(-8, 9, size=(n, dim)).astype(dtype)          # small integers: every sum is exact
    G = rng.integers(0, n, size=(n, D)).astype(np.uint32)
    if connected:
        G[:, 0] = (np.arange(n) + 1) % n                          # a ring: everything reachable from anywhere
    return X, G


@pytest.mark.parametrize("metric", [gs.METRIC_L2, gs.METRIC_IP])
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_topm_of_everything_is_exact_knn(metric, dtype):
    """topM as large as the database and every non-expanded entry taken as a parent (p = N) on a connected graph:
    the extends are the layers of a breadth-first traversal, topM changes as long as a layer reaches anything
    new, so the loop ends only when every node has been scored and the answer is exact kNN (brute force)."""
    rng = np.random.default_rng(21 + metric)
    for n, dim, D, k in ((40, 3, 3, 5), (200, 8, 4, 17), (64, 2, 2, 64)):
        X, G = _random_instance(rng, n, dim, D, dtype)
        for _ in range(5):
            q = rng.integers(-8, 9, size=dim).astype(dtype)
            r = gs.search(X, G, [int(rng.integers(0, n))], q, k, n, n, 10 * n, metric)
            want_ids, want_sc = (a[0] for a in bruteforce.knn(X, q[None, :], k, metric))
            assert r["evals"] == n and r["n"] == k
            assert list(r["ids"]) == list(want_ids)
            assert np.array_equal(r["dist"], want_sc)


def test_complete_graph_needs_one_extend():
    """Every node linked to every other: the first extend scores everything, topM is then the exact top M."""
    rng = np.random.default_rng(5)
    n, dim = 50, 4
    X = rng.integers(-8, 9, size=(n, dim)).astype(np.float32)
    G = np.array([[j for j in range(n) if j != i] for i in range(n)], dtype=np.uint32)
    q = rng.integers(-8, 9, size=dim).astype(np.float32)
    r = gs.search(X, G, [7], q, 10, 16, 1, 100, gs.METRIC_L2, trace=True)
    want_ids, want_sc = (a[0] for a in bruteforce.knn(X, q[None, :], 16, gs.METRIC_L2))
    assert r["trace"][1]["ids"] == list(want_ids) and list(r["ids"]) == list(want_ids[:10])
    assert r["iters"] == 2 and r["evals"] == n        # the second extend finds nothing new and ends the request


@pytest.mark.parametrize("metric", [gs.METRIC_L2, gs.METRIC_IP])
def test_extend_loop_invariants(metric):
    rng = np.random.default_rng(77)
    n, dim, D, M, p = 500, 6, 8, 24, 3
    X, G = _random_instance(rng, n, dim, D, np.float32, connected=False)
    G[rng.random(G.shape) < 0.1] = 0xFFFFFFFF                    # some padding entries
    seeds = [3, 3, 499, 17]                                      # a duplicate entry point is scored once
    sign = 1.0 if metric == gs.METRIC_L2 else -1.0
    for _ in range(20):
        q = rng.integers(-8, 9, size=dim).astype(np.float32)
        r = gs.search(X, G, seeds, q, 10, M, p, 40, metric, trace=True)
        tr = r["trace"]
        assert len(tr) == r["iters"] + 1 and r["iters"] <= 40
        assert r["evals"] <= 3 + r["iters"] * p * D
        for a, b in zip(tr, tr[1:]):
            assert len(b["ids"]) <= M and len(set(b["ids"])) == len(b["ids"])
            key = [sign * d for d in b["dist"]]
            assert key == sorted(key)
            assert len(b["ids"]) >= len(a["ids"])
            m = min(len(a["ids"]), 10)
            assert all(sign * y <= sign * x for x, y in zip(a["dist"][:m], b["dist"][:m]))   # never gets worse
        # every reported distance is the true one
        assert np.array_equal(r["dist"][:r["n"]], gs.scores(X, r["ids"][:r["n"]], q, metric))
        # the paper's stop rule: every extend but the last changed topM
        for a, b in zip(tr[:-2], tr[1:-1]):
            assert set(a["ids"]) != set(b["ids"])


def test_planted_mistakes_fail_the_hand_worked_cases():
    """Mutants of the oracle's source (a dropped visited filter, parents never marked, a wrong stop rule,
    ties by descending id) must disagree with the hand-worked trajectories."""
    src = open(gs.__file__).read()
    data = json.load(open(GOLDEN))
    X = np.asarray(data["base"], dtype=np.float32)
    G = np.asarray(data["graph"], dtype=np.uint32)
    q = np.asarray(data["q"], dtype=np.float32)
    mutants = {
        "no visited filter": ("if v < n and not visited[v]:\n                    visited[v] = True\n                    cand.append(v)",
                              "if v < n:\n                    visited[v] = True\n                    cand.append(v)"),
        "parents never marked": ("top_exp[i] = True", "pass"),
        "stop only at empty frontier": ("if not changed:\n            break", "pass"),
        "worst parents first": ("parents = [i for i, e in enumerate(top_exp) if not e][:p]",
                                "parents = [i for i, e in enumerate(top_exp) if not e][-p:]"),
        "ties by descending id": ("np.lexsort((np.asarray(ids, dtype=np.int64), key))",
                                  "np.lexsort((-np.asarray(ids, dtype=np.int64), key))"),
    }
    for name, (old, new) in mutants.items():
        assert old in src, name
        ns = {}
        exec(compile(src.replace(old, new), f"<mutant {name}>", "exec"), ns)
        bad = False
        for c in data["cases"]:
            try:
                r = ns["search"](X, G, c["seeds"], q, c["k"], c["topm"], c["p"], min(c["max_iters"], 40), gs.METRIC_L2, trace=True)
                bad |= r["trace"] != c["trace"] or r["iters"] != c["iters"] or r["evals"] != c["evals"]
            except Exception:
                bad = True
        if name == "ties by descending id":       # the chain has no ties: this mutant is caught by brute force instead
            rng = np.random.default_rng(1)
            Xi = rng.integers(0, 2, size=(30, 2)).astype(np.float32)
            Gi = np.stack([(np.arange(30) + 1) % 30, (np.arange(30) + 7) % 30], axis=1).astype(np.uint32)
            qi = np.zeros(2, dtype=np.float32)
            r = ns["search"](Xi, Gi, [0], qi, 10, 30, 30, 300, gs.METRIC_L2)
            want_ids = bruteforce.knn(Xi, qi[None, :], 10, gs.METRIC_L2)[0][0]
            bad |= list(r["ids"]) != list(want_ids)
        assert bad, f"mutant '{name}' passed the pins"
