"""Pins for the oracle's index helpers (oracle/index.py): each checks them against something that
is not themselves.

* hand-worked cases (tests/golden/index_examples.json): Lloyd iterations in one dimension with an
  empty cluster, spherical k-means in two dimensions, the clustering objective, assignment ties,
  a near-tie at the acceptance boundary of the index checker
* the hand-worked search examples (tests/golden/worked_examples.json): their lists are what the
  oracle's own construction must produce, and what the checker must accept
* assignment against an enumeration in Python integers (exact on integer-valued data) with
  duplicated centroids
* the index checker against planted faults: a row in a wrong list, in its WORST list, a duplicated
  id, broken offsets -- each must be refused
* planted mistakes: mutated copies of oracle/index.py must FAIL these pins
"""
import importlib.util
import json
import math
import os
import sys

import numpy as np
import pytest

import oracle
from oracle import Index, METRIC_IP, METRIC_L2
from oracle import index as oindex

HERE = os.path.dirname(__file__)
GOLDEN_INDEX = os.path.join(HERE, "golden", "index_examples.json")
GOLDEN_SEARCH = os.path.join(HERE, "golden", "worked_examples.json")
_NAMES = {"sqrt": math.sqrt}


def _metric(name):
    return METRIC_L2 if name == "l2" else METRIC_IP


def _value(expr):
    """A golden value given as an expression ("3/sqrt(10)") or a number."""
    return float(eval(expr, {"__builtins__": {}}, _NAMES)) if isinstance(expr, str) else float(expr)


def _index_from_lists(base, centroids, lists):
    off = np.zeros(len(lists) + 1, dtype=np.uint64)
    off[1:] = np.cumsum([len(l) for l in lists])
    ids = np.array([i for l in lists for i in l], dtype=np.int64)
    return Index(base, np.asarray(centroids, dtype=np.float32), off, ids)


def _lists_of(index):
    return [index.list_ids[int(index.list_off[j]):int(index.list_off[j + 1])].tolist() for j in range(index.nlist)]


# ------------------------------------------------------------------------------------------------
# The pins as functions of the module under test, so that the planted mistakes below can be run
# through the very same checks.  Each returns a list of failure strings (empty = pass).
def pin_lloyd_hand_cases(mod):
    fails = []
    with open(GOLDEN_INDEX) as f:
        data = json.load(f)
    for case in data["lloyd"]:
        metric = _metric(case["metric"])
        base = np.asarray(case["base"], dtype=np.float32)
        init = np.asarray(case["init"], dtype=np.float32)
        table = case.get("after") or case["after_expr"]
        for iters, want in table.items():
            want = np.array([[_value(v) for v in row] for row in want])
            got = mod.lloyd(base, init, int(iters), metric)
            if got.shape != want.shape or not np.allclose(got, want, rtol=0, atol=1e-12):
                fails.append(f"{case['name']}: centroids after {iters} iterations {got.tolist()} != {want.tolist()}")
        # the partition and the objective after two iterations (centroids as the hand calculation has them)
        two = table["2"]
        cent = np.array([[_value(v) for v in row] for row in two])
        assign = mod.assign_rows(base, cent, metric)
        off, ids = mod.partition(assign, cent.shape[0])
        idx = Index(base, cent.astype(np.float32), off, ids)
        if _lists_of(idx) != case["lists_after_2"]:
            fails.append(f"{case['name']}: lists {_lists_of(idx)} != {case['lists_after_2']}")
        want_obj = _value(case.get("inertia_after_2", case.get("inertia_after_2_expr")))
        good = _index_from_lists(base, cent, case["lists_after_2"])
        got_obj = mod.inertia(base, good, metric)
        if abs(got_obj - want_obj) > 1e-6:        # (the index keeps its centroids in fp32)
            fails.append(f"{case['name']}: objective {got_obj} != {want_obj}")
    return fails


def pin_assign_hand_cases(mod):
    fails = []
    with open(GOLDEN_INDEX) as f:
        data = json.load(f)
    for case in data["assign"]:
        for dtype in (np.float32, np.float16):
            got = mod.assign_rows(np.asarray(case["base"], dtype=dtype), np.asarray(case["centroids"], dtype=np.float32),
                                  _metric(case["metric"]))
            if got.tolist() != case["want"]:
                fails.append(f"{case['name']} ({np.dtype(dtype).name}): {got.tolist()} != {case['want']}")
    return fails


def _enumerate_assignment(base_int, cent_int, metric):
    """Best centroid per row in Python integers: plain loops, first best wins."""
    out = []
    for row in base_int:
        best_j, best_s = -1, None
        for j, c in enumerate(cent_int):
            if metric == METRIC_L2:
                s = sum((int(a) - int(b)) ** 2 for a, b in zip(row, c))
                better = best_s is None or s < best_s
            else:
                s = sum(int(a) * int(b) for a, b in zip(row, c))
                better = best_s is None or s > best_s
            if better:
                best_j, best_s = j, s
        out.append(best_j)
    return out


def pin_assign_against_integer_enumeration(mod, seeds=range(10)):
    fails = []
    for metric in (METRIC_L2, METRIC_IP):
        for seed in seeds:
            rng = np.random.default_rng(500 + seed)
            d = int(rng.integers(1, 6))
            nlist = int(rng.integers(2, 10))
            n = int(rng.integers(1, 80))
            cent = rng.integers(-3, 4, size=(nlist, d))
            dup = rng.integers(0, nlist, size=max(1, nlist // 2))
            cent[dup] = cent[rng.integers(0, nlist, size=dup.size)]       # duplicated centroids -> exact ties
            base = rng.integers(-3, 4, size=(n, d))
            want = _enumerate_assignment(base.tolist(), cent.tolist(), metric)
            for dtype in (np.float32, np.float16):
                got = mod.assign_rows(base.astype(dtype), cent.astype(np.float32), metric, chunk=7)
                if got.tolist() != want:
                    fails.append(f"metric {metric} seed {seed} {np.dtype(dtype).name}: assignment differs")
    return fails


def pin_partition_is_stable_and_complete(mod):
    """Rows of a list in ascending order, offsets = running counts (counted here with a dictionary)."""
    fails = []
    rng = np.random.default_rng(9)
    for n, nlist in ((1, 1), (17, 3), (5000, 4), (3000, 37)):
        a = rng.integers(0, nlist, size=n).astype(np.int64)
        if nlist > 2:
            a[a == 1] = 0                                # an empty list in the middle
        off, ids = mod.partition(a, nlist)
        counts = {}
        for v in a.tolist():
            counts[v] = counts.get(v, 0) + 1
        run = 0
        for j in range(nlist):
            if int(off[j]) != run:
                fails.append(f"n {n}: offset of list {j} is {int(off[j])}, {run} rows precede it")
                break
            rows = ids[run:run + counts.get(j, 0)].tolist()
            if any(a[r] != j for r in rows) or rows != sorted(rows):
                fails.append(f"n {n}: list {j} holds foreign rows or is not ascending")
                break
            run += counts.get(j, 0)
        if int(off[-1]) != n:
            fails.append(f"n {n}: last offset {int(off[-1])}")
    return fails


def pin_construction_reproduces_hand_worked_lists(mod):
    fails = []
    with open(GOLDEN_SEARCH) as f:
        data = json.load(f)
    for case in data["cases"]:
        for dtype in (np.float32, np.float16):
            base = np.asarray(case["base"], dtype=dtype)
            idx = mod.build_index(base, np.asarray(case["centroids"], dtype=np.float32), _metric(case["metric"]))
            if _lists_of(idx) != case["lists"]:
                fails.append(f"{case['name']} ({np.dtype(dtype).name}): lists {_lists_of(idx)} != {case['lists']}")
    return fails


def _refuses(mod, index, metric, tol=0.0, **kw):
    try:
        mod.check_index(index, metric, tol, **kw)
    except AssertionError:
        return True
    return False


def pin_checker_accepts_good_and_refuses_faulty_indexes(mod):
    fails = []
    with open(GOLDEN_SEARCH) as f:
        cases = {c["name"]: c for c in json.load(f)["cases"]}
    # ---- the hand-worked indexes are accepted, every row exactly at its best centroid
    for case in cases.values():
        base = np.asarray(case["base"], dtype=np.float32)
        good = _index_from_lists(base, case["centroids"], case["lists"])
        try:
            rep = mod.check_index(good, _metric(case["metric"]), 0.0)
            if (rep["checked"], rep["exact"], rep["near_tie"]) != (base.shape[0], base.shape[0], 0):
                fails.append(f"{case['name']}: report {rep}")
        except AssertionError as e:
            fails.append(f"{case['name']}: good index refused ({e})")
    # ---- 1-D squared L2: base i = 0..15, centroids 1.5 / 5.5 / 9.5 / 13.5
    c = cases["1d_l2"]
    base = np.asarray(c["base"], dtype=np.float32)
    lists = [list(l) for l in c["lists"]]
    moved = [lists[0][:3], [3] + lists[1], lists[2], lists[3]]          # row 3 (2.25 from 1.5) stored under 5.5 (6.25)
    if not _refuses(mod, _index_from_lists(base, c["centroids"], moved), METRIC_L2):
        fails.append("1d_l2: a row in a wrong list was accepted")
    if not _refuses(mod, _index_from_lists(base, c["centroids"], moved), METRIC_L2, tol=1e-3):
        fails.append("1d_l2: a row in a wrong list was accepted under a small tolerance")
    far = [lists[0][:3], lists[1], lists[2], lists[3] + [3]]            # ... and under its worst centroid
    if not _refuses(mod, _index_from_lists(base, c["centroids"], far), METRIC_L2, tol=0.5):
        fails.append("1d_l2: a row in its worst list was accepted")
    good = _index_from_lists(base, c["centroids"], lists)
    dup = Index(base, good.centroids, good.list_off, good.list_ids.copy())
    dup.list_ids[3] = 2                                                  # id 2 twice, id 3 missing
    if not _refuses(mod, dup, METRIC_L2):
        fails.append("1d_l2: a duplicated id was accepted")
    out_of_range = Index(base, good.centroids, good.list_off, good.list_ids.copy())
    out_of_range.list_ids[0] = 16
    try:
        mod.check_index(out_of_range, METRIC_L2, 0.0)
        fails.append("1d_l2: an id outside 0..n-1 was accepted")
    except (AssertionError, IndexError):
        pass
    for name, off in (("first offset not zero", [1, 4, 8, 12, 16]), ("last offset not n", [0, 4, 8, 12, 15]),
                      ("offsets decreasing", [0, 8, 4, 12, 16])):
        bad = Index(base, good.centroids, np.asarray(off, dtype=np.uint64), good.list_ids)
        if not _refuses(mod, bad, METRIC_L2):
            fails.append(f"1d_l2: {name} was accepted")
    shifted = Index(base, good.centroids, np.asarray([0, 3, 8, 12, 16], dtype=np.uint64), good.list_ids)
    if not _refuses(mod, shifted, METRIC_L2):                            # row 3 falls into list 1 by the offsets alone
        fails.append("1d_l2: a shifted list boundary was accepted")
    # sampled checking still sees a fault when the sample is the whole index or the planted rows are many
    if not _refuses(mod, _index_from_lists(base, c["centroids"], [lists[3], lists[2], lists[1], lists[0]]), METRIC_L2,
                    sample=8, seed=1):
        fails.append("1d_l2: sampled check accepted an index with every list under the wrong centroid")
    # ---- inner product: a row under its WORST centroid (what a swapped min / max would call the best)
    c = cases["2d_ip"]
    base = np.asarray(c["base"], dtype=np.float32)
    lists = [list(l) for l in c["lists"]]
    worst = [[0], lists[1], lists[2] + [1]]                              # row (2,0): scores 2, 0, -2 -> stored under -2
    if not _refuses(mod, _index_from_lists(base, c["centroids"], worst), METRIC_IP, tol=0.5):
        fails.append("2d_ip: a row in its worst list was accepted")
    second = [[0], lists[1] + [1], lists[2]]                             # ... under the middle one
    if not _refuses(mod, _index_from_lists(base, c["centroids"], second), METRIC_IP):
        fails.append("2d_ip: a row in its second-best list was accepted")
    # the L2 checker must not accept the IP index's logic and vice versa: row (0,3) is best under (0,1) for IP,
    # while under squared L2 (0,3) is 4 from (0,1), 10 from (1,0) -- still list 1; row (-2,-1): L2 1 from (-1,-1) -- list 2.
    # A row for which the two metrics disagree: (2,0) is L2-closest to (1,0) [1] and IP-best under (1,0) [2] -- agree;
    # use (0,3) moved under (1,0): IP score 0 vs best 3 -> refused under IP
    moved = [lists[0] + [3], [2], lists[2]]
    if not _refuses(mod, _index_from_lists(base, c["centroids"], moved), METRIC_IP, tol=0.1):
        fails.append("2d_ip: row (0,3) under centroid (1,0) was accepted")
    # ---- the near-tie band
    with open(GOLDEN_INDEX) as f:
        nt = json.load(f)["near_tie"]
    base = np.asarray(nt["base"], dtype=np.float32)
    idx = _index_from_lists(base, nt["centroids"], nt["lists"])
    try:
        rep = mod.check_index(idx, _metric(nt["metric"]), nt["accept_tol"])
        if (rep["exact"], rep["near_tie"]) != (2, 1):
            fails.append(f"near tie: report {rep}, expected 2 exact rows and 1 near-tie")
    except AssertionError as e:
        fails.append(f"near tie: refused at tolerance {nt['accept_tol']} ({e})")
    if not _refuses(mod, idx, _metric(nt["metric"]), tol=nt["reject_tol"]):
        fails.append(f"near tie: accepted at tolerance {nt['reject_tol']}")
    if not _refuses(mod, idx, _metric(nt["metric"]), tol=0.0):
        fails.append("near tie: accepted at tolerance zero")
    return fails


ALL_PINS = [pin_lloyd_hand_cases, pin_assign_hand_cases, pin_assign_against_integer_enumeration,
            pin_partition_is_stable_and_complete, pin_construction_reproduces_hand_worked_lists,
            pin_checker_accepts_good_and_refuses_faulty_indexes]


@pytest.mark.parametrize("pin", ALL_PINS, ids=[p.__name__ for p in ALL_PINS])
def test_index_helpers_meet_their_pins(pin):
    assert pin(oindex) == []


def test_lloyd_never_raises_the_objective_and_matches_scipy_on_separated_blobs():
    """Two properties no single formula of the module states: the objective is monotone over Lloyd iterations
    (the textbook convergence argument), and on well-separated blobs the fixed point is the blob means --
    checked against scipy's k-means from the same start."""
    from scipy.cluster.vq import kmeans2
    rng = np.random.default_rng(3)
    centres = np.array([[0, 0, 0], [10, 0, 0], [0, 10, 0], [0, 0, 10]], dtype=np.float64)
    base = np.concatenate([c + 0.3 * rng.standard_normal((50, 3)) for c in centres]).astype(np.float32)
    init = base[[0, 50, 100, 150]] + np.float32(0.5)
    prev = None
    for iters in range(0, 5):
        idx = oindex.build_index(base, oindex.lloyd(base, init, iters, METRIC_L2).astype(np.float32), METRIC_L2)
        obj = oindex.inertia(base, idx, METRIC_L2)
        assert prev is None or obj <= prev * (1 + 1e-9)
        prev = obj
    got = oindex.lloyd(base, init, 4, METRIC_L2)
    want, _ = kmeans2(base.astype(np.float64), init.astype(np.float64), iter=4, minit="matrix")
    assert np.allclose(got, want, atol=1e-9)
    blob_means = base.astype(np.float64).reshape(4, 50, 3).mean(axis=1)
    assert np.allclose(got, blob_means, atol=1e-9)


# ----------------------------------------------------------------------------- planted mistakes
MUTATIONS = [
    ("L2 assignment takes the largest score", "np.argmin(sc, axis=1) if metric == METRIC_L2 else np.argmax(sc, axis=1)",
     "np.argmax(sc, axis=1) if metric == METRIC_L2 else np.argmax(sc, axis=1)"),
    ("IP assignment takes the smallest score", "np.argmin(sc, axis=1) if metric == METRIC_L2 else np.argmax(sc, axis=1)",
     "np.argmin(sc, axis=1) if metric == METRIC_L2 else np.argmin(sc, axis=1)"),
    ("checker: min and max swapped", "best = sc.min(axis=1) if build_metric == METRIC_L2 else sc.max(axis=1)",
     "best = sc.max(axis=1) if build_metric == METRIC_L2 else sc.min(axis=1)"),
    ("checker: IP best taken as the minimum", "best = sc.min(axis=1) if build_metric == METRIC_L2 else sc.max(axis=1)",
     "best = sc.min(axis=1)"),
    ("checker: tolerance absolute instead of relative", "is_near = (~is_exact) & (gap <= tol * scale)",
     "is_near = (~is_exact) & (gap <= tol)"),
    ("checker: tolerance scaled twice", "is_near = (~is_exact) & (gap <= tol * scale)",
     "is_near = (~is_exact) & (gap <= tol * scale * scale)"),
    ("checker: permutation test dropped", 'assert np.all(seen == 1), "ids are not a permutation of the rows"', "pass"),
    ("checker: monotone test dropped", 'assert np.all(off[1:] >= off[:-1]), "list_off not monotone"', "pass"),
    ("checker: a row's own list read from the wrong array",
     "list_of_row[ids] = np.repeat(np.arange(nlist, dtype=np.int64), np.diff(off).astype(np.int64))",
     "list_of_row[np.arange(n)] = np.repeat(np.arange(nlist, dtype=np.int64), np.diff(off).astype(np.int64))"),
    ("partition: sort not stable", 'np.argsort(assignment, kind="stable")', "np.argsort(assignment)"),
    ("partition: offsets shifted", "off[1:] = np.cumsum(counts)", "off[:-1] = np.cumsum(counts)"),
    ("lloyd: empty cluster reset", "if members.shape[0] == 0:\n                continue",
     "if members.shape[0] == 0:\n                c[j] = 0.0\n                continue"),
    ("lloyd: spherical variant not normalised", "m = m / nrm", "m = m"),
    ("lloyd: sum instead of mean", "m = members.mean(axis=0)", "m = members.sum(axis=0)"),
    ("lloyd: assignment from the initial centroids every time", "a = assign_rows(base, c, metric)",
     "a = assign_rows(base, init_centroids, metric)"),
    ("scores: L2 sign", "diff = r - c[j]", "diff = r + c[j]"),
    ("objective: L2 not squared", "total += float((diff * diff).sum())", "total += float(np.abs(diff).sum())"),
    ("objective: IP sign", "total += float((1.0 - x @ c[j]).sum())", "total += float((1.0 + x @ c[j]).sum())"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_in_the_index_helpers_is_caught(name, old, new):
    path = os.path.join(os.path.dirname(oracle.__file__), "index.py")
    src = open(path).read()
    assert src.count(old) == 1, "mutation anchor not found exactly once"
    spec = importlib.util.spec_from_loader("oracle._index_mutant", loader=None, origin=path)
    mod = importlib.util.module_from_spec(spec)
    mod.__package__ = "oracle"
    sys.modules["oracle._index_mutant"] = mod
    try:
        exec(compile(src.replace(old, new), path + " (mutated)", "exec"), mod.__dict__)
        fails = []
        for pin in ALL_PINS:
            try:
                fails += pin(mod)
            except Exception as e:          # a mutated module may also fail outright
                fails.append(f"{pin.__name__}: {type(e).__name__}: {e}")
        assert fails, f"planted mistake '{name}' went unnoticed"
    finally:
        del sys.modules["oracle._index_mutant"]
