"""GPU parity of the graph engine (include/trinity_graph.h) against oracle/graph_search.py, through the C ABI.

On integer-valued data every score is exact in fp32 in any summation order, so the engine's whole
trajectory -- which candidates enter topM, which parents are expanded, when a request stops -- must
equal the oracle's: ids, score bits, number of extends and number of distance evaluations are compared
exactly.  On real-valued data the two may order near-equal scores differently and follow different
trajectories, so there only what is unique is compared (every reported score is the true score of its
id, lists are sorted and duplicate-free) and recall against brute force must match the oracle's closely."""
import json
import os

import numpy as np
import pytest

import graph_inputs
from oracle import graph_search as gs
from tests import bruteforce, harness

pytestmark = pytest.mark.gpu


def _say(msg):
    harness.say(f"[graph] {msg}")


def _lib():
    import paper_2512_02281_amd as tri
    from paper_2512_02281_amd import graph as tg
    return tri, tg


def _oracle_all(X, G, seeds, Q, k, metric, M, p, max_iters):
    nq = Q.shape[0]
    k = np.broadcast_to(np.asarray(k), (nq,))
    metric = np.broadcast_to(np.asarray(metric), (nq,))
    return [gs.search(X, G, seeds, Q[i], int(k[i]), M, p, max_iters, int(metric[i])) for i in range(nq)]


def _check_exact(got, want, k):
    ids, dist, n_out, iters, evals = got
    nq = len(want)
    k = np.broadcast_to(np.asarray(k), (nq,))
    for i, w in enumerate(want):
        kk = int(k[i])
        assert int(n_out[i]) == w["n"], f"query {i}: n_out {n_out[i]} != {w['n']}"
        assert int(iters[i]) == w["iters"] and int(evals[i]) == w["evals"], \
            f"query {i}: extends/evals {iters[i]}/{evals[i]} != {w['iters']}/{w['evals']}"
        assert np.array_equal(ids[i, :kk], w["ids"]), f"query {i}: ids {ids[i, :kk]} != {w['ids']}"
        # (integer-valued data: every sum is exact in fp32 in any order, so the fp32 scores equal the oracle's fp64 ones)
        assert np.array_equal(dist[i, :kk].astype(np.float64), w["dist"]), f"query {i}: scores"


@pytest.mark.parametrize("np_dtype", [np.float32, np.float16])
def test_hand_worked_trajectories_through_the_library(np_dtype):
    tri, tg = _lib()
    data = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "graph_examples.json")))
    X = np.asarray(data["base"], dtype=np_dtype)
    G = np.asarray(data["graph"], dtype=np.uint32)
    q = np.asarray([data["q"]], dtype=np_dtype)
    dt = tri.TRI_F16 if np_dtype == np.float16 else tri.TRI_F32
    for c in data["cases"]:
        with tg.GraphPool(X, G, np.asarray(c["seeds"], dtype=np.uint32), dt, slots=4, topm=c["topm"], parents=c["p"],
                          max_iters=min(c["max_iters"], 1000)) as pool:
            ids, dist, n_out, iters, evals, steps = pool.run_all(q, c["k"], tri.TRI_L2)
            assert list(ids[0]) == c["ids"] and list(dist[0]) == c["dist"], c["name"]
            assert (int(iters[0]), int(evals[0]), int(n_out[0])) == (c["iters"], c["evals"], len(c["ids"])), c["name"]


@pytest.mark.parametrize("np_dtype,dim", [(np.float16, 768), (np.float32, 128), (np.float16, 96), (np.float32, 200)])
def test_integer_data_trajectories_equal_the_oracle(np_dtype, dim):
    """Every row length class of the distance kernel (1536, 512 bytes: unrolled; 256, 1024: generic), both
    metrics, heterogeneous k, more queries than slots (slot reuse, arrivals joining mid-stream)."""
    tri, tg = _lib()
    n, nq, D, M, p, iters = 20_000, 300, 16, 48, 3, 40
    Xt, Z = graph_inputs.make_points(n, dim, 8, np_dtype, graph_inputs.SEED_POINTS, integer=True)
    Qt, _ = graph_inputs.make_points(nq, dim, 8, np_dtype, graph_inputs.SEED_QUERIES, integer=True)
    Gt = graph_inputs.make_graph(Z, D, 4, graph_inputs.SEED_EDGES)
    X, Q, G = Xt.numpy(), Qt.numpy(), Gt.numpy().astype(np.uint32)
    G[::97, 5] = tg.TRI_GRAPH_PAD                                   # some padding entries
    seeds = np.r_[graph_inputs.entry_points(n, 24), [7, 7, n + 5]].astype(np.uint32)   # a duplicate, an invalid one
    k = np.random.default_rng(1).integers(1, M + 1, size=nq).astype(np.uint32)
    metric = (np.arange(nq) % 2).astype(np.uint32)
    dt = tri.TRI_F16 if np_dtype == np.float16 else tri.TRI_F32
    want = _oracle_all(X, G, seeds, Q, k, metric, M, p, iters)
    for slots, groups in ((64, 2), (300, 1), (7, 4), (2, 3)):
        with tg.GraphPool(X, G, seeds, dt, slots=slots, topm=M, parents=p, max_iters=iters, max_outstanding=1024,
                          groups=groups) as pool:
            ids, dist, n_out, it, ev, steps = pool.run_all(Q, k, metric)
            _say(f"{np_dtype.__name__} dim {dim}: {slots} slots in {groups} groups: {steps} steps, "
                 f"mean extends {it.mean():.1f}, mean evaluations {ev.mean():.0f}")
            _check_exact((ids, dist, n_out, it, ev), want, k)
            # the same pool again, queries from device memory, the other class mix: identical
            import torch
            ids2, dist2, n2, it2, ev2, _ = pool.run_all(torch.from_numpy(Q).cuda(), k, metric,
                                                        klass=(np.arange(nq) % 3 == 0).astype(np.uint32))
            assert np.array_equal(ids, ids2) and np.array_equal(dist.view(np.uint32), dist2.view(np.uint32))
            assert np.array_equal(it, it2) and np.array_equal(ev, ev2)


@pytest.mark.parametrize("flag", ["hash", "bits"])
def test_both_kinds_of_visited_set_are_exact(flag):
    """A request's visited set is a hash table sized by what the request can see, or a bit per database row
    (whichever is smaller, unless forced): both must reproduce the oracle's trajectories on integer data.  Two
    workloads: many short requests through few slots (tables cleared and reused), and requests that walk the whole
    of a small graph, which fills the small table in front and spills into the large one behind it."""
    tri, tg = _lib()
    flags = tg.TRI_GRAPH_VISITED_HASH if flag == "hash" else tg.TRI_GRAPH_VISITED_BITS
    n, nq, dim, D, M, p, iters = 20_000, 200, 96, 16, 48, 3, 40
    Xt, Z = graph_inputs.make_points(n, dim, 8, np.float16, graph_inputs.SEED_POINTS, integer=True)
    Qt, _ = graph_inputs.make_points(nq, dim, 8, np.float16, graph_inputs.SEED_QUERIES, integer=True)
    Gt = graph_inputs.make_graph(Z, D, 4, graph_inputs.SEED_EDGES)
    X, Q, G = Xt.numpy(), Qt.numpy(), Gt.numpy().astype(np.uint32)
    seeds = graph_inputs.entry_points(n, 24)
    k = np.random.default_rng(2).integers(1, M + 1, size=nq).astype(np.uint32)
    metric = (np.arange(nq) % 2).astype(np.uint32)
    want = _oracle_all(X, G, seeds, Q, k, metric, M, p, iters)
    for slots, groups in ((32, 2), (5, 3)):
        with tg.GraphPool(X, G, seeds, tri.TRI_F16, slots=slots, topm=M, parents=p, max_iters=iters, max_outstanding=1024,
                          groups=groups, flags=flags) as pool:
            ids, dist, n_out, it, ev, steps = pool.run_all(Q, k, metric)
            _check_exact((ids, dist, n_out, it, ev), want, k)
    # whole-graph walks: a ring with chords, every node reachable, topM as long as the limit allows, no early stop
    # before everything has been seen (integer coordinates on a circle-like curve keep topM changing)
    rng = np.random.default_rng(5)
    n2, D2, M2, p2 = 250, 8, 250, 8
    X2 = rng.integers(-6, 7, size=(n2, 12)).astype(np.float32)
    G2 = np.stack([(np.arange(n2) + d) % n2 for d in (1, 2, 3, 5, 8, 13, 21, 34)], axis=1).astype(np.uint32)
    Q2 = rng.integers(-6, 7, size=(40, 12)).astype(np.float32)
    seeds2 = np.array([0, 125], dtype=np.uint32)
    k2 = np.full(40, 20, dtype=np.uint32)
    m2 = (np.arange(40) % 2).astype(np.uint32)
    want2 = _oracle_all(X2, G2, seeds2, Q2, k2, m2, M2, p2, 1000)
    _say(f"visited {flag}: whole-graph walks score {np.mean([w['evals'] for w in want2]):.0f} of {n2} rows on average")
    assert np.mean([w["evals"] for w in want2]) > 0.8 * n2
    with tg.GraphPool(X2, G2, seeds2, tri.TRI_F32, slots=6, topm=M2, parents=p2, max_iters=1000, max_outstanding=64, groups=2,
                      flags=flags) as pool:
        for _ in range(2):                                # twice: the second round runs in tables the first one used
            ids, dist, n_out, it, ev, steps = pool.run_all(Q2, k2, m2)
            _check_exact((ids, dist, n_out, it, ev), want2, k2)


def test_squared_l2_comes_back_in_the_difference_form():
    """Real-valued data, squared L2.  The search ranks by |x|^2 + |q|^2 - 2 x.q; what is handed back is
    sum (x - q)^2 of the k rows, in fp32, ordered by (that, id): every distance within fp32 summation error of the
    fp64 one (far tighter than the expanded form allows when q is close to x), ascending, and a query that is a
    stored row gets that row first with distance exactly zero."""
    import torch
    tri, tg = _lib()
    n, dim, D, M, p, iters, k = 20_000, 768, 32, 64, 4, 64, 10
    for np_dt, dt in ((np.float16, tri.TRI_F16), (np.float32, tri.TRI_F32)):
        Xt, _ = graph_inputs.make_points(n, dim, 12, np_dt, graph_inputs.SEED_POINTS, device="cuda")
        Qf, _ = graph_inputs.make_points(48, dim, 12, np_dt, graph_inputs.SEED_QUERIES, device="cuda")
        Gt = graph_inputs.make_graph(Xt, D, 8, graph_inputs.SEED_EDGES)
        X = Xt.cpu().numpy()
        stored = np.arange(48) * 397 % n
        Q = np.concatenate([X[stored], Qf.cpu().numpy()])
        seeds = graph_inputs.entry_points(n, 64)
        with tg.GraphPool(Xt, Gt.to(dtype=torch.int32), seeds, dt, slots=64, topm=M, parents=p, max_iters=iters) as pool:
            ids, dist, n_out, it, ev, steps = pool.run_all(Q, k, tri.TRI_L2)
        found = 0
        for i in range(Q.shape[0]):
            assert int(n_out[i]) == k and len(set(ids[i].tolist())) == k
            true_sc = gs.scores(X, ids[i], Q[i], gs.METRIC_L2)
            assert np.all(np.abs(dist[i] - true_sc) <= 4e-6 * true_sc), f"query {i}: not the difference form of its id"
            assert np.all(dist[i][:-1] <= dist[i][1:])
            if i < 48 and stored[i] in ids[i]:
                found += 1
                assert int(ids[i][0]) == int(stored[i]) and dist[i][0] == 0.0, f"query {i}: its own row is not at distance 0"
        _say(f"L2 difference form ({np.dtype(np_dt).name}): {found}/48 stored queries found their own row, each at distance exactly 0")
        assert found >= 40


def test_real_valued_data_same_trajectories_where_no_decision_is_a_near_tie():
    """Real-valued fp16 data, inner product.  A search is a chain of decisions taken on scores; the oracle reports
    the smallest relative gap between neighbouring scores at any decision of a query (min_gap).  How far the
    kernel's fp32 sums are from the oracle's fp64 ones is measured on the returned scores; every query whose min_gap
    is above eight times that must come out with the oracle's ids, in its order, after the same number of extends and distance
    evaluations, every score within the fp16 tolerance of the oracle's.  The others (a near-tie somewhere) may
    take another valid path: their results must be well-formed, every score its id's true score, and recall against
    brute force as good as the oracle's."""
    tri, tg = _lib()
    n, nq, dim, D, M, p, iters, k = 50_000, 256, 768, 32, 64, 4, 64, 10
    Xt, Z = graph_inputs.make_points(n, dim, 12, np.float16, graph_inputs.SEED_POINTS, device="cuda")
    Qt, _ = graph_inputs.make_points(nq, dim, 12, np.float16, graph_inputs.SEED_QUERIES, device="cuda")
    Gt = graph_inputs.make_graph(Xt, D, 8, graph_inputs.SEED_EDGES)
    X, Q, G = Xt.cpu().numpy(), Qt.cpu().numpy(), Gt.cpu().numpy().astype(np.uint32)
    seeds = graph_inputs.entry_points(n, 64)
    with tg.GraphPool(Xt, Gt.to(dtype=__import__("torch").int32), seeds, tri.TRI_F16, slots=128, topm=M, parents=p,
                      max_iters=iters) as pool:
        ids, dist, n_out, it, ev, steps = pool.run_all(Q, k, tri.TRI_IP)
    want = _oracle_all(X, G, seeds, Q, k, tri.TRI_IP, M, p, iters)
    true_ids, _ = bruteforce.knn(X, Q, k, bruteforce.METRIC_IP)
    # how far the kernel's fp32 sums are from the fp64 ones, measured on every returned score; a decision whose two
    # scores differ by eight times that (relative) cannot come out the other way
    worst = 0.0
    for i in range(nq):
        true_sc = gs.scores(X, ids[i], Q[i], gs.METRIC_IP)
        worst = max(worst, float(np.max(np.abs(dist[i] - true_sc) / np.abs(true_sc))))
    clear_gap = max(8.0 * worst, 2e-6)
    _say(f"real-valued: kernel scores within {worst:.2e} relative of the fp64 sums; decisions count as clear above {clear_gap:.2e}")
    clear = 0
    for i in range(nq):
        assert int(n_out[i]) == k and len(set(ids[i].tolist())) == k
        true_sc = gs.scores(X, ids[i], Q[i], gs.METRIC_IP)
        assert np.all(np.abs(dist[i] - true_sc) <= 2e-3 * np.abs(true_sc) + 4e-6), f"query {i}: a score is not its id's score"
        assert np.all(dist[i][:-1] >= dist[i][1:])
        if want[i]["min_gap"] > clear_gap:
            clear += 1
            assert np.array_equal(ids[i], want[i]["ids"]), f"query {i} (min_gap {want[i]['min_gap']:.2e}): ids differ from the oracle's"
            assert int(it[i]) == want[i]["iters"] and int(ev[i]) == want[i]["evals"], f"query {i}: another trajectory"
            assert np.all(np.abs(dist[i] - want[i]["dist"]) <= 2e-3 * np.abs(want[i]["dist"]) + 4e-6)
    r_gpu = bruteforce.recall_at_k(ids, true_ids)
    r_orc = bruteforce.recall_at_k(np.stack([w["ids"] for w in want]), true_ids)
    _say(f"real-valued: {clear}/{nq} queries without a near-tie at any decision, all identical to the oracle; recall@{k} GPU "
         f"{r_gpu:.4f}, oracle {r_orc:.4f}; mean extends {it.mean():.1f} (oracle {np.mean([w['iters'] for w in want]):.1f})")
    assert clear >= nq // 4 and abs(r_gpu - r_orc) <= 0.02


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_configurations_against_the_oracle(seed):
    """Seeded random shapes: database size, dimension (any), degree, topM, parents, entry points, extend budget, slots and
    groups, storage type, per-query k and metric, random neighbour lists with padding and self-loops -- on integer-valued
    data, so everything must equal the oracle exactly."""
    tri, tg = _lib()
    rng = np.random.default_rng(seed)
    for case in range(4):
        n = int(rng.integers(1, 5000))
        dim = int(rng.choice([1, 5, 33, 64, 100, 128, 300, 640]))
        degree = int(rng.choice([1, 2, 7, 16, 32, 64]))
        p = int(rng.integers(1, max(2, 256 // degree + 1)))
        M = int(rng.integers(1, 257))
        iters = int(rng.choice([0, 1, 5, 30, 30, 64]))
        n_seeds = int(rng.integers(1, 257))
        f16 = bool(rng.integers(0, 2))
        dt = np.float16 if f16 else np.float32
        X = rng.integers(-6, 7, size=(n, dim)).astype(dt)
        G = rng.integers(0, n, size=(n, degree)).astype(np.uint32)
        G[rng.random(G.shape) < 0.05] = tg.TRI_GRAPH_PAD
        seeds = rng.integers(0, n + 3, size=n_seeds).astype(np.uint32)          # duplicates and a few invalid ones
        nq = int(rng.integers(1, 90))
        Q = rng.integers(-6, 7, size=(nq, dim)).astype(dt)
        k = rng.integers(1, M + 1, size=nq).astype(np.uint32)
        metric = rng.integers(0, 2, size=nq).astype(np.uint32)
        slots, groups = int(rng.integers(1, 40)), int(rng.integers(1, 5))
        _say(f"random case {seed}.{case}: n {n} dim {dim} {'f16' if f16 else 'f32'} degree {degree} p {p} topM {M} extends <= {iters} "
             f"entry points {n_seeds} queries {nq} slots {slots} groups {groups}")
        want = _oracle_all(X, G, seeds, Q, k, metric, M, p, iters)
        with tg.GraphPool(X, G, seeds, tri.TRI_F16 if f16 else tri.TRI_F32, slots=slots, topm=M, parents=p, max_iters=iters,
                          max_outstanding=256, groups=groups) as pool:
            got = pool.run_all(Q, k, metric)
            _check_exact(got[:5], want, k)


def test_largest_shapes_and_degenerate_graphs():
    """The limits of the implementation in one pool -- topM 256, parents * degree 256, 256 entry points, rows of
    4096 bytes, k = topM, a database whose size is no multiple of 32 -- and degenerate graphs: degree 1 (a ring),
    every neighbour entry padding, a single row."""
    tri, tg = _lib()
    rng = np.random.default_rng(3)
    n, dim = 1003, 2048
    X = rng.integers(-3, 4, size=(n, dim)).astype(np.float16)
    Q = rng.integers(-3, 4, size=(40, dim)).astype(np.float16)
    G = rng.integers(0, n, size=(n, 32)).astype(np.uint32)
    seeds = rng.choice(n, size=256, replace=False).astype(np.uint32)
    want = _oracle_all(X, G, seeds, Q, 256, np.arange(40) % 2, 256, 8, 30)
    with tg.GraphPool(X, G, seeds, tri.TRI_F16, slots=16, topm=256, parents=8, max_iters=30, groups=2) as pool:
        ids, dist, n_out, it, ev, steps = pool.run_all(Q, 256, (np.arange(40) % 2).astype(np.uint32))
        _check_exact((ids, dist, n_out, it, ev), want, 256)
        assert int(ev.max()) > 700                                   # most of the database was scored
    # a ring of degree 1, one entry point: one new row per extend until the walk stops improving
    Xr = np.arange(64, dtype=np.float32).reshape(64, 1)
    Gr = ((np.arange(64) + 1) % 64).astype(np.uint32).reshape(64, 1)
    qr = np.array([[20.25]], dtype=np.float32)
    want = _oracle_all(Xr, Gr, [3], qr, 4, tri.TRI_L2, 4, 1, 100)
    with tg.GraphPool(Xr, Gr, np.array([3], dtype=np.uint32), tri.TRI_F32, slots=1, topm=4, parents=1, max_iters=100) as pool:
        got = pool.run_all(qr, 4, tri.TRI_L2)
        _check_exact(got[:5], want, 4)
        assert int(got[3][0]) == want[0]["iters"] >= 18
    # no edges at all: the answer is the entry points, after one extend that finds nothing
    Gp = np.full((64, 2), tg.TRI_GRAPH_PAD, dtype=np.uint32)
    want = _oracle_all(Xr, Gp, [5, 30, 31], qr, 3, tri.TRI_L2, 8, 2, 10)
    with tg.GraphPool(Xr, Gp, np.array([5, 30, 31], dtype=np.uint32), tri.TRI_F32, slots=3, topm=8, parents=2, max_iters=10) as pool:
        got = pool.run_all(qr, 3, tri.TRI_L2)
        _check_exact(got[:5], want, 3)
        assert list(got[0][0]) == [30, 31, 5] and int(got[3][0]) == 1
    # a database of one row
    X1 = np.array([[2.0, 1.0]], dtype=np.float32)
    G1 = np.zeros((1, 1), dtype=np.uint32)
    with tg.GraphPool(X1, G1, np.array([0], dtype=np.uint32), tri.TRI_F32, slots=2, topm=2, parents=1, max_iters=5) as pool:
        ids, dist, n_out, it, ev, _ = pool.run_all(np.array([[1.0, 1.0]], dtype=np.float32), 2, tri.TRI_IP)
        assert list(ids[0]) == [0, -1] and dist[0, 0] == 3.0 and int(n_out[0]) == 1 and int(ev[0]) == 1
        ids, dist, n_out, it, ev, _ = pool.run_all(np.zeros((0, 2), dtype=np.float32), np.zeros(0, dtype=np.uint32),
                                                   np.zeros(0, dtype=np.uint32))     # an empty batch
        assert ids.shape[0] == 0


@pytest.mark.timeout(600)
def test_full_size_in_the_benchmark_configuration():
    """The workload and launch configuration bench.py --workload graph times (1M x 768 fp16, degree 32, topM 128,
    4 parents, 8192 slots in 3 groups, device-resident queries): a sample of the batch against the oracle, query
    by query.  On this real-valued data trajectories may differ where scores nearly tie, so every sampled result
    must be valid and nearly all must equal the oracle's."""
    import torch
    tri, tg = _lib()
    n, dim, D, M, p, iters, k, S = 1_000_000, 768, 32, 128, 4, 64, 10, 8192
    X, Z = graph_inputs.make_points(n, dim, 12, np.float16, graph_inputs.SEED_POINTS, device="cuda")
    Qv, _ = graph_inputs.make_points(2 * S, dim, 12, np.float16, graph_inputs.SEED_QUERIES, device="cuda")
    G = graph_inputs.make_graph(Z, D, 8, graph_inputs.SEED_EDGES, block=1024).to(torch.int32)
    seeds = graph_inputs.entry_points(n, 64)
    torch.cuda.synchronize()
    _say("full size: inputs ready")
    with tg.GraphPool(X, G, seeds, tri.TRI_F16, slots=S, topm=M, parents=p, max_iters=iters, max_outstanding=4 * S,
                      groups=3, own_stream=True) as pool:
        ids, dist, n_out, it, ev, steps = pool.run_all(Qv, k, tri.TRI_IP)
    Xh, Gh, Qh = X.cpu().numpy(), G.cpu().numpy().astype(np.uint32), Qv.cpu().numpy()
    sel = np.arange(0, 2 * S, 64)
    worst = max(float(np.max(np.abs(dist[i] - gs.scores(Xh, ids[i], Qh[i], gs.METRIC_IP)) / np.abs(gs.scores(Xh, ids[i], Qh[i], gs.METRIC_IP))))
                for i in sel)
    clear_gap = max(8.0 * worst, 2e-7)     # (the kernel's sums are this close to the fp64 ones on the returned scores)
    same = clear = 0
    for i in sel:
        w = gs.search(Xh, Gh, seeds, Qh[i], k, M, p, iters, gs.METRIC_IP)
        assert int(n_out[i]) == w["n"] == k and len(set(ids[i].tolist())) == k
        true_sc = gs.scores(Xh, ids[i], Qh[i], gs.METRIC_IP)
        assert np.all(np.abs(dist[i] - true_sc) <= 2e-3 * np.abs(true_sc) + 4e-6)
        assert np.all(dist[i][:-1] >= dist[i][1:])
        identical = np.array_equal(ids[i], w["ids"]) and int(it[i]) == w["iters"] and int(ev[i]) == w["evals"]
        same += identical
        if w["min_gap"] > clear_gap:        # no decision of this query was a near-tie: the trajectory is determined
            clear += 1
            assert identical, f"query {i} (min_gap {w['min_gap']:.2e}): not the oracle's trajectory"
    _say(f"full size: {steps} steps, {same}/{sel.size} sampled queries with the oracle's ids, extends and evaluations "
         f"({clear} of them without a near-tie at any decision: gaps above {clear_gap:.1e}, eight times the kernel's measured error)")
    assert same >= 0.97 * sel.size


def test_serving_loop_continuous_and_static_batches():
    """graph_run_stream: timed arrivals, results delivered as steps complete, with continuous batching and with
    static batches -- identical to the step-by-step results (which equal the oracle's, tested above) either way;
    every latency is positive."""
    tri, tg = _lib()
    n, nq, dim, D, M, p, iters = 20_000, 400, 128, 16, 32, 2, 30
    Xt, Z = graph_inputs.make_points(n, dim, 8, np.float32, graph_inputs.SEED_POINTS, integer=True)
    Qt, _ = graph_inputs.make_points(nq, dim, 8, np.float32, graph_inputs.SEED_QUERIES, integer=True)
    X, Q, G = Xt.numpy(), Qt.numpy(), graph_inputs.make_graph(Z, D, 4, graph_inputs.SEED_EDGES).numpy().astype(np.uint32)
    seeds = graph_inputs.entry_points(n, 16)
    k = np.random.default_rng(2).integers(1, M + 1, size=nq).astype(np.uint32)
    metric = (np.arange(nq) % 2).astype(np.uint32)
    arrival = np.cumsum(np.random.default_rng(3).exponential(20e-6, size=nq))        # about 50,000 arrivals a second
    with tg.GraphPool(X, G, seeds, tri.TRI_F32, slots=48, topm=M, parents=p, max_iters=iters, max_outstanding=512,
                      groups=2) as pool:
        ref = pool.run_all(Q, k, metric)
        steps = {}
        for static in (False, True):
            ids, dist, n_out, done_s, st = pool.run_stream(Q, arrival, k, metric, static_batches=static)
            for i in range(nq):
                kk = int(k[i])
                assert np.array_equal(ids[i, :kk], ref[0][i, :kk]) and int(n_out[i]) == int(ref[2][i])
                assert np.array_equal(dist[i, :kk].view(np.uint32), ref[1][i, :kk].view(np.uint32))
            assert np.all(done_s > arrival) and st.wall_s >= done_s.max() - 1e-9
            steps[static] = int(st.steps)
            _say(f"stream, static batches {static}: {st.steps} steps, p50 latency {np.percentile(done_s - arrival, 50) * 1e3:.3f} ms, "
                 f"p99 {np.percentile(done_s - arrival, 99) * 1e3:.3f} ms")
        assert min(steps.values()) > 0                                  # (how many steps each scheme needs depends on timing)
        again = pool.run_all(Q, k, metric)                              # the pool is usable step by step afterwards
        assert np.array_equal(again[0], ref[0])
        with pytest.raises(tri.TriError):
            pool.run_stream(Q, arrival[::-1].copy(), k, metric)          # arrival times must not decrease


def test_high_class_is_admitted_first():
    """Two classes: with every slot taken and low-class queries waiting, a high-class query submitted later gets the
    first slot that frees."""
    tri, tg = _lib()
    rng = np.random.default_rng(8)
    n, dim = 4000, 32
    X = rng.integers(-4, 5, size=(n, dim)).astype(np.float32)
    G = rng.integers(0, n, size=(n, 8)).astype(np.uint32)
    Q = rng.integers(-4, 5, size=(12, dim)).astype(np.float32)
    seeds = rng.choice(n, size=8, replace=False).astype(np.uint32)
    with tg.GraphPool(X, G, seeds, tri.TRI_F32, slots=2, topm=16, parents=2, max_iters=20, max_outstanding=64, groups=1) as pool:
        low, rc = pool.submit(Q[:10], 5, tri.TRI_L2)
        pool.step()                                                   # two low-class queries running, eight waiting
        high, rc = pool.submit(Q[10:11], 5, tri.TRI_L2, klass=np.array([tri.TRI_CLASS_HIGH], dtype=np.uint32))
        done_at = {}
        for step in range(1, 2000):
            st = pool.step()
            pool.sync()
            for name, t in [("high", high[0])] + [(f"low{i}", t) for i, t in enumerate(low)]:
                if name not in done_at:
                    status = pool.poll(np.array([t], dtype=np.uint64), 5)[5]
                    if status[0] == tri.TRI_OK:
                        done_at[name] = step
            if len(done_at) == 11:
                break
        assert len(done_at) == 11
        # none of the eight low-class queries that were waiting when it arrived finishes before it started, and at
        # least six of them finish strictly after it (at most one can share its step in the other slot each time)
        later = sum(1 for i in range(2, 10) if done_at[f"low{i}"] > done_at["high"])
        assert later >= 6, done_at
        want = _oracle_all(X, G, seeds, Q[10:11], 5, tri.TRI_L2, 16, 2, 20)
        ids, dist, n_out, it, ev, _ = pool.run_all(Q[10:11], 5, tri.TRI_L2)
        _check_exact((ids, dist, n_out, it, ev), want, 5)


def test_argument_errors_and_empty_steps():
    tri, tg = _lib()
    X = np.arange(32, dtype=np.float32).reshape(16, 2)
    G = np.stack([(np.arange(16) + 1) % 16, (np.arange(16) + 15) % 16], axis=1).astype(np.uint32)
    seeds = np.array([0], dtype=np.uint32)
    with pytest.raises(tri.TriError):
        tg.GraphPool(X, G, seeds, tri.TRI_F32, slots=4, topm=300, parents=1, max_iters=5)
    with pytest.raises(tri.TriError):
        tg.GraphPool(X, G, seeds, tri.TRI_F32, slots=4, topm=8, parents=200, max_iters=5)
    with tg.GraphPool(X, G, seeds, tri.TRI_F32, slots=4, topm=8, parents=1, max_iters=5, max_outstanding=6) as pool:
        st = pool.step()                                           # nothing to do: a no-op
        assert (st.admitted, st.running, st.pending) == (0, 0, 0)
        with pytest.raises(tri.TriError):
            pool.submit(X[:1], 9, tri.TRI_L2)                      # k > topm
        with pytest.raises(tri.TriError):
            pool.submit(X[:1], 2, 7)                               # metric
        t, rc = pool.submit(X[:8], 2, tri.TRI_L2)
        assert rc == tri.TRI_EAGAIN and t.shape[0] == 6            # max_outstanding tickets alive
        ids, dist, n_out, iters, evals, status = pool.poll(t, 2)
        assert np.all(status == tri.TRI_EAGAIN)                    # not finished: not delivered, not consumed
        for _ in range(100):
            st = pool.step()
            if st.running == 0 and st.pending == 0:
                break
        pool.sync()
        ids, dist, n_out, iters, evals, status = pool.poll(t, 2)
        assert np.all(status == tri.TRI_OK) and np.all(n_out == 2)
        want = _oracle_all(X, G, seeds, X[:6], 2, tri.TRI_L2, 8, 1, 5)
        _check_exact((ids, dist, n_out, iters, evals), want, 2)
        assert np.all(pool.poll(t, 2)[5] == tri.TRI_ENOENT)        # consumed
        # max_iters = 0: the answer is the entry points' topM
    with tg.GraphPool(X, G, np.array([3, 9], dtype=np.uint32), tri.TRI_F32, slots=2, topm=4, parents=1, max_iters=0) as pool:
        ids, dist, n_out, iters, evals, _ = pool.run_all(X[4:5], 4, tri.TRI_L2)
        assert list(ids[0]) == [3, 9, -1, -1] and int(n_out[0]) == 2 and int(iters[0]) == 0 and int(evals[0]) == 2


def test_several_threads_submit_while_one_steps():
    """graph_submit is safe from several threads while one driver thread steps: integer-valued data, so
    every answer must equal the oracle's exactly, whichever step its request happened to join."""
    import threading
    import time
    tri, tg = _lib()
    n, dim, D, M, p, iters, nq = 4000, 64, 16, 32, 2, 40, 240
    Xt, Z = graph_inputs.make_points(n, dim, 8, np.float32, graph_inputs.SEED_POINTS + 9, integer=True)
    Qt, _ = graph_inputs.make_points(nq, dim, 8, np.float32, graph_inputs.SEED_QUERIES + 9, integer=True)
    Gt = graph_inputs.make_graph(Z, D, 4, graph_inputs.SEED_EDGES + 9)
    X, Q, G = Xt.numpy(), Qt.numpy(), Gt.numpy().astype(np.uint32)
    seeds = graph_inputs.entry_points(n, 16).astype(np.uint32)
    k = np.random.default_rng(3).integers(1, M + 1, size=nq).astype(np.uint32)
    metric = (np.arange(nq) % 2).astype(np.uint32)
    want = _oracle_all(X, G, seeds, Q, k, metric, M, p, iters)
    n_threads = 4
    with tg.GraphPool(X, G, seeds, tri.TRI_F32, slots=24, topm=M, parents=p, max_iters=iters, max_outstanding=1024,
                      groups=3) as pool:
        tickets = np.zeros(nq, dtype=np.uint64)
        errors = []

        def submitter(w):
            try:
                mine = np.arange(w, nq, n_threads)
                for c0 in range(0, mine.size, 5):
                    sel = mine[c0:c0 + 5]
                    t, rc = pool.submit(np.ascontiguousarray(Q[sel]), k[sel], metric[sel])
                    assert rc == tri.TRI_OK and t.shape[0] == sel.size
                    tickets[sel] = t
                    time.sleep(0.0005)
            except Exception as e:          # (reported by the main thread)
                errors.append(e)

        threads = [threading.Thread(target=submitter, args=(w,)) for w in range(n_threads)]
        for th in threads:
            th.start()
        steps = 0
        while True:
            st = pool.step()
            steps += 1
            assert steps < 500000, "graph_step loop did not drain"
            if not any(th.is_alive() for th in threads) and st.running == 0 and st.pending == 0:
                break
        for th in threads:
            th.join()
        assert not errors, errors
        pool.sync()
        assert len(set(tickets.tolist())) == nq, "a ticket was handed out twice"
        ids, dist, n_out, it, ev, status = pool.poll(tickets, M)
        assert np.all(status == tri.TRI_OK)
        _say(f"4 submitters, {steps} steps")
        _check_exact((ids, dist, n_out, it, ev), want, k)
