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
from tests import bruteforce

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[graph] {msg}", flush=True)


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
        assert np.array_equal(dist[i, :kk].view(np.uint32), w["dist"].view(np.uint32)), f"query {i}: scores"


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


def test_real_valued_data_valid_results_and_recall():
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
    same = 0
    for i in range(nq):
        assert int(n_out[i]) == k and len(set(ids[i].tolist())) == k
        true_sc = gs.scores(X, ids[i], Q[i], gs.METRIC_IP)
        assert np.all(np.abs(dist[i] - true_sc) <= 2e-3 * np.abs(true_sc) + 4e-6), f"query {i}: a score is not its id's score"
        assert np.all(dist[i][:-1] >= dist[i][1:])
        same += np.array_equal(ids[i], want[i]["ids"])
    r_gpu = bruteforce.recall_at_k(ids, true_ids)
    r_orc = bruteforce.recall_at_k(np.stack([w["ids"] for w in want]), true_ids)
    _say(f"real-valued: recall@{k} GPU {r_gpu:.4f}, oracle {r_orc:.4f}; {same}/{nq} queries identical to the oracle; "
         f"mean extends {it.mean():.1f} (oracle {np.mean([w['iters'] for w in want]):.1f})")
    assert abs(r_gpu - r_orc) <= 0.02 and same >= 0.9 * nq


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
