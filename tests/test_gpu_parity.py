"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle."""
import json
import os

import numpy as np
import pytest

import oracle
from oracle import index as oindex
import workloads
from tests import bruteforce, checker, harness

pytestmark = pytest.mark.gpu

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


def _say(msg):
    harness.say(msg)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_worked_examples_through_the_library(dtype):
    """The hand-computed examples: centroids given, lists = best-centroid assignment, results exact."""
    tri = harness.lib()
    np_dt, code = (np.float32, tri.TRI_F32) if dtype == "f32" else (np.float16, tri.TRI_F16)
    with open(GOLDEN) as f:
        data = json.load(f)
    for case in data["cases"]:
        _say(f"worked example {case['name']} {dtype}")
        base = np.asarray(case["base"], dtype=np_dt)
        metric = tri.TRI_L2 if case["metric"] == "l2" else tri.TRI_IP
        with harness.default_pool(tri, slots=8, max_nlist=16, max_total_lists=16, max_dim=case["dim"],
                                  max_outstanding=16) as pool:
            idx = pool.build_index(base, case["dim"], len(case["centroids"]), code, metric, 0,
                                   centroids=np.asarray(case["centroids"], dtype=np.float32))
            cent, off, ids = tri.ivf_export(idx)
            assert [ids[int(off[l]):int(off[l + 1])].tolist() for l in range(len(case["lists"]))] == case["lists"]
            for qc in case["queries"]:
                vec = np.asarray([qc["q"]], dtype=np_dt)
                q = tri.make_queries(idx, vec, qc["k"], qc["nprobe"], metric)
                got_ids, got_dist, n_out, probes, _ = harness.run_all(tri, pool, q)
                n = len(qc["ids"])
                assert int(n_out[0]) == n
                assert probes[0].tolist() == qc["probe"]
                assert got_ids[0, :n].tolist() == qc["ids"]
                assert got_dist[0, :n].tolist() == [float(v) for v in qc["dist"]]
                assert np.all(got_ids[0, n:] == -1)
                assert np.all(got_dist[0, n:] == (np.inf if metric == tri.TRI_L2 else -np.inf))


def test_config0_whole_against_oracle_and_bruteforce():
    """Configuration 0: GPU k-means build (10 Lloyd iterations), nprobe 8 / k 10 against the oracle,
    nprobe = nlist against exact kNN, clustering objective against the oracle's own Lloyd."""
    tri = harness.lib()
    cfg = workloads.CONFIGS[0]
    base, queries, rows = workloads.make_config01(cfg)
    _say("config 0: build")
    with harness.default_pool(tri, max_dim=cfg.dim) as pool:
        idx = pool.build_index(base, cfg.dim, cfg.nlist, tri.TRI_F32, tri.TRI_L2, cfg.train_iters,
                               centroids=base[rows])
        oidx = harness.oracle_index(tri, idx, base)
        rep = oindex.check_index(oidx, oracle.METRIC_L2, tol=1e-4)
        _say(f"config 0: index check {rep}")
        own = oindex.build_index(base, base[rows], oracle.METRIC_L2, train_iters=cfg.train_iters)
        j_gpu, j_own = oindex.inertia(base, oidx, 0), oindex.inertia(base, own, 0)
        assert abs(j_gpu - j_own) <= 0.01 * j_own, (j_gpu, j_own)
        q = tri.make_queries(idx, queries, cfg.k, cfg.nprobe, tri.TRI_L2)
        ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
        rep = harness.compare_with_oracle(oidx, base, queries, cfg.k, cfg.nprobe, 0, ids, dist, n_out, probes)
        _say(f"config 0: parity {rep}")
        true_ids, _ = bruteforce.knn(base, queries, cfg.k, 0)
        assert bruteforce.recall_at_k(ids, true_ids) >= 0.9
        q = tri.make_queries(idx, queries, cfg.k, cfg.nlist, tri.TRI_L2)
        ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
        rep = harness.compare_with_oracle(oidx, base, queries, cfg.k, cfg.nlist, 0, ids, dist, n_out, probes)
        assert np.array_equal(ids, true_ids), "nprobe = nlist must be exact kNN"


def _build_f32(tri, pool, cfg, base, rows):
    return pool.build_index(base, cfg.dim, cfg.nlist, tri.TRI_F32, tri.TRI_L2, cfg.train_iters, centroids=base[rows])


@pytest.mark.parametrize("scale", ["scaled", "full"])
def test_config1_integer_data_is_bit_exact(scale):
    """Configuration 1 (byte-valued fp32, d=128): every partial sum is an integer below 2^24, so the
    fp32 distances must equal the oracle's bit for bit and ties are true ties (strict mode)."""
    tri = harness.lib()
    cfg = workloads.CONFIGS[1]
    if scale == "scaled":
        cfg = cfg.scaled(n_base=100_000, n_components=128, nlist=128, n_queries=300)
    _say(f"config 1 {scale}: generate")
    base, queries, rows = workloads.make_config01(cfg)
    nprobe = 16 if scale == "scaled" else cfg.nprobe
    with harness.default_pool(tri, slots=1024, items_per_step=32768, max_dim=cfg.dim, max_nlist=1024,
                              max_total_lists=1024, score_capacity=96 << 20) as pool:
        _say(f"config 1 {scale}: build")
        idx = _build_f32(tri, pool, cfg, base, rows)
        oidx = harness.oracle_index(tri, idx, base)
        rep = oindex.check_index(oidx, oracle.METRIC_L2, tol=1e-4, sample=20000, seed=7)
        _say(f"config 1 {scale}: index check {rep}, longest list {tri.ivf_info(idx)['max_list_len']}")
        q = tri.make_queries(idx, queries, cfg.k, nprobe, tri.TRI_L2)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        _say(f"config 1 {scale}: {len(stats)} steps; compare")
        rep = harness.compare_with_oracle(oidx, base, queries, cfg.k, nprobe, 0, ids, dist, n_out, probes, strict=True)
        _say(f"config 1 {scale}: parity {rep}")
        assert rep["checked"] == cfg.n_queries
        if scale == "full":
            sub = np.arange(0, cfg.n_queries, 8)
            true_ids, _ = bruteforce.knn(base, queries[sub], cfg.k, 0)
            rec = bruteforce.recall_at_k(ids[sub], true_ids)
            _say(f"config 1 full: recall@10 = {rec:.4f}")
            assert rec >= 0.9


def _f16_setup(tri, cfg, pool_over=None):
    import torch
    base_t, queries_t, rows = workloads.make_config_f16(cfg, device="cuda")
    torch.cuda.synchronize()
    base = base_t.cpu().numpy()
    queries = queries_t.cpu().numpy()
    return base_t, base, queries, rows


@pytest.mark.parametrize("scale", ["scaled", "full"])
def test_config2_fp16_inner_product_heterogeneous(scale):
    """Configuration 2: fp16 unit-norm embeddings, inner product, per-query k in {1,10,100} and nprobe
    in {8..128}.  Full size checks a seeded sample of queries one by one."""
    tri = harness.lib()
    cfg = workloads.CONFIGS[2]
    if scale == "scaled":
        cfg = cfg.scaled(n_base=60_000, n_components=256, nlist=256, n_queries=200)
    _say(f"config 2 {scale}: generate")
    base_t, base, queries, rows = _f16_setup(tri, cfg)
    k, nprobe = workloads.hetero_params(cfg.n_queries, cfg.seed_params)
    with harness.default_pool(tri, slots=2048, items_per_step=1 << 18, max_dim=cfg.dim, max_nlist=4096,
                              max_total_lists=4096, score_capacity=128 << 20) as pool:
        _say(f"config 2 {scale}: build")
        idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, cfg.train_iters,
                               centroids=base[rows].astype(np.float32))
        oidx = harness.oracle_index(tri, idx, base)
        rep = oindex.check_index(oidx, oracle.METRIC_IP, tol=2e-3, sample=5000, seed=7)
        _say(f"config 2 {scale}: index check {rep}, longest list {tri.ivf_info(idx)['max_list_len']}")
        q = tri.make_queries(idx, queries, k, nprobe, tri.TRI_IP)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        sample = None if scale == "scaled" else np.sort(np.random.default_rng(5).choice(cfg.n_queries, 640, replace=False))
        _say(f"config 2 {scale}: {len(stats)} steps; compare")
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, 1, ids, dist, n_out, probes, sample=sample,
                                          batch_first=scale == "full")
        _say(f"config 2 {scale}: parity {rep}")
        assert rep["checked"] == (cfg.n_queries if sample is None else sample.size)
        # the unit-norm identity: the same queries under L2 return the same neighbours (outside ties)
        sub = np.arange(0, cfg.n_queries, max(1, cfg.n_queries // 64))[:64]
        sub_vecs = np.ascontiguousarray(queries[sub])      # must outlive the submit: records hold pointers
        q2 = tri.make_queries(idx, sub_vecs, 10, 16, tri.TRI_L2)
        ids2, dist2, n2, probes2, _ = harness.run_all(tri, pool, q2)
        harness.compare_with_oracle(oidx, base, sub_vecs, 10, 16, 0, ids2, dist2, n2, probes2)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_l2_distances_of_duplicates_and_near_duplicates(dtype):
    """Squared L2 comes back in the difference form: a query that IS a stored vector gets distance exactly zero,
    one that nearly is gets its tiny distance to the relative tolerance (the expanded form the scan ranks with
    would return noise of the size of the norms' rounding there), and no distance is negative."""
    tri = harness.lib()
    rng = np.random.default_rng(91)
    np_dtype = np.float32 if dtype == "f32" else np.float16
    n, d, nlist = 20_000, 96 if dtype == "f32" else 200, 32
    centres = rng.normal(0.0, 2.0, size=(nlist, d))
    base = (3.0 + centres[rng.integers(0, nlist, n)] + rng.normal(0.0, 1.0, size=(n, d))).astype(np_dtype)
    rows = rng.choice(n, 90, replace=False)
    exact = base[rows[:30]]
    near = (base[rows[30:60]].astype(np.float64) + rng.normal(0.0, 2e-3 if dtype == "f32" else 1e-2, size=(30, d))).astype(np_dtype)
    far = (base[rows[60:]].astype(np.float64) + rng.normal(0.0, 1.0, size=(30, d))).astype(np_dtype)
    queries = np.ascontiguousarray(np.concatenate([exact, near, far]))
    with harness.default_pool(tri, slots=64, lists_per_query_step=3, max_dim=d, max_nlist=nlist, max_total_lists=nlist) as pool:
        idx = pool.build_index(base, d, nlist, tri.TRI_F32 if dtype == "f32" else tri.TRI_F16, tri.TRI_L2, 4,
                               centroids=base[rng.choice(n, nlist, replace=False)].astype(np.float32))
        oidx = harness.oracle_index(tri, idx, base)
        q = tri.make_queries(idx, queries, 10, 8, tri.TRI_L2)
        ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
        assert np.all(dist[:, :10] >= 0.0)
        assert np.all(dist[:30, 0] == 0.0)
        for i in range(30):                      # the stored vector itself heads the list (or an identical twin of it)
            assert np.array_equal(base[ids[i, 0]], exact[i])
        true_near = ((base[rows[30:60]].astype(np.float64) - near.astype(np.float64)) ** 2).sum(axis=1)
        assert true_near.min() > 0.0
        _say(f"L2 {dtype}: near-duplicate distances {true_near.min():.3e}..{true_near.max():.3e}, "
             f"returned within {np.max(np.abs(dist[30:60, 0] - true_near) / true_near):.2e} relative")
        assert np.all(ids[30:60, 0] == rows[30:60])
        rep = harness.compare_with_oracle(oidx, base, queries, 10, 8, 0, ids, dist, n_out, probes)
        assert rep["checked"] == 90


@pytest.mark.parametrize("dtype,dim", [("f16", 768), ("f32", 128), ("f32", 384), ("f16", 320), ("f16", 1024)])
def test_a_candidate_region_that_is_too_small_costs_time_not_exactness(dtype, dim):
    """Every query of a step gets a region of the candidate buffer sized by what the scan's filter is expected to
    let through.  With the reserve forced down to a handful of pairs every query asks for more than it was given, and
    the merge kernel scores its lists again itself: the results must be the same bit for bit as with the estimated
    reserve (and as the oracle's), for every kind of scan kernel (register-resident rows of 1536 and 512 bytes, the LDS
    kernel's pipelined 1536-byte fp32 rows, its generic path, 2048-byte rows), both metrics, several steps per query."""
    tri = harness.lib()
    rng = np.random.default_rng(400 + dim)
    np_dtype = np.float32 if dtype == "f32" else np.float16
    n, nlist, nq = 12_000, 24, 60
    centres = rng.normal(0.0, 1.0, size=(nlist, dim))
    base = (centres[rng.integers(0, nlist, n)] + rng.normal(0.0, 0.6, size=(n, dim))).astype(np_dtype)
    queries = np.ascontiguousarray((centres[rng.integers(0, nlist, nq)] + rng.normal(0.0, 0.6, size=(nq, dim))).astype(np_dtype))
    k = rng.choice([1, 10, 100, 300], size=nq).astype(np.uint32)
    nprobe = rng.choice([1, 3, 8], size=nq).astype(np.uint32)
    metric = rng.integers(0, 2, size=nq).astype(np.uint32)
    init = base[rng.choice(n, nlist, replace=False)].astype(np.float32)
    results = {}
    for reserve in (0, 5):
        with harness.default_pool(tri, slots=32, lists_per_query_step=3, kmax=512, max_dim=dim, max_nlist=nlist,
                                  max_total_lists=nlist) as pool:
            idx = pool.build_index(base, dim, nlist, tri.TRI_F32 if dtype == "f32" else tri.TRI_F16, tri.TRI_L2, 3, centroids=init)
            tri.tri_pool_set_candidate_reserve(pool.handle, reserve)
            q = tri.make_queries(idx, queries, k, nprobe, metric)
            ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
            rescans = tri.tri_pool_candidate_rescans(pool.handle)
            if reserve == 0:
                oidx = harness.oracle_index(tri, idx, base)
                rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
                assert rep["checked"] == nq
            results[reserve] = (ids, dist, n_out, rescans, len(stats))
    _say(f"overflow {dtype} dim {dim}: rescans with the estimated reserve {results[0][3]}, with 5 pairs {results[5][3]} "
         f"in {results[5][4]} steps")
    assert results[5][3] > nq / 2 and results[0][3] <= 2
    assert np.array_equal(results[0][0], results[5][0]), "ids differ when the regions overflow"
    assert np.array_equal(results[0][1], results[5][1], equal_nan=True), "scores differ when the regions overflow"
    assert np.array_equal(results[0][2], results[5][2])


def test_scheduling_does_not_change_results():
    """Continuous batching must leave results intact: one batch, one list per step, a short task
    array, fewer slots than queries (slot reuse), and mid-stream arrival all give bit-identical
    ids and scores."""
    tri = harness.lib()
    cfg = workloads.CONFIGS[0].scaled(n_base=20_000, n_components=64, nlist=96, n_queries=150)
    base, queries, rows = workloads.make_config01(cfg)
    k = np.random.default_rng(1).integers(1, 40, size=cfg.n_queries).astype(np.uint32)
    nprobe = np.random.default_rng(2).integers(1, 33, size=cfg.n_queries).astype(np.uint32)
    metric = (np.arange(cfg.n_queries) % 2).astype(np.uint32)
    variants = {
        "one batch": dict(pool=dict(), chunks=None),
        "p=1": dict(pool=dict(lists_per_query_step=1), chunks=None),
        "p=3, W=64": dict(pool=dict(lists_per_query_step=3, items_per_step=64), chunks=None),
        "7 slots": dict(pool=dict(slots=7, max_outstanding=256), chunks=None),
        "mid-stream": dict(pool=dict(lists_per_query_step=2, slots=40), chunks=[1, 5, 20, 3, 50, 1, 1]),
        "tiny score buffer": dict(pool=dict(score_capacity=2048), chunks=None),
        "recorded step": dict(pool=dict(flags=tri.TRI_FLAG_KEEP_PROBES | tri.TRI_FLAG_GRAPH), chunks=None),
        "recorded step, mid-stream": dict(pool=dict(lists_per_query_step=2, slots=40,
                                                    flags=tri.TRI_FLAG_KEEP_PROBES | tri.TRI_FLAG_GRAPH),
                                          chunks=[1, 5, 20, 3, 50, 1, 1]),
    }
    ref = None
    for name, v in variants.items():
        _say(f"invariance: {name}")
        with harness.default_pool(tri, max_dim=cfg.dim, **v["pool"]) as pool:
            idx = _build_f32(tri, pool, cfg, base, rows)
            q = tri.make_queries(idx, queries, k, nprobe, metric)
            ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q, submit_chunks=v["chunks"])
            _say(f"  {len(stats)} steps")
            if ref is None:
                oidx = harness.oracle_index(tri, idx, base)
                harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
                ref = (ids, dist, n_out, probes)
            else:
                assert np.array_equal(ids, ref[0]), name          # entries past a query's k are -1 / nan
                assert np.array_equal(dist.view(np.uint32), ref[1].view(np.uint32)), name
                assert np.array_equal(n_out, ref[2]), name
                assert all(np.array_equal(a, b) for a, b in zip(probes, ref[3])), name


def test_edge_cases():
    """Short lists (n_out < k), empty lists, nprobe = nlist, k = 1 and k = kmax, a single vector."""
    tri = harness.lib()
    rng = np.random.default_rng(11)
    base = rng.standard_normal((500, 20)).astype(np.float32)
    cent = rng.standard_normal((12, 20)).astype(np.float32)
    cent[5] = cent[2]          # duplicated centroid: list 5 is empty (ties go to the smaller number)
    cent[9] = 1e3              # far away: empty under L2
    queries = rng.standard_normal((40, 20)).astype(np.float32)
    with harness.default_pool(tri, max_dim=20, kmax=512, max_nlist=16, max_total_lists=32) as pool:
        idx = pool.build_index(base, 20, 12, tri.TRI_F32, tri.TRI_L2, 0, centroids=cent)
        oidx = harness.oracle_index(tri, idx, base)
        lens = np.diff(oidx.list_off.astype(np.int64))
        assert lens[5] == 0 and lens[9] == 0
        oindex.check_index(oidx, 0, tol=1e-5)
        for k, nprobe in [(1, 1), (512, 1), (512, 12), (7, 12), (100, 3)]:
            for metric in (0, 1):
                _say(f"edge: k={k} nprobe={nprobe} metric={metric}")
                q = tri.make_queries(idx, queries, k, nprobe, metric)
                ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
                harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
        # a query aimed at the far centroid probes the empty list first: zero candidates with nprobe=1
        far = np.full((1, 20), 1e3, dtype=np.float32)
        q = tri.make_queries(idx, far, 5, 1, tri.TRI_L2)
        ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
        assert probes[0].tolist() == [9] and n_out[0] == 0 and np.all(ids[0] == -1) and np.all(np.isinf(dist[0]))
        # one-vector index
        idx1 = pool.build_index(base[:1], 20, 1, tri.TRI_F32, tri.TRI_L2, 0, centroids=cent[:1])
        q = tri.make_queries(idx1, queries[:3], 4, 1, tri.TRI_L2)
        ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
        assert np.all(n_out == 1) and np.all(ids[:, 0] == 0) and np.all(ids[:, 1:] == -1)


def test_argument_errors_and_ticket_lifecycle():
    tri = harness.lib()
    rng = np.random.default_rng(3)
    base = rng.standard_normal((300, 16)).astype(np.float32)
    with harness.default_pool(tri, slots=4, max_dim=16, kmax=16, nprobe_max=8, max_nlist=8, max_total_lists=8,
                              max_outstanding=6) as pool:
        idx = pool.build_index(base, 16, 8, tri.TRI_F32, tri.TRI_L2, 2, centroids=None, seed=5)
        vec = base[0]
        for kw in (dict(k=0), dict(k=17), dict(nprobe=0), dict(nprobe=9), dict(metric=2), dict(klass=3)):
            args = dict(k=4, nprobe=2, metric=0, klass=1)
            args.update(kw)
            with pytest.raises(tri.TriError) as ei:
                tri.search_submit(pool.handle, idx, vec, **args)
            assert ei.value.status == tri.TRI_EINVAL
        # a step with nothing to do is a no-op
        st = tri.search_step(pool.handle)
        assert (st.admitted, st.items, st.running) == (0, 0, 0)
        # max_outstanding tickets, then EAGAIN
        first8 = np.ascontiguousarray(base[:8])
        qs = tri.make_queries(idx, first8, 4, 2, 0)
        tickets, rc = tri.search_submit_batch(pool.handle, qs)
        assert rc == tri.TRI_EAGAIN and tickets.shape[0] == 6
        assert tri.search_poll(pool.handle, int(tickets[0]), 4) is None        # queued, not finished
        tri.search_cancel(pool.handle, int(tickets[1]))                         # cancel while queued
        st = tri.search_step(pool.handle)
        assert st.admitted == 4 and st.pending_low == 1
        tri.search_cancel(pool.handle, int(tickets[2]))                         # cancel while running
        while True:
            st = tri.search_step(pool.handle)
            if st.running == 0 and st.pending_low == 0 and st.items == 0:
                break
        tri.search_sync(pool.handle)
        for i in (1, 2):
            with pytest.raises(tri.TriError) as ei:
                tri.search_poll(pool.handle, int(tickets[i]), 4)
            assert ei.value.status == tri.TRI_ENOENT
        for i in (0, 3, 4, 5):
            ids, dist, n = tri.search_poll(pool.handle, int(tickets[i]), 4)
            assert n == 4 and ids[0] == i          # the query is a base row: its own nearest neighbour
        with pytest.raises(tri.TriError) as ei:                                 # consumed
            tri.search_poll(pool.handle, int(tickets[0]), 4)
        assert ei.value.status == tri.TRI_ENOENT


def test_two_indexes_two_classes():
    """A pool with an fp16/IP index and an fp32/L2 index; with a saturated slot table a later
    high-class query is admitted before earlier low-class ones."""
    tri = harness.lib()
    cfg_a = workloads.CONFIGS[2].scaled(n_base=20_000, n_components=64, nlist=64, n_queries=60)
    cfg_b = workloads.CONFIGS[0].scaled(n_base=5_000, n_components=16, nlist=32, n_queries=60, dim=40)
    base_a_t, base_a, queries_a, rows_a = _f16_setup(tri, cfg_a)
    base_b, queries_b, rows_b = workloads.make_config01(cfg_b)
    with harness.default_pool(tri, slots=8, max_dim=768, max_outstanding=512, lists_per_query_step=4) as pool:
        ia = pool.build_index(base_a_t, cfg_a.dim, cfg_a.nlist, tri.TRI_F16, tri.TRI_IP, 5,
                              centroids=base_a[rows_a].astype(np.float32))
        ib = pool.build_index(base_b, cfg_b.dim, cfg_b.nlist, tri.TRI_F32, tri.TRI_L2, 5, centroids=base_b[rows_b])
        oa, ob = harness.oracle_index(tri, ia, base_a), harness.oracle_index(tri, ib, base_b)
        qa = tri.make_queries(ia, queries_a, 10, 16, tri.TRI_IP, tri.TRI_CLASS_LOW)
        qb = tri.make_queries(ib, queries_b, 5, 8, tri.TRI_L2, tri.TRI_CLASS_LOW)
        mixed = np.concatenate([qa, qb])
        order = np.random.default_rng(9).permutation(mixed.shape[0])
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, np.ascontiguousarray(mixed[order]),
                                                          submit_chunks=[10, 30, 5])
        inv = np.argsort(order)
        ids, dist, n_out = ids[inv], dist[inv], n_out[inv]
        probes = [probes[i] for i in inv]
        harness.compare_with_oracle(oa, base_a, queries_a, 10, 16, 1, ids[:60], dist[:60], n_out[:60], probes[:60])
        harness.compare_with_oracle(ob, base_b, queries_b, 5, 8, 0, ids[60:], dist[60:], n_out[60:], probes[60:])
        # priority: fill the table and the low queue, then submit one high-class query
        low, _ = tri.search_submit_batch(pool.handle, np.ascontiguousarray(qa[:30]))
        tri.search_step(pool.handle)                       # 8 low-class queries running, 22 waiting
        high = tri.search_submit(pool.handle, ia, queries_a[0], 10, 16, tri.TRI_IP, tri.TRI_CLASS_HIGH)
        done_at = {}
        for step in range(1, 400):
            st = tri.search_step(pool.handle)
            tri.search_sync(pool.handle)
            for name, t in [("high", high)] + [(f"low{i}", int(t)) for i, t in enumerate(low)]:
                if name not in done_at and tri.search_poll(pool.handle, t, 10) is not None:
                    done_at[name] = step
            if len(done_at) == 31:
                break
        assert len(done_at) == 31
        # the high-class query takes the first slot that frees: none of the 22 low-class queries that were
        # waiting before it finishes earlier; those not admitted at that same boundary finish strictly later
        assert all(done_at[f"low{i}"] >= done_at["high"] for i in range(8, 30))
        later = sum(1 for i in range(8, 30) if done_at[f"low{i}"] > done_at["high"])
        assert later >= 22 - 7, f"only {later} of the 22 waiting low-class queries finished after the high-class one"


@pytest.mark.parametrize("dtype,dim", [("f32", 256), ("f32", 384), ("f32", 512), ("f32", 160),
                                       ("f16", 256), ("f16", 512), ("f16", 1024), ("f16", 320)])
def test_every_row_length_class_and_long_lists(dtype, dim):
    """One case per scan-kernel variant not met by the five configurations (rows of 512 / 1024 / 1536 /
    2048 bytes and other lengths, both storage types), with lists long enough to be scanned in several
    chunks, k from 1 to 1000 (no threshold below k sample scores, more candidates than fit in LDS) and
    both metrics."""
    import torch
    tri = harness.lib()
    rng = np.random.default_rng(dim + (7 if dtype == "f16" else 0))
    n, nlist, nq = 30_000, 24, 64
    centres = rng.standard_normal((nlist, dim)).astype(np.float32)
    base = (centres[rng.integers(0, nlist, size=n)] + 0.7 * rng.standard_normal((n, dim))).astype(np.float32)
    queries = (centres[rng.integers(0, nlist, size=nq)] + 0.7 * rng.standard_normal((nq, dim))).astype(np.float32)
    if dtype == "f16":
        scale = 1.0 / np.sqrt(dim)                      # keep squared norms far from the fp16 range limit
        base, queries = (base * scale).astype(np.float16), (queries * scale).astype(np.float16)
        tdt = tri.TRI_F16
    else:
        tdt = tri.TRI_F32
    k = rng.choice(np.array([1, 10, 300, 1000], dtype=np.uint32), size=nq)
    nprobe = rng.integers(1, nlist + 1, size=nq).astype(np.uint32)
    metric = (np.arange(nq) % 2).astype(np.uint32)
    with harness.default_pool(tri, slots=64, items_per_step=64 * nlist, kmax=1024, nprobe_max=nlist, max_dim=dim,
                              max_nlist=nlist, max_total_lists=nlist, score_capacity=64 << 20) as pool:
        idx = pool.build_index(base, dim, nlist, tdt, tri.TRI_L2, 4, centroids=centres)
        info = tri.ivf_info(idx)
        _say(f"{dtype} d={dim}: longest list {info['max_list_len']}")
        assert info["max_list_len"] > 1100                # several chunks per list
        oidx = harness.oracle_index(tri, idx, base)
        q = tri.make_queries(idx, queries, k, nprobe, metric)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
        _say(f"{dtype} d={dim}: parity {rep}")
        # the same through three lists per step: thresholds then come from the running top-k as well -- and with the
        # lists read by non-temporal loads (the kernel variants a pool otherwise takes from 8 GB of vectors on)
        with harness.default_pool(tri, slots=16, items_per_step=48, lists_per_query_step=3, kmax=1024, nprobe_max=nlist,
                                  max_dim=dim, max_nlist=nlist, max_total_lists=nlist, score_capacity=64 << 20,
                                  flags=tri.TRI_FLAG_KEEP_PROBES | tri.TRI_FLAG_STREAM_LISTS) as pool2:
            idx2 = pool2.build_index(base, dim, nlist, tdt, tri.TRI_L2, 4, centroids=centres)
            q2 = tri.make_queries(idx2, queries, k, nprobe, metric)
            ids2, dist2, n2, probes2, stats2 = harness.run_all(tri, pool2, q2)
            assert np.array_equal(ids, ids2) and np.array_equal(n_out, n2)
            assert np.array_equal(dist.view(np.uint32), dist2.view(np.uint32))


def test_recorded_step_replays_match_kernel_by_kernel_launches():
    """TRI_FLAG_GRAPH: the step recorded once as a HIP graph and replayed gives, replay after replay and
    with other GPU work and synchronisations in between, bit for bit what kernel-by-kernel launches
    give -- over two indexes of different storage types, mid-stream arrivals and slot reuse -- and
    survives a change of the set of attached indexes (the recording is made again)."""
    import torch
    tri = harness.lib()
    cfg_a = workloads.CONFIGS[2].scaled(n_base=20_000, n_components=64, nlist=64, n_queries=60)
    cfg_b = workloads.CONFIGS[0].scaled(n_base=5_000, n_components=16, nlist=32, n_queries=60, dim=40)
    base_a_t, base_a, queries_a, rows_a = _f16_setup(tri, cfg_a)
    base_b, queries_b, rows_b = workloads.make_config01(cfg_b)
    order = np.random.default_rng(9).permutation(120)
    inv = np.argsort(order)
    k_a = np.random.default_rng(3).integers(1, 100, size=60).astype(np.uint32)
    results = {}
    scratch = torch.zeros(1 << 20, device="cuda")

    def busy():                        # the program's own work between two replays
        scratch.add_(1.0)
        torch.cuda.synchronize()

    # (the recorded pool also reads its lists with non-temporal loads: recordings are kept per such choice, and the
    # results must not depend on it)
    for name, flags in [("eager", tri.TRI_FLAG_KEEP_PROBES),
                        ("graph", tri.TRI_FLAG_KEEP_PROBES | tri.TRI_FLAG_GRAPH | tri.TRI_FLAG_STREAM_LISTS)]:
        _say(f"recorded step: {name}")
        with harness.default_pool(tri, slots=24, max_dim=768, max_outstanding=512, lists_per_query_step=4,
                                  flags=flags) as pool:
            ia = pool.build_index(base_a_t, cfg_a.dim, cfg_a.nlist, tri.TRI_F16, tri.TRI_IP, 5,
                                  centroids=base_a[rows_a].astype(np.float32))
            qa = tri.make_queries(ia, queries_a, k_a, 16, tri.TRI_IP, tri.TRI_CLASS_LOW)
            if name == "graph":        # steps recorded with one index attached ...
                ids, dist, n_out, probes, _ = harness.run_all(tri, pool, qa, between_steps=busy)
                results["graph, one index"] = (ids, dist, n_out, probes)
            ib = pool.build_index(base_b, cfg_b.dim, cfg_b.nlist, tri.TRI_F32, tri.TRI_L2, 5, centroids=base_b[rows_b])
            qb = tri.make_queries(ib, queries_b, 5, 8, tri.TRI_L2, tri.TRI_CLASS_HIGH)
            mixed = np.ascontiguousarray(np.concatenate([qa, qb])[order])
            runs = []
            for rep in range(3 if name == "graph" else 1):      # ... and again with two
                ids, dist, n_out, probes, stats = harness.run_all(tri, pool, mixed, submit_chunks=[10, 30, 5],
                                                                  between_steps=busy if rep != 1 else None)
                runs.append((ids[inv], dist[inv], n_out[inv], [probes[i] for i in inv]))
                _say(f"  run {rep}: {len(stats)} steps")
            results[name] = runs
            if name == "eager":
                oa, ob = harness.oracle_index(tri, ia, base_a), harness.oracle_index(tri, ib, base_b)
                ids, dist, n_out, probes = runs[0]
                harness.compare_with_oracle(oa, base_a, queries_a, k_a, 16, 1, ids[:60], dist[:60], n_out[:60], probes[:60])
                harness.compare_with_oracle(ob, base_b, queries_b, 5, 8, 0, ids[60:], dist[60:], n_out[60:], probes[60:])
    ref = results["eager"][0]
    for rep, got in enumerate(results["graph"]):
        assert np.array_equal(got[0], ref[0]), f"replayed run {rep}: ids"
        assert np.array_equal(got[1].view(np.uint32), ref[1].view(np.uint32)), f"replayed run {rep}: scores"
        assert np.array_equal(got[2], ref[2]), f"replayed run {rep}: counts"
        assert all(np.array_equal(a, b) for a, b in zip(got[3], ref[3])), f"replayed run {rep}: probe lists"
    one = results["graph, one index"]
    assert np.array_equal(one[0][:, :1], ref[0][:60, :1])       # (same queries, same index: same best neighbour)
    assert float(scratch[0]) > 0


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_configurations_against_the_oracle(seed):
    """Seeded random shapes nobody picked by hand: dimension (any, not only multiples of the row padding), base size,
    number and balance of lists, slots, lists per step, items per step, storage type, per-query k / nprobe / metric /
    class, arrivals in chunks -- each compared with the oracle query by query."""
    tri = harness.lib()
    rng = np.random.default_rng(seed)
    for case in range(3):
        dim = int(rng.choice([3, 17, 40, 64, 100, 128, 200, 257, 384, 500]))
        f16 = bool(rng.integers(0, 2))
        n = int(rng.integers(500, 12_000))
        nlist = int(rng.integers(2, 97))
        nq = int(rng.integers(1, 120))
        spread = float(rng.choice([0.3, 1.0, 3.0]))                  # tight clusters ... one blob (very uneven lists)
        centres = rng.standard_normal((nlist, dim)).astype(np.float32)
        weights = rng.dirichlet(np.full(nlist, 0.5))                 # unbalanced list sizes, some nearly empty
        base = (centres[rng.choice(nlist, size=n, p=weights)] + spread * rng.standard_normal((n, dim))).astype(np.float32)
        queries = (centres[rng.integers(0, nlist, size=nq)] + spread * rng.standard_normal((nq, dim))).astype(np.float32)
        if f16:
            scale = 1.0 / np.sqrt(dim)
            base, queries = (base * scale).astype(np.float16), (queries * scale).astype(np.float16)
        k = rng.integers(1, 130, size=nq).astype(np.uint32)
        nprobe = rng.integers(1, nlist + 1, size=nq).astype(np.uint32)
        metric = rng.integers(0, 2, size=nq).astype(np.uint32)
        klass = rng.integers(0, 2, size=nq).astype(np.uint32)
        slots = int(rng.integers(1, 70))
        p = int(rng.choice([0, 1, 2, 5]))
        items = int(rng.integers(1, 400)) if p else slots * nlist
        chunks = [int(c) for c in rng.integers(1, 30, size=4)]
        _say(f"random case {seed}.{case}: dim {dim} {'f16' if f16 else 'f32'} n {n} nlist {nlist} nq {nq} slots {slots} "
             f"p {p} W {items} spread {spread}")
        with harness.default_pool(tri, slots=slots, items_per_step=items, lists_per_query_step=p, kmax=129, nprobe_max=nlist,
                                  max_dim=dim, max_nlist=nlist, max_total_lists=nlist, max_outstanding=max(256, slots),
                                  score_capacity=32 << 20) as pool:
            idx = pool.build_index(base, dim, nlist, tri.TRI_F16 if f16 else tri.TRI_F32, int(rng.integers(0, 2)), 3,
                                   centroids=centres)
            oidx = harness.oracle_index(tri, idx, base)
            q = tri.make_queries(idx, queries, k, nprobe, metric, klass)
            ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q, submit_chunks=chunks)
            rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
            _say(f"  {len(stats)} steps, parity {rep}")


def test_more_probed_lists_than_cached_segments():
    """nprobe far beyond what the merge kernel caches of candidate segments (200 lists x 4 chunk
    segments in one step), small lists, and a k that keeps nearly everything."""
    tri = harness.lib()
    rng = np.random.default_rng(21)
    n, dim, nlist, nq = 20_000, 64, 200, 48
    centres = rng.standard_normal((nlist, dim)).astype(np.float32) * 2
    base = (centres[rng.integers(0, nlist, size=n)] + rng.standard_normal((n, dim))).astype(np.float32)
    queries = (centres[rng.integers(0, nlist, size=nq)] + rng.standard_normal((nq, dim))).astype(np.float32)
    k = rng.choice(np.array([5, 100, 900], dtype=np.uint32), size=nq)
    nprobe = rng.choice(np.array([150, 200], dtype=np.uint32), size=nq)
    metric = (np.arange(nq) % 2).astype(np.uint32)
    with harness.default_pool(tri, slots=48, items_per_step=48 * 200, kmax=1024, nprobe_max=200, max_dim=dim,
                              max_nlist=nlist, max_total_lists=nlist, score_capacity=64 << 20) as pool:
        idx = pool.build_index(base, dim, nlist, tri.TRI_F32, tri.TRI_L2, 3, centroids=centres)
        oidx = harness.oracle_index(tri, idx, base)
        q = tri.make_queries(idx, queries, k, nprobe, metric)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        assert len(stats) <= 3                            # everything in one scanning step
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
        _say(f"many segments: parity {rep}")


def test_control_loop_moves_the_policy_inside_the_pool():
    """Sec. 3.3's control loop run by search_step: reported signals and the pool's own measurement of the
    high class's waits move the reserved share and the high-class flush time-out in the paper's
    directions, the admission split follows the moved share, and results stay those of the oracle."""
    import time
    tri = harness.lib()
    cfg = workloads.CONFIGS[0].scaled(n_base=8_000, n_components=32, nlist=32, n_queries=96)
    base, queries, rows = workloads.make_config01(cfg)
    fb = tri.tri_feedback_cfg(0.25, 0.75, 0.25, 2.0, 1e-4, 8e-3, 0.9, 0.05, 0.1, 0.0, 50e-6, 0.0)   # period 0: every step
    with harness.default_pool(tri, slots=8, lists_per_query_step=4, max_dim=cfg.dim, max_outstanding=512) as pool:
        idx = _build_f32(tri, pool, cfg, base, rows)
        oidx = harness.oracle_index(tri, idx, base)
        tri.search_set_policy(pool.handle, high_share=0.0, flush_timeout_high_s=4e-3)
        tri.search_set_feedback(pool.handle, fb)
        pol, _ = tri.search_get_policy(pool.handle)
        assert pol.high_share == 0.25                         # clamped into [r_min, r_max] at once
        klass = np.r_[np.full(48, tri.TRI_CLASS_HIGH), np.full(48, tri.TRI_CLASS_LOW)].astype(np.uint32)
        q = tri.make_queries(idx, queries, 10, 16, tri.TRI_L2, klass)
        tickets, rc = tri.search_submit_batch(pool.handle, q)
        tri.search_report_signals(pool.handle, 0.5, 0.0)      # KV link starved -> r rises step by step, then tau shrinks
        shares, taus, waits = [], [], []
        for _ in range(5):
            time.sleep(0.001)                                  # (the waiting high-class queries age past the 50 us budget)
            st = tri.search_step(pool.handle)
            pol, _ = tri.search_get_policy(pool.handle)
            shares.append(round(float(pol.high_share), 3))
            taus.append(pol.flush_timeout_high_s)
            waits.append(tri.search_get_feedback(pool.handle)[1].wait_p95_s)
        assert shares == [0.25, 0.5, 0.75, 0.75, 0.75], shares           # (the first call only starts the clock)
        # tau_pre: halved whenever admitted high-class queries had waited beyond the budget, and once r is at r_max
        assert taus[0] == 4e-3 and all(b <= a for a, b in zip(taus, taus[1:])) and taus[-1] <= taus[0] / 4, taus
        assert max(w for w in waits if w == w) > 50e-6, waits
        periods, last = tri.search_get_feedback(pool.handle)
        assert periods == 4 and abs(last.u_kv - 0.5) < 1e-6
        # link at target, decode stalls rising -> r falls again, down to r_min
        for stall in (0.2, 0.3, 0.4, 0.5):
            tri.search_report_signals(pool.handle, 0.95, stall)
            tri.search_step(pool.handle)
        pol, _ = tri.search_get_policy(pool.handle)
        assert abs(pol.high_share - 0.25) < 1e-6
        tri.search_set_feedback(pool.handle, None)
        tri.search_report_signals(pool.handle, 0.1, 0.0)
        for _ in range(200):
            st = tri.search_step(pool.handle)
            if st.running == 0 and st.pending_high == 0 and st.pending_low == 0 and st.items == 0:
                break
        pol2, _ = tri.search_get_policy(pool.handle)
        assert pol2.high_share == pol.high_share              # switched off: nothing moves any more
        tri.search_sync(pool.handle)
        probes = [tri.search_probes(pool.handle, int(t), 16) for t in tickets]
        ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, 10)
        assert np.all(status == tri.TRI_OK)
        harness.compare_with_oracle(oidx, base, queries, 10, 16, 0, ids, dist, n_out, probes)
        with pytest.raises(Exception):
            tri.search_report_signals(pool.handle, 1.5, 0.0)


def test_streaming_read_probe_measures_something_plausible():
    import torch
    tri = harness.lib()
    buf = torch.ones(64 << 20, dtype=torch.float32, device="cuda")       # 256 MiB
    gbs = tri.tri_stream_read_bandwidth(buf, 5)
    _say(f"streaming read of 256 MiB: {gbs:.0f} GB/s")
    assert 200.0 < gbs < 20000.0


def test_static_batches_drain_before_admitting():
    """tri_policy.static_batches (the scheme continuous batching replaces, kept for comparison): no query is
    admitted while one is running; results are those of continuous batching."""
    tri = harness.lib()
    cfg = workloads.CONFIGS[0].scaled(n_base=8_000, n_components=32, nlist=32, n_queries=40)
    base, queries, rows = workloads.make_config01(cfg)
    nprobe = np.where(np.arange(40) % 5 == 0, 16, 4).astype(np.uint32)         # some queries need 4 steps, most 1
    with harness.default_pool(tri, slots=8, lists_per_query_step=4, max_dim=cfg.dim, max_outstanding=512) as pool:
        idx = _build_f32(tri, pool, cfg, base, rows)
        q = tri.make_queries(idx, queries, 10, nprobe, tri.TRI_L2)
        ref = harness.run_all(tri, pool, q)
        tri.search_set_policy(pool.handle, static_batches=True)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        tri.search_set_policy(pool.handle)
        assert np.array_equal(ids, ref[0]) and np.array_equal(dist.view(np.uint32), ref[1].view(np.uint32))
        # (admitted, retired, running, items) per step: admissions only into an empty table, 8 at a time
        running_before = 0
        for admitted, retired, running, items in stats:
            assert admitted == 0 or (running_before == 0 and admitted == min(8, admitted))
            running_before = running - retired
        assert len(stats) > len(ref[4])                                   # the drain costs steps
        assert sum(a for a, _, _, _ in stats) == 40


def test_scheduling_policy_reservation_slack_and_flush():
    """The step-boundary policy of the paper's Sec. 3.3 on the GPU path: the reserved share splits the free
    slots between the classes, the slack order admits the most urgent high-class query first, flush
    time-outs let an idle pool collect a fuller batch -- and none of it changes any result."""
    tri = harness.lib()
    cfg = workloads.CONFIGS[0].scaled(n_base=8_000, n_components=32, nlist=32, n_queries=96)
    base, queries, rows = workloads.make_config01(cfg)
    with harness.default_pool(tri, slots=8, lists_per_query_step=4, max_dim=cfg.dim, max_outstanding=512) as pool:
        idx = _build_f32(tri, pool, cfg, base, rows)
        oidx = harness.oracle_index(tri, idx, base)
        # (a) reserved share: 8 free slots, 40 + 40 waiting
        klass = np.r_[np.full(40, tri.TRI_CLASS_HIGH), np.full(40, tri.TRI_CLASS_LOW)].astype(np.uint32)
        q = tri.make_queries(idx, queries[:80], 10, 16, tri.TRI_L2, klass)
        for share, want in ((0.25, (2, 6)), (1.0, (8, 0)), (0.0, (0, 8))):
            tri.search_set_policy(pool.handle, high_share=share)
            tickets, rc = tri.search_submit_batch(pool.handle, q)
            st = tri.search_step(pool.handle)
            assert (40 - st.pending_high, 40 - st.pending_low) == want, (share, st.pending_high, st.pending_low)
            for _ in range(200):
                st = tri.search_step(pool.handle)
                if st.running == 0 and st.pending_high == 0 and st.pending_low == 0 and st.items == 0:
                    break
            tri.search_sync(pool.handle)
            probes = [tri.search_probes(pool.handle, int(t), 16) for t in tickets]
            ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, 10)
            assert np.all(status == tri.TRI_OK)
            harness.compare_with_oracle(oidx, base, queries[:80], 10, 16, 0, ids, dist, n_out, probes)
        # with a share of 0.25 the low class is not starved while the high-class queue stays long
        tri.search_set_policy(pool.handle, high_share=0.25)
        tickets, rc = tri.search_submit_batch(pool.handle, q)
        for step in range(12):
            tri.search_step(pool.handle)
        tri.search_sync(pool.handle)
        polled = [i for i in range(40, 80) if tri.search_poll(pool.handle, int(tickets[i]), 10) is not None]
        assert len(polled) >= 12, len(polled)             # 6 of 8 slots per generation of 4 steps
        for _ in range(200):
            st = tri.search_step(pool.handle)
            if st.running == 0 and st.pending_high == 0 and st.pending_low == 0 and st.items == 0:
                break
        tri.search_sync(pool.handle)
        rest = np.array([i for i in range(80) if i not in polled])
        _, _, _, status = tri.search_poll_batch(pool.handle, tickets[rest], 10)
        assert np.all(status == tri.TRI_OK)

    # (b) slack order: one slot, three waiting high-class queries
    with harness.default_pool(tri, slots=1, lists_per_query_step=4, max_dim=cfg.dim, max_outstanding=64) as pool:
        idx = _build_f32(tri, pool, cfg, base, rows)
        for order, want in ((tri.TRI_ORDER_SLACK, ["tight", "loose", "none"]), (tri.TRI_ORDER_FIFO, ["loose", "tight", "none"])):
            tri.search_set_policy(pool.handle, order_high=order)
            first = tri.search_submit(pool.handle, idx, queries[0], 5, 16, tri.TRI_L2, tri.TRI_CLASS_LOW)
            tri.search_step(pool.handle)                   # occupies the only slot for four steps
            t = {"loose": tri.search_submit(pool.handle, idx, queries[1], 5, 16, tri.TRI_L2, tri.TRI_CLASS_HIGH, 10**9),
                 "tight": tri.search_submit(pool.handle, idx, queries[2], 5, 16, tri.TRI_L2, tri.TRI_CLASS_HIGH, 10**6),
                 "none": tri.search_submit(pool.handle, idx, queries[3], 5, 16, tri.TRI_L2, tri.TRI_CLASS_HIGH, 0)}
            finished = []
            for step in range(40):
                tri.search_step(pool.handle)
                tri.search_sync(pool.handle)
                for name, tk in t.items():
                    if name not in finished and tri.search_poll(pool.handle, tk, 5) is not None:
                        finished.append(name)
                if len(finished) == 3:
                    break
            assert finished == want, (order, finished)
            assert tri.search_poll(pool.handle, first, 5) is not None
        pol, mean_step = tri.search_get_policy(pool.handle)
        assert pol.order_high == tri.TRI_ORDER_FIFO and 0 < mean_step < 0.1

    # (c) flush time-outs in the serving loop: sparse arrivals into an idle pool
    with harness.default_pool(tri, slots=64, lists_per_query_step=0, max_dim=cfg.dim, max_outstanding=512) as pool:
        idx = _build_f32(tri, pool, cfg, base, rows)
        n = 60
        arrival = np.arange(n) * 150e-6                     # one query every 150 us: 9 ms in all
        klass = np.full(n, tri.TRI_CLASS_LOW, dtype=np.uint32)
        klass[30] = tri.TRI_CLASS_HIGH
        q = tri.make_queries(idx, queries[:n], 10, 8, tri.TRI_L2, klass)
        out = {}
        for name, pol in (("at once", dict()), ("global 4 ms", dict(flush_timeout_s=4e-3, flush_timeout_high_s=4e-3)),
                          ("global 4 ms, high 0.3 ms", dict(flush_timeout_s=4e-3, flush_timeout_high_s=0.3e-3))):
            tri.search_set_policy(pool.handle, **pol)
            ids, dist, n_out, done_s, st, _ = tri.search_run_stream(pool.handle, q, arrival, 10)
            out[name] = (ids, st.steps, (done_s - arrival) * 1e3)
            _say(f"flush {name}: {st.steps} steps, mean latency {out[name][2].mean():.2f} ms, high-class query {out[name][2][30]:.2f} ms")
        assert out["global 4 ms"][1] * 3 <= out["at once"][1]                 # far fewer, fuller steps
        assert out["global 4 ms"][2].max() < 4.0 + 8.0                        # nobody waits much beyond the time-out
        assert out["global 4 ms, high 0.3 ms"][2][30] < 0.3 + 2.5             # the high-class query is flushed early
        assert out["global 4 ms, high 0.3 ms"][2][30] < out["global 4 ms"][2][30]
        for name in out:
            assert np.array_equal(out[name][0], out["at once"][0])            # results do not depend on the policy


@pytest.mark.parametrize("scale", ["scaled", "full"])
@pytest.mark.timeout(900)
def test_config3_stream_over_two_indexes(scale):
    """Configuration 3: Poisson arrivals over a RAG index and a prompt-cache index in one pool, driven
    by the library's native serving loop.  Every query is answered; a seeded sample (both kinds) equals
    the oracle; the cache-hit flag (top-1 similarity >= 0.95) agrees with the oracle's top-1 outside the
    tolerance band; latencies are consistent."""
    import torch
    tri = harness.lib()
    if scale == "scaled":
        rag_cfg = workloads.CONFIGS[2].scaled(n_base=60_000, n_components=256, nlist=256, n_queries=0)
        cache_cfg = workloads.CACHE_INDEX.scaled(n_base=20_000, n_components=64, nlist=64, n_queries=0)
        n, slots, rate, n_check = 3000, 256, 2.0e5, 120
    else:
        rag_cfg, cache_cfg = workloads.CONFIGS[2], workloads.CACHE_INDEX
        n, slots, rate, n_check = 100_000, 4096, 4.0e5, 1088
    _say(f"config 3 {scale}: generate")
    w = workloads.make_config3(n, "cuda", rag_cfg, cache_cfg)
    torch.cuda.synchronize()
    rag_base, cache_base = w["rag_base"].cpu().numpy(), w["cache_base"].cpu().numpy()
    queries = np.ascontiguousarray(w["queries"].cpu().numpy())
    arrival = workloads.poisson_arrivals(n, rate, 4003)
    with harness.default_pool(tri, slots=slots, items_per_step=slots * 8, lists_per_query_step=8, kmax=128,
                              nprobe_max=32, max_dim=768, max_nlist=rag_cfg.nlist,
                              max_total_lists=rag_cfg.nlist + cache_cfg.nlist, max_outstanding=4 * slots,
                              score_capacity=256 << 20) as pool:
        _say(f"config 3 {scale}: build two indexes")
        ir = pool.build_index(w["rag_base"], rag_cfg.dim, rag_cfg.nlist, tri.TRI_F16, tri.TRI_IP, rag_cfg.train_iters,
                              centroids=rag_base[w["rag_rows"]].astype(np.float32))
        ic = pool.build_index(w["cache_base"], cache_cfg.dim, cache_cfg.nlist, tri.TRI_F16, tri.TRI_IP,
                              cache_cfg.train_iters, centroids=cache_base[w["cache_rows"]].astype(np.float32))
        index_of = np.where(w["is_rag"], ir, ic).astype(np.uint64)
        q = tri.make_queries(index_of, queries, w["k"], w["nprobe"], tri.TRI_IP, w["klass"])
        _say(f"config 3 {scale}: stream of {n} queries at {rate:.0f}/s")
        ids, dist, n_out, done_s, st, probes = tri.search_run_stream(pool.handle, q, arrival, 100, depth=2, nprobe_max=32)
        lat = done_s - arrival
        _say(f"config 3 {scale}: {n / st.wall_s:.0f} q/s over {st.steps} steps, padding "
             f"{1 - st.items / max(st.capacity, 1):.3f}, latency p50 {np.percentile(lat, 50) * 1e3:.2f} ms "
             f"p99 {np.percentile(lat, 99) * 1e3:.2f} ms, longest queue {st.max_pending}")
        # every query answered, in time order
        assert np.all(n_out == w["k"]) and np.all(lat > 0) and done_s.max() <= st.wall_s
        assert st.items <= st.capacity and st.items == int(w["nprobe"].sum())
        k = w["k"]
        assert all(ids[i, :k[i]].min() >= 0 for i in range(0, n, 37))
        # the high class (cache lookups: one step each) does not wait behind the low class
        hi, lo = lat[~w["is_rag"]], lat[w["is_rag"]]
        _say(f"config 3 {scale}: mean latency cache {hi.mean() * 1e3:.2f} ms, RAG {lo.mean() * 1e3:.2f} ms")
        assert np.median(hi) <= np.median(lo)
        # parity on a sample of each kind
        rng = np.random.default_rng(33)
        for name, sel, idx, base in (("RAG", np.flatnonzero(w["is_rag"]), ir, rag_base),
                                     ("cache", np.flatnonzero(~w["is_rag"]), ic, cache_base)):
            sample = np.sort(rng.choice(sel, n_check // 2, replace=False))
            oidx = harness.oracle_index(tri, idx, base)
            pl = [probes[i, :w["nprobe"][i]] for i in range(n)]
            rep = harness.compare_with_oracle(oidx, base, queries, w["k"], w["nprobe"], 1, ids, dist, n_out, pl,
                                              sample=sample, batch_first=True)
            _say(f"config 3 {scale}: {name} parity {rep}")
            assert rep["checked"] == sample.size
            if name == "cache":
                # hit flag against the oracle's top-1 score
                flips = 0
                for i in sample:
                    top = float(oracle.search(oidx, queries[i], 1, int(w["nprobe"][i]), 1)[2][0])
                    if abs(top - 0.95) > 2e-3 * 0.95 + checker.ABS_EPS:
                        assert (dist[i, 0] >= 0.95) == (top >= 0.95)
                    else:
                        flips += 1
                hits = dist[~w["is_rag"], 0] >= 0.95
                dup = w["near_dup"][~w["is_rag"]]
                _say(f"config 3 {scale}: hit rate {hits.mean():.3f}, near-duplicates {dup.mean():.3f}, in band {flips}")
                assert hits[dup].mean() > 0.98 and hits[~dup].mean() < 0.02


@pytest.mark.timeout(900)
def test_config4_full_size_in_the_benchmark_configuration():
    """Configuration 4 at full size (10M x 768 fp16, nlist 16384, 4096 queries, nprobe 64, k 100) in
    the launch configuration the benchmark times (4096 slots, one step per batch, device-resident
    query vectors): a seeded sample of more than 512 queries is checked against the oracle (the oracle side in
    one multi-threaded call, the tie-aware checker for every query whose result is not exactly the oracle's),
    every query against the properties that hold at any size."""
    import torch
    tri = harness.lib()
    cfg = workloads.CONFIGS[4]
    _say("config 4: generate")
    base_t, queries_t, rows = workloads.make_config_f16(cfg, device="cuda")
    torch.cuda.synchronize()
    Q = cfg.n_queries
    pool = tri.Pool(slots=Q, items_per_step=Q * cfg.nprobe, lists_per_query_step=0, kmax=128, nprobe_max=cfg.nprobe,
                    max_indexes=1, max_total_lists=cfg.nlist, max_nlist=cfg.nlist, max_dim=cfg.dim,
                    max_outstanding=Q * 2, coarse_rows=0, flags=tri.TRI_FLAG_KEEP_PROBES, score_capacity=(1 << 27))
    try:
        _say("config 4: build")
        init = base_t[torch.from_numpy(rows).cuda()].float().cpu().numpy()
        idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, cfg.train_iters, centroids=init)
        _say(f"config 4: built, longest list {tri.ivf_info(idx)['max_list_len']}; search")
        tickets, rc = tri.search_submit_batch_dev(pool.handle, idx, queries_t.data_ptr(), cfg.dim * 2, Q, cfg.k,
                                                  cfg.nprobe, tri.TRI_IP)
        assert rc == tri.TRI_OK
        st = tri.search_step(pool.handle)
        assert st.admitted == Q and st.retired == Q and st.items == Q * cfg.nprobe     # one launch per batch
        tri.search_sync(pool.handle)
        probes = [tri.search_probes(pool.handle, int(tickets[i]), cfg.nprobe) for i in range(Q)]
        ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, cfg.k)
        assert np.all(status == tri.TRI_OK)
        # properties for every query
        assert np.all(n_out == cfg.k)
        assert ids.min() >= 0 and ids.max() < cfg.n_base
        assert np.all(np.diff(dist, axis=1) <= 0), "inner-product scores must be descending"
        srt = np.sort(ids, axis=1)
        assert np.all(srt[:, 1:] != srt[:, :-1]), "duplicate ids in a result"
        _say("config 4: copy the base to the host, export, compare the sample with the oracle")
        base = base_t.cpu().numpy()
        queries = queries_t.cpu().numpy()
        oidx = harness.oracle_index(tri, idx, base)
        rep = oindex.check_index(oidx, oracle.METRIC_IP, tol=2e-3, sample=512, seed=3)
        _say(f"config 4: index check {rep}")
        # the sample: 512 seeded queries, plus queries that probe the longest list and the shortest ones (among them
        # lists shorter than the 64-vector sample the thresholds are taken from, if the index has any)
        lens = np.diff(oidx.list_off).astype(np.int64)
        pm = np.stack(probes)
        extreme = np.r_[np.argsort(lens, kind="stable")[:8], np.argmax(lens)]
        extra = np.concatenate([np.flatnonzero((pm == l).any(axis=1))[:8] for l in extreme])
        sample = np.unique(np.r_[np.random.default_rng(44).choice(Q, 512, replace=False), extra])
        _say(f"config 4: list lengths {lens.min()}..{lens.max()}; {sample.size} queries against the oracle "
             f"({extra.size} of them probe a shortest or the longest list)")
        rep = harness.compare_with_oracle(oidx, base, queries, cfg.k, cfg.nprobe, 1, ids, dist, n_out, probes,
                                          sample=sample, batch_first=True)
        _say(f"config 4: parity {rep}")
        assert rep["checked"] == sample.size >= 512
        # returned scores of ALL queries against fp64 dot products of the stored vectors
        for i in range(0, Q, 97):
            want = base[ids[i]].astype(np.float64) @ queries[i].astype(np.float64)
            assert np.all(np.abs(dist[i] - want) <= 2e-3 * np.abs(want) + checker.ABS_EPS)
    finally:
        pool.close()


def test_massive_ties_take_the_exact_path():
    """Thousands of identical vectors: far more candidates tie at the k-th score than fit the sorted
    pool, so selection must fall back to the exact radix path and still order ties by id."""
    tri = harness.lib()
    rng = np.random.default_rng(21)
    protos = rng.integers(-3, 4, size=(3, 16)).astype(np.float32)
    base = protos[rng.integers(0, 3, size=30_000)]
    cent = np.stack([protos[0], protos[1], protos[2], protos[0] + 0.5]).astype(np.float32)
    queries = (protos[rng.integers(0, 3, size=12)] + 0.25).astype(np.float32)
    with harness.default_pool(tri, max_dim=16, kmax=1024, max_nlist=8, max_total_lists=8, score_capacity=1 << 20) as pool:
        idx = pool.build_index(base, 16, 4, tri.TRI_F32, tri.TRI_L2, 0, centroids=cent)
        oidx = harness.oracle_index(tri, idx, base)
        for k, nprobe, metric in [(100, 4, 0), (1024, 2, 0), (7, 4, 1), (1000, 4, 1)]:
            _say(f"ties: k={k} nprobe={nprobe} metric={metric}")
            q = tri.make_queries(idx, queries, k, nprobe, metric)
            ids, dist, n_out, probes, _ = harness.run_all(tri, pool, q)
            # integer-valued data + quarter offsets: every score is exact in fp32 -> strict comparison
            harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes, strict=True)


def test_every_path_of_the_coarse_selection():
    """The probe list of a new query is chosen by one wavefront when its one pass settles the row, and by the general
    workgroup selection when it does not; rows of the second kind are queued, with queue heads that alternate between
    the steps.  Two indexes in one pool (two coarse groups in every step): one with distinct centroids, one whose 640
    centroids are 5 prototypes repeated 128 times -- every score ties 128 times, far more equal keys than the
    wavefront's pool holds, so those rows are deferred and must come out with the tie rule (smaller centroid number
    first) intact.  Few slots, so that many consecutive steps admit queries of both kinds; nprobe from 1 to above the
    wavefront path's limit; probe lists and results against the oracle, strictly (integer-valued data)."""
    tri = harness.lib()
    rng = np.random.default_rng(55)
    dim = 16
    cent_a = rng.integers(-8, 9, size=(700, dim)).astype(np.float32)              # (700: the row ends inside a 128-byte line)
    protos = rng.integers(-8, 9, size=(5, dim)).astype(np.float32)
    cent_b = protos[np.arange(640) % 5]
    base_a = (cent_a[rng.integers(0, 700, size=20_000)] + rng.integers(-1, 2, size=(20_000, dim))).astype(np.float32)
    base_b = (cent_b[rng.integers(0, 640, size=12_000)] + rng.integers(-1, 2, size=(12_000, dim))).astype(np.float32)
    nq = 60
    qa = (cent_a[rng.integers(0, 700, size=nq)] + rng.integers(-1, 2, size=(nq, dim))).astype(np.float32)
    qb = (protos[rng.integers(0, 5, size=nq)] + rng.integers(-1, 2, size=(nq, dim))).astype(np.float32)
    k = np.full(nq, 10, dtype=np.uint32)
    nprobe = np.array([1, 7, 32, 64, 128, 129, 200], dtype=np.uint32)[np.arange(nq) % 7]
    metric = (np.arange(nq) // 3 % 2).astype(np.uint32)
    with harness.default_pool(tri, slots=6, items_per_step=6 * 256, kmax=16, nprobe_max=256, max_dim=dim, max_nlist=704,
                              max_total_lists=1344, max_indexes=2, score_capacity=8 << 20) as pool:
        ia = pool.build_index(base_a, dim, 700, tri.TRI_F32, tri.TRI_L2, 0, centroids=cent_a)
        ib = pool.build_index(base_b, dim, 640, tri.TRI_F32, tri.TRI_L2, 0, centroids=cent_b)
        oa, ob = harness.oracle_index(tri, ia, base_a), harness.oracle_index(tri, ib, base_b)
        q = []
        for i in range(nq):                                                       # (interleaved: both groups in every step)
            q.append(tri.make_queries(ia, qa[i:i + 1], k[i:i + 1], nprobe[i:i + 1], metric[i:i + 1]))
            q.append(tri.make_queries(ib, qb[i:i + 1], k[i:i + 1], nprobe[i:i + 1], metric[i:i + 1]))
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, np.concatenate(q))
        ra = harness.compare_with_oracle(oa, base_a, qa, k, nprobe, metric, ids[0::2], dist[0::2], n_out[0::2],
                                         [probes[i] for i in range(0, 2 * nq, 2)] if probes is not None else None, strict=True)
        rb = harness.compare_with_oracle(ob, base_b, qb, k, nprobe, metric, ids[1::2], dist[1::2], n_out[1::2],
                                         [probes[i] for i in range(1, 2 * nq, 2)] if probes is not None else None, strict=True)
        _say(f"coarse selection paths: {len(stats)} steps, distinct centroids {ra}, repeated centroids {rb}")
        assert len(stats) >= 15


def test_several_threads_submit_while_one_steps():
    """search_submit_batch is safe from several threads while one driver thread steps and polls: four
    submitters feed their shares in small chunks; every query is answered once and as the oracle says."""
    import threading
    import time
    tri = harness.lib()
    cfg = workloads.CONFIGS[0].scaled(n_base=20_000, n_components=64, nlist=96, n_queries=400)
    base, queries, rows = workloads.make_config01(cfg)
    k = np.random.default_rng(5).integers(1, 40, size=cfg.n_queries).astype(np.uint32)
    nprobe = np.random.default_rng(6).integers(1, 33, size=cfg.n_queries).astype(np.uint32)
    metric = (np.arange(cfg.n_queries) % 2).astype(np.uint32)
    klass = (np.arange(cfg.n_queries) % 3 == 0).astype(np.uint32)
    n_threads = 4
    with harness.default_pool(tri, max_dim=cfg.dim, slots=48, lists_per_query_step=4) as pool:
        idx = _build_f32(tri, pool, cfg, base, rows)
        q = tri.make_queries(idx, queries, k, nprobe, metric, klass)
        tickets = np.zeros(cfg.n_queries, dtype=np.uint64)
        errors = []

        def submitter(w):
            try:
                mine = np.arange(w, cfg.n_queries, n_threads)
                for c0 in range(0, mine.size, 7):
                    sel = mine[c0:c0 + 7]
                    t, rc = tri.search_submit_batch(pool.handle, np.ascontiguousarray(q[sel]))
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
            st = tri.search_step(pool.handle)
            steps += 1
            assert steps < 200000, "search_step loop did not drain"
            alive = any(th.is_alive() for th in threads)
            if not alive and st.running == 0 and st.pending_high == 0 and st.pending_low == 0 and st.items == 0:
                break
        for th in threads:
            th.join()
        assert not errors, errors
        tri.search_sync(pool.handle)
        assert len(set(tickets.tolist())) == cfg.n_queries, "a ticket was handed out twice"
        probes = [tri.search_probes(pool.handle, int(tickets[i]), int(nprobe[i])) for i in range(cfg.n_queries)]
        ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, int(k.max()))
        assert np.all(status == tri.TRI_OK)
        oidx = harness.oracle_index(tri, idx, base)
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
        _say(f"4 submitters, {steps} steps: {rep}")


@pytest.mark.parametrize("recorded", [False, True])
def test_indexes_come_and_go_in_a_living_pool(recorded):
    """Indexes are destroyed and built while the pool lives: finished, unpolled results of a destroyed index
    stay pollable; a new index of another row class takes the freed place (and, when it was the last one
    attached, its list range); the first index leaves a hole in the list table that later steps must skip.
    After every change the surviving and the new indexes answer as the oracle says -- also with recorded
    steps, which have to be recorded afresh whenever the set of attached indexes changes."""
    tri = harness.lib()
    cfg_a = workloads.CONFIGS[0].scaled(n_base=12_000, n_components=32, nlist=64, n_queries=50)
    cfg_b = workloads.CONFIGS[2].scaled(n_base=9_000, n_components=32, nlist=32, n_queries=50, dim=96)
    cfg_c = workloads.CONFIGS[0].scaled(n_base=7_000, n_components=16, nlist=48, n_queries=50, dim=200)
    cfg_d = workloads.CONFIGS[0].scaled(n_base=3_000, n_components=8, nlist=16, n_queries=50, dim=40)
    base_a, q_a, rows_a = workloads.make_config01(cfg_a)
    base_b_t, base_b, q_b, rows_b = _f16_setup(tri, cfg_b)
    base_c, q_c, rows_c = workloads.make_config01(cfg_c)
    base_d, q_d, rows_d = workloads.make_config01(cfg_d)
    flags = tri.TRI_FLAG_KEEP_PROBES | (tri.TRI_FLAG_GRAPH if recorded else 0)

    def check(pool, parts):
        """parts: list of (index handle, oracle index, base, queries, k, nprobe, metric); one mixed run."""
        qs = np.concatenate([tri.make_queries(ix, q, k, npb, m) for ix, _, _, q, k, npb, m in parts])
        order = np.random.default_rng(3).permutation(qs.shape[0])
        ids, dist, n_out, probes, _ = harness.run_all(tri, pool, np.ascontiguousarray(qs[order]), submit_chunks=[7, 40, 9])
        inv = np.argsort(order)
        ids, dist, n_out, probes = ids[inv], dist[inv], n_out[inv], [probes[i] for i in inv]
        at = 0
        for ix, oidx, base, q, k, npb, m in parts:
            n = q.shape[0]
            harness.compare_with_oracle(oidx, base, q, k, npb, m, ids[at:at + n], dist[at:at + n], n_out[at:at + n],
                                        probes[at:at + n])
            at += n

    with harness.default_pool(tri, slots=24, max_dim=256, max_outstanding=512, lists_per_query_step=3,
                              max_total_lists=160, max_nlist=64, flags=flags) as pool:
        ia = pool.build_index(base_a, cfg_a.dim, cfg_a.nlist, tri.TRI_F32, tri.TRI_L2, 4, centroids=base_a[rows_a])
        ib = pool.build_index(base_b_t, cfg_b.dim, cfg_b.nlist, tri.TRI_F16, tri.TRI_IP, 4,
                              centroids=base_b[rows_b].astype(np.float32))
        oa, ob = harness.oracle_index(tri, ia, base_a), harness.oracle_index(tri, ib, base_b)
        part_a = (ia, oa, base_a, q_a, 10, 12, tri.TRI_L2)
        _say("lifecycle: A + B")
        check(pool, [part_a, (ib, ob, base_b, q_b, 7, 9, tri.TRI_IP)])
        # results of B that nobody has polled yet outlive B
        qb = tri.make_queries(ib, q_b, 7, 9, tri.TRI_IP)
        tb, rc = tri.search_submit_batch(pool.handle, qb)
        assert rc == tri.TRI_OK
        for _ in range(1000):
            st = tri.search_step(pool.handle)
            if st.running == 0 and st.pending_high == 0 and st.pending_low == 0 and st.items == 0:
                break
        tri.search_sync(pool.handle)
        probes_b = [tri.search_probes(pool.handle, int(t), 9) for t in tb]
        pool.destroy_index(ib)
        ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tb, 7)
        assert np.all(status == tri.TRI_OK)
        harness.compare_with_oracle(ob, base_b, q_b, 7, 9, tri.TRI_IP, ids, dist, n_out, probes_b)
        # C (another row class) takes B's place and B's list range
        ic = pool.build_index(base_c, cfg_c.dim, cfg_c.nlist, tri.TRI_F32, tri.TRI_L2, 4, centroids=base_c[rows_c])
        oc = harness.oracle_index(tri, ic, base_c)
        part_c = (ic, oc, base_c, q_c, 5, 48, tri.TRI_IP)          # every list probed, the other metric
        _say("lifecycle: A + C")
        check(pool, [part_a, part_c])
        # A goes: its 64 lists stay a hole at the head of the table; D joins behind C
        pool.destroy_index(ia)
        idd = pool.build_index(base_d, cfg_d.dim, cfg_d.nlist, tri.TRI_F32, tri.TRI_L2, 4, centroids=base_d[rows_d])
        od = harness.oracle_index(tri, idd, base_d)
        _say("lifecycle: C + D")
        check(pool, [part_c, (idd, od, base_d, q_d, 12, 5, tri.TRI_L2)])
        # a query for an index that is gone is refused
        with pytest.raises(Exception):
            tri.search_submit_batch(pool.handle, tri.make_queries(ia, q_a[:1], 1, 1, 0))


def test_largest_k_and_nprobe():
    """The limits of the boundary together (TRI_KMAX_LIMIT, TRI_NPROBE_LIMIT): k = 1024 and nprobe = 1024 = nlist
    (every list probed: the result must be exact kNN by brute force), and neighbours of those limits, on many
    short lists."""
    tri = harness.lib()
    rng = np.random.default_rng(33)
    n, dim, nlist, nq = 40_000, 32, 1024, 24
    centres = rng.standard_normal((nlist, dim)).astype(np.float32) * 3
    base = (centres[rng.integers(0, nlist, size=n)] + rng.standard_normal((n, dim))).astype(np.float32)
    queries = (centres[rng.integers(0, nlist, size=nq)] + rng.standard_normal((nq, dim))).astype(np.float32)
    k = np.array([1024, 1000, 1], dtype=np.uint32)[np.arange(nq) % 3]
    nprobe = np.array([1024, 1024, 1023, 700], dtype=np.uint32)[np.arange(nq) % 4]
    metric = (np.arange(nq) // 2 % 2).astype(np.uint32)
    with harness.default_pool(tri, slots=8, items_per_step=8 * 1024, kmax=1024, nprobe_max=1024, max_dim=dim,
                              max_nlist=nlist, max_total_lists=nlist, score_capacity=64 << 20) as pool:
        idx = pool.build_index(base, dim, nlist, tri.TRI_F32, tri.TRI_L2, 3, centroids=centres)
        oidx = harness.oracle_index(tri, idx, base)
        q = tri.make_queries(idx, queries, k, nprobe, metric)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
        _say(f"largest k and nprobe: {len(stats)} steps, parity {rep}")
        for i in np.nonzero(nprobe == nlist)[0]:
            # (as sets, and up to a swap at the k-th place: fp32 and fp64 may order two near-equal scores differently)
            true_ids, _ = bruteforce.knn(base, queries[i:i + 1], int(k[i]), int(metric[i]))
            common = len(set(ids[i, :k[i]].tolist()) & set(true_ids[0].tolist()))
            assert common >= int(k[i]) - 1, f"query {i}: nprobe = nlist must be exact kNN ({common} of {k[i]})"


@pytest.mark.parametrize("lists_per_step", [0, 2])
def test_every_path_of_the_per_slot_selection_kernels(lists_per_step):
    """The threshold and merge kernels take a slot by one wavefront when it fits their registers and their one-pass
    cut settles it, and otherwise by slower routes.  Built to reach all of them, every result against the oracle:
    no threshold at all (fewer samples than k: every vector of the probed lists is a candidate, far more than the
    merge's registers hold, so it streams them pass by pass); running top-k across steps (with lists_per_step 2);
    k above 256 (the general workgroup selection, and a running top-k longer than the threshold kernel's registers);
    and samples with extreme outliers -- stored vectors of huge norm with the smallest ids, so that they head every
    list's sample -- which stretch the value range until the bucket of rank k holds nearly everything and the cut
    has to be refined."""
    tri = harness.lib()
    rng = np.random.default_rng(77)
    n, d, nlist = 24_000, 64, 12
    centres = rng.normal(0.0, 1.0, size=(nlist, d))
    base = (centres[rng.integers(0, nlist, n)] + rng.normal(0.0, 0.5, size=(n, d))).astype(np.float32)
    base[:nlist * 2] = (centres[np.arange(nlist * 2) % nlist] * 400.0).astype(np.float32)      # outliers, smallest ids
    cases = [(200, 2, 0), (200, 2, 1), (250, 6, 0), (100, 8, 1), (10, 8, 0), (300, 4, 1), (700, 6, 0), (1, 3, 1), (64, 12, 0)]
    nq = 6 * len(cases)
    queries = np.ascontiguousarray((centres[rng.integers(0, nlist, nq)] + rng.normal(0.0, 0.5, size=(nq, d))).astype(np.float32))
    k = np.array([cases[i % len(cases)][0] for i in range(nq)], dtype=np.uint32)
    nprobe = np.array([cases[i % len(cases)][1] for i in range(nq)], dtype=np.uint32)
    metric = np.array([cases[i % len(cases)][2] for i in range(nq)], dtype=np.uint32)
    with harness.default_pool(tri, slots=32, lists_per_query_step=lists_per_step, kmax=1024, max_dim=d, max_nlist=nlist,
                              max_total_lists=nlist, score_capacity=1 << 22) as pool:
        idx = pool.build_index(base, d, nlist, tri.TRI_F32, tri.TRI_L2, 0, centroids=centres.astype(np.float32))
        oidx = harness.oracle_index(tri, idx, base)
        q = tri.make_queries(idx, queries, k, nprobe, metric)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, metric, ids, dist, n_out, probes)
        _say(f"selection paths, {lists_per_step or 'all'} lists per step: {len(stats)} steps, parity {rep}, "
             f"rescans {tri.tri_pool_candidate_rescans(pool.handle)}")
        assert rep["checked"] == nq
