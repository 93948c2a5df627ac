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
    print(msg, flush=True)


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
