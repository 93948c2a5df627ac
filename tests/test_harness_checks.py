"""The comparison helpers of the GPU parity tests, exercised on the CPU: a result that IS the oracle's
is settled by the batch path, anything else reaches the tie-aware checker, which accepts reordered
ties and refuses a missing neighbour, a foreign id and a score that is off."""
import numpy as np
import pytest

import oracle
from oracle import index as oindex
import workloads
from tests import harness


def _case():
    cfg = workloads.CONFIGS[0].scaled(n_base=3000, n_components=16, nlist=16, n_queries=24, dim=24)
    base, queries, rows = workloads.make_config01(cfg)
    idx = oindex.build_index(base, base[rows], oracle.METRIC_L2, train_iters=2)
    k = np.full(cfg.n_queries, 7, dtype=np.uint32)
    nprobe = np.full(cfg.n_queries, 3, dtype=np.uint32)
    out = oracle.search_batch(idx, queries, k, nprobe, 0)
    probes = [out["probe"][i, :3].copy() for i in range(cfg.n_queries)]
    return idx, base, queries, k, nprobe, out["ids"].copy(), out["dist"].astype(np.float32), out["n"].copy(), probes


def test_the_oracles_own_result_is_settled_by_the_batch_path():
    idx, base, queries, k, nprobe, ids, dist, n_out, probes = _case()
    rep = harness.compare_with_oracle(idx, base, queries, k, nprobe, 0, ids, dist, n_out, probes, batch_first=True)
    assert rep["checked"] == rep["settled_by_batch"] == queries.shape[0]
    sample = np.array([1, 5, 9])
    rep = harness.compare_with_oracle(idx, base, queries, k, nprobe, 0, ids, dist, n_out, probes, sample=sample, batch_first=True)
    assert rep["checked"] == 3


def test_a_probe_list_in_another_order_is_still_the_same_candidate_set():
    idx, base, queries, k, nprobe, ids, dist, n_out, probes = _case()
    probes[4] = probes[4][::-1].copy()
    rep = harness.compare_with_oracle(idx, base, queries, k, nprobe, 0, ids, dist, n_out, probes, batch_first=True)
    assert rep["checked"] == queries.shape[0]


@pytest.mark.parametrize("fault", ["missing neighbour", "foreign id", "score off", "short result", "wrong probe list"])
def test_a_faulty_result_is_not_settled_and_the_checker_refuses_it(fault):
    idx, base, queries, k, nprobe, ids, dist, n_out, probes = _case()
    i = 6
    if fault == "missing neighbour":           # best neighbour replaced by the first candidate beyond rank k
        _, _, _, cand_ids, cand_sc = oracle.scan(idx, queries[i], probes[i], 7, 0, all_candidates=True)
        assert cand_sc[20] > cand_sc[6] * 1.01
        ids[i, :7] = np.r_[cand_ids[1:7], cand_ids[20]]
        dist[i, :7] = np.r_[cand_sc[1:7], cand_sc[20]].astype(np.float32)
    elif fault == "foreign id":                # a row of a list that was not probed
        others = np.setdiff1d(np.arange(idx.nlist), probes[i])
        ids[i, 3] = idx.list_ids[int(idx.list_off[others[0]])]
    elif fault == "score off":
        dist[i, 2] *= np.float32(1.001)
    elif fault == "short result":
        n_out[i] = 6
        ids[i, 6] = -1
        dist[i, 6] = np.inf
    else:                                      # a list that is far from the boundary of the coarse ranking
        coarse = oracle.coarse_scores(idx, queries[i], 0)
        probes[i] = probes[i].copy()
        probes[i][2] = int(np.argmax(coarse))
    with pytest.raises(AssertionError):
        harness.compare_with_oracle(idx, base, queries, k, nprobe, 0, ids, dist, n_out, probes, batch_first=True)


def test_reordered_exact_ties_pass_through_the_checker():
    """Integer-valued data: rows at the same distance may come back in either order."""
    rng = np.random.default_rng(2)
    base = rng.integers(0, 3, size=(400, 4)).astype(np.float32)
    cent = base[:4].copy()
    idx = oindex.build_index(base, cent, oracle.METRIC_L2)
    queries = rng.integers(0, 3, size=(6, 4)).astype(np.float32)
    k = np.full(6, 9, dtype=np.uint32)
    nprobe = np.full(6, 4, dtype=np.uint32)
    out = oracle.search_batch(idx, queries, k, nprobe, 0)
    ids, dist = out["ids"].copy(), out["dist"].astype(np.float32)
    swapped = 0
    for i in range(6):
        for j in range(8):
            if dist[i, j] == dist[i, j + 1]:
                ids[i, [j, j + 1]] = ids[i, [j + 1, j]]
                swapped += 1
                break
    assert swapped
    probes = [out["probe"][i, :4].copy() for i in range(6)]
    rep = harness.compare_with_oracle(idx, base, queries, k, nprobe, 0, ids, dist, out["n"], probes, batch_first=True)
    assert rep["checked"] == 6 and rep["settled_by_batch"] < 6 and rep["tie_positions"] >= 2
