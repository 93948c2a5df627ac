"""Pins for the CPU oracle: each checks it against something that is not the oracle.

* hand-computed worked examples (tests/golden/worked_examples.json)
* exact kNN by brute force in numpy when nprobe == nlist (tiny random instances, both
  metrics, both storage types; and configuration 0 whole)
* probe sets against a numpy enumeration, with duplicated centroids to force ties
* integer-valued data against int64 arithmetic (exactness)
* the unit-norm identity |x-q|^2 = |x|^2 + |q|^2 - 2 x.q linking the two metrics
* output invariants (sorted, unique, members of probed lists, prefix property in k,
  monotone in nprobe)
* planted mistakes: mutated copies of the oracle's C source must FAIL these pins
"""
import ctypes
import json
import os
import subprocess
import tempfile

import numpy as np
import pytest

import oracle
from oracle import Index, METRIC_IP, METRIC_L2
from oracle import index as oindex
import workloads
from tests import bruteforce

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "worked_examples.json")


def _index_from_lists(base, centroids, lists):
    off = np.zeros(len(lists) + 1, dtype=np.uint64)
    off[1:] = np.cumsum([len(l) for l in lists])
    ids = np.array([i for l in lists for i in l], dtype=np.int64)
    return Index(base, np.asarray(centroids, dtype=np.float32), off, ids)


def _run_golden(dtype):
    """Evaluate every golden case; returns list of failure strings (empty = all pass)."""
    fails = []
    with open(GOLDEN) as f:
        data = json.load(f)
    for case in data["cases"]:
        base = np.asarray(case["base"], dtype=dtype)
        idx = _index_from_lists(base, case["centroids"], case["lists"])
        metric = METRIC_L2 if case["metric"] == "l2" else METRIC_IP
        for qi, qc in enumerate(case["queries"]):
            q = np.asarray(qc["q"], dtype=dtype)
            probe, ids, dist, n = oracle.search(idx, q, qc["k"], qc["nprobe"], metric)
            tag = f"{case['name']}[{qi}]"
            if list(probe) != qc["probe"]:
                fails.append(f"{tag}: probe {list(probe)} != {qc['probe']}")
            if n != len(qc["ids"]):
                fails.append(f"{tag}: n_out {n} != {len(qc['ids'])}")
                continue
            if list(ids[:n]) != qc["ids"]:
                fails.append(f"{tag}: ids {list(ids[:n])} != {qc['ids']}")
            if list(dist[:n]) != [float(v) for v in qc["dist"]]:
                fails.append(f"{tag}: dist {list(dist[:n])} != {qc['dist']}")
            if not np.all(ids[n:] == -1):
                fails.append(f"{tag}: tail ids not -1")
            pad = np.inf if metric == METRIC_L2 else -np.inf
            if not np.all(dist[n:] == pad):
                fails.append(f"{tag}: tail scores not {pad}")
    return fails


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_golden_worked_examples(dtype):
    assert _run_golden(dtype) == []


def test_half_conversion_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def _tiny_instance(rng, dtype, integer):
    n = int(rng.integers(1, 513))
    d = int(rng.integers(1, 9))
    nlist = int(rng.integers(1, min(8, n) + 1))
    if integer:
        base = rng.integers(-4, 5, size=(n, d)).astype(dtype)
        queries = rng.integers(-4, 5, size=(5, d)).astype(dtype)
    else:
        base = rng.standard_normal((n, d)).astype(dtype)
        queries = rng.standard_normal((5, d)).astype(dtype)
    cent = base[rng.choice(n, size=nlist, replace=False)].astype(np.float32)
    return base, queries, cent


def _brute_equals_oracle(metric, dtype, integer, seeds):
    fails = []
    for seed in seeds:
        rng = np.random.default_rng(seed)
        base, queries, cent = _tiny_instance(rng, dtype, integer)
        idx = oindex.build_index(base, cent, metric)
        k = int(rng.integers(1, 20))
        want_ids, want_sc = bruteforce.knn(base, queries, k, metric)
        for i, q in enumerate(queries):
            _, ids, dist, n = oracle.search(idx, q, k, idx.nlist, metric)
            kk = min(k, base.shape[0])
            if n != kk:
                fails.append(f"seed {seed} q{i}: n {n} != {kk}")
                continue
            if integer:
                # integer data: all scores exact, ties are true ties -> identical id lists
                if not np.array_equal(ids[:n], want_ids[i]):
                    fails.append(f"seed {seed} q{i}: ids differ")
                if not np.array_equal(dist[:n], want_sc[i]):
                    fails.append(f"seed {seed} q{i}: scores differ")
            else:
                if not np.allclose(dist[:n], want_sc[i], rtol=1e-9, atol=1e-9):
                    fails.append(f"seed {seed} q{i}: scores differ")
                # ids equal wherever neighbouring scores are separated
                sep = np.abs(np.diff(want_sc[i])) > 1e-9
                solid = np.r_[True, sep] & np.r_[sep, True]
                if not np.array_equal(ids[:n][solid], want_ids[i][solid]):
                    fails.append(f"seed {seed} q{i}: ids differ")
    return fails


@pytest.mark.parametrize("metric", [METRIC_L2, METRIC_IP])
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("integer", [True, False])
def test_full_probe_equals_bruteforce_knn_on_tiny_instances(metric, dtype, integer):
    assert _brute_equals_oracle(metric, dtype, integer, range(12)) == []


@pytest.mark.parametrize("metric", [METRIC_L2, METRIC_IP])
def test_probe_set_matches_numpy_enumeration_with_tied_centroids(metric):
    for seed in range(20):
        rng = np.random.default_rng(100 + seed)
        d = int(rng.integers(1, 6))
        nlist = int(rng.integers(2, 12))
        cent = rng.integers(-3, 4, size=(nlist, d)).astype(np.float32)
        dup = rng.integers(0, nlist, size=nlist // 2)
        cent[dup] = cent[rng.integers(0, nlist, size=dup.size)]  # duplicated centroids -> exact ties
        base = rng.integers(-3, 4, size=(nlist * 3, d)).astype(np.float32)
        idx = oindex.build_index(base, cent, metric)
        q = rng.integers(-3, 4, size=d).astype(np.float32)
        c64, q64 = cent.astype(np.float64), q.astype(np.float64)
        if metric == METRIC_L2:
            sc = ((c64 - q64) ** 2).sum(1)
            order = np.lexsort((np.arange(nlist), sc))
        else:
            sc = c64 @ q64
            order = np.lexsort((np.arange(nlist), -sc))
        got_sc = oracle.coarse_scores(idx, q, metric)
        assert np.array_equal(got_sc, sc)
        for nprobe in range(1, nlist + 1):
            assert list(oracle.probe_set(got_sc, nprobe, metric)) == list(order[:nprobe])


def test_integer_data_scores_equal_int64_arithmetic():
    """Byte-valued data at d=128: every score is an integer the oracle must hit exactly."""
    cfg = workloads.CONFIGS[1].scaled(n_base=4000, n_components=16, nlist=16, n_queries=8)
    base, queries, rows = workloads.make_config01(cfg)
    idx = oindex.build_index(base, base[rows], METRIC_L2)
    bi, qi = base.astype(np.int64), queries.astype(np.int64)
    for i, q in enumerate(queries):
        probe, ids, dist, n = oracle.search(idx, q, 10, 4, METRIC_L2)
        want = ((bi[ids[:n]] - qi[i]) ** 2).sum(axis=1)
        assert np.array_equal(dist[:n], want.astype(np.float64))
        # and the list is the exact top-k of the probed lists under integer arithmetic
        cand = np.concatenate([idx.list_ids[int(idx.list_off[l]):int(idx.list_off[l + 1])] for l in probe])
        all_d = ((bi[cand] - qi[i]) ** 2).sum(axis=1)
        order = np.lexsort((cand, all_d))[:10]
        assert np.array_equal(ids[:n], cand[order])


def test_unit_norm_identity_links_l2_and_ip():
    cfg = workloads.CONFIGS[2].scaled(n_base=3000, n_components=24, nlist=12, n_queries=6, dim=64)
    base_t, queries_t, rows = workloads.make_config_f16(cfg)
    base, queries = base_t.numpy(), queries_t.numpy()
    idx = oindex.build_index(base, base[rows].astype(np.float32), METRIC_IP)
    for q in queries:
        probe_ip, ids_ip, s_ip, n = oracle.search(idx, q, 20, idx.nlist, METRIC_IP)
        _, ids_l2, s_l2, n2 = oracle.search(idx, q, 20, idx.nlist, METRIC_L2)
        assert n == n2 == 20
        qn = (q.astype(np.float64) ** 2).sum()
        xn = (base[ids_ip].astype(np.float64) ** 2).sum(axis=1)
        # identity with the measured norms of the fp16-rounded vectors
        assert np.allclose(xn + qn - 2.0 * s_ip, [
            ((base[i].astype(np.float64) - q.astype(np.float64)) ** 2).sum() for i in ids_ip], atol=1e-12)
        # norms are 1 +- ~1e-3, so rankings agree except where scores are that close
        assert len(set(ids_ip[:10].tolist()) & set(ids_l2.tolist())) >= 9


@pytest.mark.parametrize("metric", [METRIC_L2, METRIC_IP])
def test_output_invariants(metric):
    cfg = workloads.CONFIGS[0].scaled(n_base=2000, n_components=16, nlist=16, n_queries=10, dim=16)
    base, queries, rows = workloads.make_config01(cfg)
    idx = oindex.build_index(base, base[rows], metric, train_iters=2)
    sign = 1.0 if metric == METRIC_L2 else -1.0
    for q in queries:
        prev_kth = None
        for nprobe in (1, 2, 4, 8, 16):
            probe, ids, dist, n = oracle.search(idx, q, 25, nprobe, metric)
            assert len(set(probe.tolist())) == nprobe
            assert n <= 25 and np.all(ids[:n] >= 0) and len(set(ids[:n].tolist())) == n
            assert np.all(np.diff(sign * dist[:n]) >= 0)
            members = set()
            for l in probe:
                members |= set(idx.list_ids[int(idx.list_off[l]):int(idx.list_off[l + 1])].tolist())
            assert set(ids[:n].tolist()) <= members
            # probe sets nest, so the k-th best score cannot get worse as nprobe grows
            if n == 25:
                kth = sign * dist[24]
                if prev_kth is not None:
                    assert kth <= prev_kth
                prev_kth = kth
            # prefix property: the answer for a smaller k is the head of the answer for k
            _, ids5, dist5, n5 = oracle.search(idx, q, 5, nprobe, metric)
            assert np.array_equal(ids5[:n5], ids[:min(n, 5)]) and np.array_equal(dist5[:n5], dist[:min(n, 5)])


def test_batch_equals_single_queries():
    cfg = workloads.CONFIGS[0].scaled(n_base=1500, n_components=8, nlist=8, n_queries=9, dim=12)
    base, queries, rows = workloads.make_config01(cfg)
    idx = oindex.build_index(base, base[rows], METRIC_L2)
    k = np.array([1, 3, 7, 2, 9, 4, 4, 1, 5], dtype=np.uint32)
    nprobe = np.array([1, 2, 8, 3, 4, 1, 8, 8, 2], dtype=np.uint32)
    metric = np.array([0, 1, 0, 1, 0, 1, 0, 1, 0], dtype=np.uint32)
    out = oracle.search_batch(idx, queries, k, nprobe, metric)
    for i, q in enumerate(queries):
        probe, ids, dist, n = oracle.search(idx, q, int(k[i]), int(nprobe[i]), int(metric[i]))
        assert out["n"][i] == n
        assert np.array_equal(out["probe"][i, :nprobe[i]], probe)
        assert np.array_equal(out["ids"][i, :k[i]], ids)
        assert np.array_equal(out["dist"][i, :k[i]], dist)
        assert np.all(out["ids"][i, k[i]:] == -1)


def test_config0_full_probe_is_exact_knn_and_recall_gate():
    """Configuration 0 whole: nprobe = nlist equals brute force; recall@10 at nprobe=8 >= 0.9."""
    cfg = workloads.CONFIGS[0]
    base, queries, rows = workloads.make_config01(cfg)
    idx = oindex.build_index(base, base[rows], METRIC_L2, train_iters=cfg.train_iters)
    rep = oindex.check_index(idx, METRIC_L2, tol=0.0)
    assert rep["checked"] == cfg.n_base and rep["near_tie"] == 0
    true_ids, true_sc = bruteforce.knn(base, queries, cfg.k, METRIC_L2)
    full = oracle.search_batch(idx, queries, cfg.k, cfg.nlist, METRIC_L2)
    assert np.array_equal(full["ids"], true_ids)
    assert np.allclose(full["dist"], true_sc, rtol=1e-9)
    ivf = oracle.search_batch(idx, queries, cfg.k, cfg.nprobe, METRIC_L2)
    assert bruteforce.recall_at_k(ivf["ids"], true_ids) >= 0.9


# ----------------------------------------------------------------------------- planted mistakes
MUTATIONS = [
    ("sign of the difference", "double t = q[i] - x[i];", "double t = q[i] + x[i];"),
    ("L2 not squared", "s += t * t;", "s += t < 0 ? -t : t;"),
    ("dropped last term", "for (uint32_t i = 0; i < d; ++i)\n            s += q[i] * x[i];",
     "for (uint32_t i = 0; i + 1 < d || i == 0; ++i)\n            s += q[i] * x[i];"),
    ("IP ranked ascending", "if (a->score > b->score) return -1;\n    if (a->score < b->score) return 1;",
     "if (a->score < b->score) return -1;\n    if (a->score > b->score) return 1;"),
    ("tie-break to larger id", "return (a->id > b->id) - (a->id < b->id);\n}\n\nstatic int cmp_ip",
     "return (a->id < b->id) - (a->id > b->id);\n}\n\nstatic int cmp_ip"),
    ("scan skips last vector of a list", "for (uint64_t p = list_off[l]; p < list_off[l + 1]; ++p) {",
     "for (uint64_t p = list_off[l]; p + 1 < list_off[l + 1]; ++p) {"),
    ("probe one list too few", "for (uint32_t r = 0; r < nprobe; ++r) {\n        uint32_t l = probe[r];",
     "for (uint32_t r = 0; r + 1 < nprobe || r == 0; ++r) {\n        uint32_t l = probe[r];"),
    ("half exponent bias off by one", "ldexp((double)(f + 1024), e - 25)", "ldexp((double)(f + 1024), e - 24)"),
    ("coarse uses wrong centroid stride", "(double)centroids[(size_t)j * d + i]", "(double)centroids[(size_t)i * nlist + j]"),
]


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, monkeypatch):
    """A plausible mistake planted in a copy of the oracle's source must fail the pins."""
    src = open(os.path.join(os.path.dirname(oracle.__file__), "ivf_oracle.c")).read()
    assert src.count(old) >= 1, "mutation anchor not found"
    mutated = src.replace(old, new, 1)
    with tempfile.TemporaryDirectory() as tmp:
        c_path, so_path = os.path.join(tmp, "m.c"), os.path.join(tmp, "m.so")
        open(c_path, "w").write(mutated)
        subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", so_path, c_path, "-lm"])
        monkeypatch.setattr(oracle, "_lib", oracle._bind(so_path))
        fails = []
        try:
            fails += _run_golden(np.float32) + _run_golden(np.float16)
            for metric in (METRIC_L2, METRIC_IP):
                fails += _brute_equals_oracle(metric, np.float32, True, range(4))
                fails += _brute_equals_oracle(metric, np.float16, False, range(4))
        except (AssertionError, RuntimeError) as e:   # a mutated oracle may also error out
            fails.append(str(e))
        assert fails, f"planted mistake '{name}' went unnoticed"


# ------------------------------------------------------------------------------------------------
# Control loop of Sec. 3.3 (oracle/control.py).  The paper prints no numbers for it; what it fixes are
# directions, and those are the pins: none of them re-types the rule.
def _ctl_cfg(**over):
    from oracle import control
    base = dict(r_min=0.1, r_max=0.8, r_step=0.05, tau_factor=2.0, tau_min_s=1e-4, tau_max_s=8e-3,
                u_kv_target=0.9, u_kv_band=0.05, stall_target=0.1, wait_p95_budget_s=2e-3)
    base.update(over)
    return control.Config(**base)


def test_control_loop_follows_the_papers_directions():
    from oracle import control
    cfg = _ctl_cfg()
    rng = np.random.default_rng(11)
    nan = float("nan")
    for _ in range(2000):
        r = float(rng.uniform(0.0, 1.0))
        tau = float(rng.uniform(0.0, 1e-2))
        u = float(rng.uniform(0, 1)) if rng.random() < 0.8 else nan
        st = float(rng.uniform(0, 1)) if rng.random() < 0.8 else nan
        stp = float(rng.uniform(0, 1)) if rng.random() < 0.8 else nan
        w = float(rng.uniform(0, 6e-3)) if rng.random() < 0.8 else nan
        r0 = min(max(r, cfg.r_min), cfg.r_max)
        t0 = min(max(tau, cfg.tau_min_s), cfg.tau_max_s)
        r1, t1, _ = control.period(cfg, r, tau, u, st, stp, w)
        # bounds, always
        assert cfg.r_min - 1e-6 <= r1 <= cfg.r_max + 1e-6 and cfg.tau_min_s <= t1 <= cfg.tau_max_s
        # one period moves r by at most one step and tau by at most two factors
        assert abs(r1 - r0) <= cfg.r_step + 1e-6 and t0 / cfg.tau_factor ** 2 - 1e-12 <= t1 <= t0 * cfg.tau_factor + 1e-12
        if u == u and u < cfg.u_kv_target - cfg.u_kv_band - 1e-6:
            # link under-used: prefill is accelerated -- r never falls, tau_pre never grows, and one of them moves
            # unless both are at their limits; decode stalls cannot take share away in the same period
            assert r1 >= r0 - 1e-7 and t1 <= t0 + 1e-15
            assert r1 > r0 or t1 < t0 or (r0 >= cfg.r_max - 1e-6 and t0 <= cfg.tau_min_s)
        elif st == st and stp == stp and st > cfg.stall_target + 1e-6 and st > stp + 1e-6 and u == u \
                and u > cfg.u_kv_target - cfg.u_kv_band + 1e-6:
            # link fine, decode stalls rising: r falls (until r_min)
            assert r1 < r0 or r0 <= cfg.r_min + 1e-6
        if w == w and w > cfg.wait_p95_budget_s:
            assert t1 < t0 or t0 <= cfg.tau_min_s                  # waits over budget: tau_pre is shortened


def test_control_loop_fixed_point_and_relaxation():
    from oracle import control
    cfg = _ctl_cfg()
    # everything on target, waits well inside the budget: r stays, tau_pre relaxes to its upper bound and stays
    r, tau = 0.4, 1e-3
    for _ in range(10):
        r, tau, rules = control.period(cfg, r, tau, 0.95, 0.05, 0.05, 0.5e-3)
        assert rules == {4}
    assert abs(r - 0.4) < 1e-6 and tau == cfg.tau_max_s
    # waits between half the budget and the budget: nothing moves at all
    r2, tau2, rules = control.period(cfg, 0.4, 1e-3, 0.95, 0.05, 0.05, 1.5e-3)
    assert (abs(r2 - 0.4) < 1e-6, tau2, rules) == (True, 1e-3, set())
    # a stall level above target that is NOT rising does not move r (the paper speaks of rising stalls)
    r3, _, rules = control.period(cfg, 0.4, 1e-3, 0.95, 0.3, 0.3, 1.5e-3)
    assert abs(r3 - 0.4) < 1e-6 and 3 not in rules


def test_control_loop_settles_against_a_toy_plant():
    """Closed loop: a plant in which the KV link fills with the prefill share (u_kv = r / 0.5, capped) and
    decode stalls grow once prefill takes more than 0.6 of a batch.  From either end r moves into the
    window where the link is at target and stalls are not rising, and stays there."""
    from oracle import control
    cfg = _ctl_cfg()
    for r_start in (cfg.r_min, cfg.r_max):
        r, tau, stall_prev = r_start, 4e-3, 0.0
        trace = []
        for _ in range(60):
            u = min(1.0, r / 0.5)
            stall = max(0.0, (r - 0.6)) * 2.0 + 0.05 + (0.01 if r > 0.6 else 0.0) * len(trace)   # keeps rising while r > 0.6
            r, tau, _ = control.period(cfg, r, tau, u, stall, stall_prev, 1e-3)
            stall_prev = stall
            trace.append(r)
        tail = trace[-20:]
        assert max(tail) - min(tail) < 1e-6, f"r still moving: {tail}"
        assert 0.5 * (cfg.u_kv_target - cfg.u_kv_band) - 1e-6 <= tail[-1] <= 0.6 + 1e-6, tail[-1]
