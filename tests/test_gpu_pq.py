"""GPU parity of IVF search over product-quantised lists (include/trinity_pq.h) against oracle/pq.py, through the C ABI."""
import ctypes

import numpy as np
import pytest

import oracle
from oracle import pq as opq
from tests import checker, harness

pytestmark = pytest.mark.gpu


def _say(msg):
    harness.say(msg)


def _setup(tri, dtype, n, d, nlist, seed, integer=False):
    import torch
    rng = np.random.default_rng(seed)
    np_dtype = np.float32 if dtype == "f32" else np.float16
    centres = rng.normal(0.0, 1.0, size=(nlist, d))
    base = centres[rng.integers(0, nlist, n)] + rng.normal(0.0, 0.4, size=(n, d))
    if integer:
        base = np.round(base * 4.0)
    base = base.astype(np_dtype)
    init = base[rng.choice(n, nlist, replace=False)].astype(np.float32)
    pool = harness.default_pool(tri, slots=16, max_dim=d, max_nlist=nlist, max_total_lists=nlist)
    idx = pool.build_index(base, d, nlist, tri.TRI_F32 if dtype == "f32" else tri.TRI_F16, tri.TRI_L2, 3, centroids=init)
    oidx = harness.oracle_index(tri, idx, base)
    return rng, base, pool, idx, oidx, torch


def _to_host(ids, dist, n_out, probes):
    ids = ids.cpu().numpy().view(np.uint32).astype(np.int64)
    ids[ids == 0xFFFFFFFF] = -1
    return ids, dist.cpu().numpy(), n_out.cpu().numpy().astype(np.int64), probes.cpu().numpy().view(np.uint32)


def _compare(oidx, codes_lm, cb, queries, k, nprobe, metric, ids, dist, n_out, probes, tol, strict=False):
    """Every query through the tie-aware checker, with the oracle's scores of ALL candidates of the probed lists."""
    n, d = oidx.n, oidx.d
    xhat = np.empty((n, d), dtype=np.float64)
    xhat[oidx.list_ids] = opq.decode(codes_lm, cb)
    report = dict(checked=0, coarse_near_tie=0, tie_positions=0)
    for i in range(queries.shape[0]):
        q = queries[i]
        coarse = oracle.coarse_scores(oidx, q, metric)
        want_probe = oracle.probe_set(coarse, nprobe, metric)
        got_probe = probes[i]
        assert len(set(got_probe.tolist())) == nprobe
        use = want_probe
        if set(got_probe.tolist()) != set(want_probe.tolist()):
            qn2 = float((q.astype(np.float64) ** 2).sum())
            cn2 = float((oidx.centroids.astype(np.float64) ** 2).sum(axis=1).max())
            eps = checker.ABS_EPS * (qn2 + cn2 if metric == 0 else np.sqrt(qn2 * cn2))
            assert checker.probe_sets_equivalent(got_probe, want_probe, coarse, metric, checker.tolerance_for(oidx.dtype), eps), \
                f"query {i}: probe set differs beyond a boundary near-tie"
            report["coarse_near_tie"] += 1
            use = got_probe
        _, _, _, _, cand_ids, cand_sc = opq.search(oidx, codes_lm, cb, q, k, nprobe, metric, probe=use, all_candidates=True)
        report["tie_positions"] += checker.check_result(q, xhat, metric, k, ids[i, :k], dist[i, :k], int(n_out[i]), cand_ids, cand_sc,
                                                        0.0 if strict else tol, strict=strict)
        report["checked"] += 1
    return report


@pytest.mark.parametrize("dtype,d,m", [("f16", 768, 96), ("f32", 128, 16), ("f16", 320, 20)])
def test_codebooks_codes_and_search_against_the_oracle(dtype, d, m):
    """Trained codebooks are exported and handed to the oracle; the library's codes must be the oracle's (nearest
    entry, ties to the smaller number; a code may differ only where two entries are equally near to rounding), the
    training must not be worse than the oracle's Lloyd from the same start, and the search results must pass the
    tie-aware checker with the oracle's scores of every candidate."""
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    n, nlist = 16_000, 24
    rng, base, pool, idx, oidx, torch = _setup(tri, dtype, n, d, nlist, seed=500 + d)
    with pool:
        X_lm = base[oidx.list_ids].astype(np.float64)
        with tpq.PQ(pool, idx, m, train_iters=0, seed=3) as start:
            cb0, _ = start.export(n, d)
        with tpq.PQ(pool, idx, m, train_iters=6, train_rows=4000, seed=3) as pq:
            cb, codes = pq.export(n, d)
            assert np.all(np.isfinite(cb))
            # codes: the oracle's, except where the runner-up is as near to rounding
            want = opq.encode(X_lm, cb)
            diff = np.argwhere(want != codes)
            w = d // m
            for r, mm in diff[:2000]:
                sub = X_lm[r, mm * w:(mm + 1) * w]
                d_got = ((sub - cb[mm, codes[r, mm]]) ** 2).sum()
                d_best = ((sub - cb[mm, want[r, mm]]) ** 2).sum()
                assert d_got <= d_best * (1 + 1e-5) + 1e-9, f"row {r} sub-space {mm}: code {codes[r, mm]} is not a nearest entry"
            # training: the sample is every n/4000-th stored vector; fp64 Lloyd from the same start
            sample = X_lm[::n // 4000][:4000]
            cb_oracle = opq.train(sample, cb0, 6)
            err_gpu = opq.quantisation_error(X_lm, codes, cb)
            err_oracle = opq.quantisation_error(X_lm, opq.encode(X_lm, cb_oracle), cb_oracle)
            err_start = opq.quantisation_error(X_lm, opq.encode(X_lm, cb0), cb0)
            _say(f"pq {dtype} d={d} m={m}: {diff.shape[0]} of {n * m} codes differ from the oracle's (near-ties); quantisation error "
                 f"start {err_start:.4f} -> gpu {err_gpu:.4f}, oracle's Lloyd {err_oracle:.4f}")
            assert diff.shape[0] <= n * m * 1e-3
            assert err_gpu < err_start and err_gpu <= err_oracle * 1.02
            # search
            nq = 40
            queries = np.ascontiguousarray((base[rng.choice(n, nq)].astype(np.float64) + rng.normal(0, 0.3, size=(nq, d))).astype(base.dtype))
            qt = torch.from_numpy(queries).cuda()
            tol = 2e-4
            for k, nprobe, metric in [(10, 4, 0), (100, 8, 1), (1, 1, 0), (256, nlist, 1)]:
                ids, dist, n_out, probes = _to_host(*pq.search(qt, k, nprobe, metric))
                pq.sync()
                ids, dist, n_out, probes = _to_host(*pq.search(qt, k, nprobe, metric))    # (a second call reuses nothing stale)
                pq.sync()
                rep = _compare(oidx, codes, cb, queries, k, nprobe, metric, ids, dist, n_out, probes, tol)
                _say(f"pq {dtype} d={d}: k={k} nprobe={nprobe} metric={metric} parity {rep}")
                assert rep["checked"] == nq


def test_lossless_codebooks_reproduce_the_flat_search_bit_for_bit():
    """Integer-valued vectors assembled from integer codebook entries are their own reconstructions and every sum is
    exact in fp32: the codes must be exactly the oracle's, and ids, order and scores exactly the IVF-Flat oracle's."""
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    import torch
    rng = np.random.default_rng(41)
    m, w, n, nlist = 8, 4, 6000, 10
    d = m * w
    cb = np.zeros((m, 256, w), dtype=np.float32)
    cb[:, :, :] = rng.integers(-6, 7, size=(m, 256, w))
    src = rng.integers(0, 256, size=(n, m))
    base = np.concatenate([cb[mm][src[:, mm]] for mm in range(m)], axis=1).astype(np.float32)
    init = base[rng.choice(n, nlist, replace=False)]
    with harness.default_pool(tri, slots=16, max_dim=d, max_nlist=nlist, max_total_lists=nlist) as pool:
        idx = pool.build_index(base, d, nlist, tri.TRI_F32, tri.TRI_L2, 2, centroids=init)
        oidx = harness.oracle_index(tri, idx, base)
        with tpq.PQ(pool, idx, m, codebooks=cb) as pq:
            cb_back, codes = pq.export(n, d)
            assert np.array_equal(cb_back, cb)
            assert np.array_equal(codes, opq.encode(base[oidx.list_ids], cb))
            assert np.array_equal(opq.decode(codes, cb), base[oidx.list_ids].astype(np.float64))
            queries = rng.integers(-6, 7, size=(30, d)).astype(np.float32)
            qt = torch.from_numpy(queries).cuda()
            for k, nprobe, metric in [(10, 3, 0), (50, 10, 1)]:
                ids, dist, n_out, probes = _to_host(*pq.search(qt, k, nprobe, metric))
                pq.sync()
                for i in range(queries.shape[0]):
                    fp, fids, fdist, fn = oracle.search(oidx, queries[i], k, nprobe, metric)
                    assert np.array_equal(probes[i], fp) and n_out[i] == fn
                    assert np.array_equal(ids[i, :k], fids), f"query {i}"
                    assert np.array_equal(dist[i, :fn].astype(np.float64), fdist[:fn])


def test_edge_cases_and_argument_errors():
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    n, d, nlist, m = 3000, 64, 40, 16
    rng, base, pool, idx, oidx, torch = _setup(tri, "f32", n, d, nlist, seed=9)
    with pool:
        for bad_m in (0, 6, 24, 128):                       # not a multiple of 4, not a divisor of 64, sub-space wider than allowed ...
            with pytest.raises(tri.TriError) as ei:
                tpq.PQ(pool, idx, bad_m)
            assert ei.value.status == tri.TRI_EINVAL
        with tpq.PQ(pool, idx, m, train_iters=3) as pq:
            cb, codes = pq.export(n, d)
            queries = np.ascontiguousarray(base[rng.choice(n, 12)])
            # rows with a pitch wider than a query, and what lies between them must never be read as data
            wide = torch.full((12, d + 24), 1e9, dtype=torch.float32, device="cuda")
            wide[:, :d] = torch.from_numpy(queries).cuda()
            # k beyond what one short list holds: n_out < k, padded tails
            ids, dist, n_out, probes = _to_host(*pq.search(wide[:, :d], 256, 1, 0))
            pq.sync()
            rep = _compare(oidx, codes, cb, queries, 256, 1, 0, ids, dist, n_out, probes, 2e-4)
            assert rep["checked"] == 12 and np.any(n_out < 256)
            ids, dist, n_out, probes = _to_host(*pq.search(wide[:, :d], 5, nlist, 1))           # every list probed
            pq.sync()
            _compare(oidx, codes, cb, queries, 5, nlist, 1, ids, dist, n_out, probes, 2e-4)
            qt = torch.from_numpy(queries).cuda()
            for k, nprobe, metric in [(0, 1, 0), (257, 1, 0), (5, 0, 0), (5, nlist + 1, 0), (5, 1, 2)]:
                with pytest.raises(tri.TriError) as ei:
                    pq.search(qt, k, nprobe, metric)
                assert ei.value.status == tri.TRI_EINVAL
            ws_t, ws_bytes = pq.workspace(12)
            with pytest.raises(tri.TriError) as ei:
                pq.search(qt, 5, 2, 0, ws=(ws_t, ws_bytes - 256))
            assert ei.value.status == tri.TRI_ENOMEM


@pytest.mark.parametrize("dtype,d,m,refine", [("f16", 768, 96, False), ("f32", 128, 16, False), ("f16", 768, 96, True), ("f32", 128, 16, True)])
def test_reranked_search_against_the_two_stage_oracle(dtype, d, m, refine):
    """k_adc > 0: the short list chosen by table sums is re-ranked by exact scores against the stored rows.  Where
    the short list ends, table sums within rounding of each other may be cut either way, so the check is the
    tie-aware one of both stages: every returned id belongs to a short list the oracle allows (its table score is not
    worse than the oracle's k_adc-th beyond the tolerance), carries its exact score, the order is by exact score, and
    no candidate that is surely in the short list and surely better than the returned k-th is missing.
    refine: the tri_pq re-ranks from its own row-major copy of the vectors (pq_params.refine_rows); beside the oracle
    check, its answers must be bit for bit those of a tri_pq with the same codebooks that reads the index's blocks."""
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    n, nlist = 16_000, 24
    rng, base, pool, idx, oidx, torch = _setup(tri, dtype, n, d, nlist, seed=700 + d)
    tol = checker.tolerance_for(oidx.dtype)
    with pool, tpq.PQ(pool, idx, m, train_iters=4, train_rows=4000, seed=5, refine_rows=refine) as pq:
        cb, codes = pq.export(n, d)
        nq = 32
        queries = np.ascontiguousarray((base[rng.choice(n, nq)].astype(np.float64) + rng.normal(0, 0.3, size=(nq, d))).astype(base.dtype))
        qt = torch.from_numpy(queries).cuda()
        for k, k_adc, nprobe, metric in [(10, 100, 6, 0), (10, 256, 8, 1), (5, 5, 3, 1), (64, 200, nlist, 0)]:
            ids, dist, n_out, probes = _to_host(*pq.search(qt, k, nprobe, metric, k_adc=k_adc))
            pq.sync()
            if refine:
                with tpq.PQ(pool, idx, m, codebooks=cb) as plain:
                    ids2, dist2, n_out2, probes2 = _to_host(*plain.search(qt, k, nprobe, metric, k_adc=k_adc))
                    plain.sync()
                assert np.array_equal(ids, ids2) and np.array_equal(n_out, n_out2) and np.array_equal(probes, probes2)
                assert np.array_equal(dist.view(np.uint32), dist2.view(np.uint32))
            changed = 0
            for i in range(nq):
                q = queries[i]
                coarse = oracle.coarse_scores(oidx, q, metric)
                want_probe = oracle.probe_set(coarse, nprobe, metric)
                use = want_probe if set(probes[i].tolist()) == set(want_probe.tolist()) else probes[i]
                _, oids, odist, on, cand_ids, cand_sc = opq.search_reranked(oidx, codes, cb, q, k, k_adc, nprobe, metric, probe=use)
                sign = 1.0 if metric == 0 else -1.0
                assert n_out[i] == on
                got = ids[i, :on]
                assert len(set(got.tolist())) == on
                # stage 1: what may be, and what must be, in the short list
                if cand_ids.shape[0] > k_adc:
                    tau1 = float(cand_sc[k_adc - 1])
                    qn = float(np.sqrt((q.astype(np.float64) ** 2).sum()))
                    band1 = 2e-4 * abs(tau1) + checker.ABS_EPS * qn * qn * 4
                    allowed = set(cand_ids[sign * (cand_sc - tau1) <= band1].tolist())
                    surely = cand_ids[sign * (tau1 - cand_sc) > band1]
                else:
                    allowed, surely = set(cand_ids.tolist()), cand_ids
                assert set(got.tolist()) <= allowed, f"query {i}: an id outside every admissible short list"
                # stage 2: exact scores, order, completeness
                x = base[got].astype(np.float64)
                exact = ((x - q.astype(np.float64)) ** 2).sum(axis=1) if metric == 0 else (x * q.astype(np.float64)).sum(axis=1)
                scale = np.sqrt((q.astype(np.float64) ** 2).sum() * (x ** 2).sum(axis=1))
                assert np.all(np.abs(dist[i, :on] - exact) <= checker.score_allowance(metric, tol, exact, scale)), f"query {i}: score is not the exact one"
                assert np.all(sign * np.diff(dist[i, :on].astype(np.float64)) >= 0)
                if on == k and surely.shape[0]:
                    xs = base[surely].astype(np.float64)
                    es = ((xs - q.astype(np.float64)) ** 2).sum(axis=1) if metric == 0 else (xs * q.astype(np.float64)).sum(axis=1)
                    kth = float(exact[-1])
                    band2 = tol * abs(kth) + checker.ABS_EPS * float(scale.max())
                    must = set(surely[sign * (kth - es) > band2].tolist())
                    assert must <= set(got.tolist()), f"query {i}: a surely better candidate is missing"
                changed += int(not np.array_equal(got, oids[:on]))
            _say(f"pq reranked {dtype} d={d}: k={k} k_adc={k_adc} nprobe={nprobe} metric={metric}: {nq - changed} of {nq} queries exactly the oracle's ids")
            assert changed <= nq // 4


def test_probe_lists_from_both_selection_kernels():
    """The probe lists of a batch are chosen by one wavefront per query when the row of centroid scores is short
    enough and one pass settles it, and by the workgroup selection otherwise (longer rows, nprobe above the wavefront
    kernel's limit, rows it gives up on).  Integer-valued data, so every score is exact and the lists must be the
    oracle's, in its order: 700 and 3000 distinct centroids (rows that end inside a load, rows of several loads), and
    640 centroids that are 5 prototypes repeated 128 times -- every score ties 128 times, more equal keys than the
    wavefront's pool holds once two prototypes are wanted, so those rows are handed over and must come out with the
    tie rule (smaller centroid number first) intact."""
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    import torch
    rng = np.random.default_rng(77)
    dim, nq = 16, 48
    protos = rng.integers(-8, 9, size=(5, dim)).astype(np.float32)
    for name, cent in [("700 distinct", rng.integers(-8, 9, size=(700, dim)).astype(np.float32)),
                       ("3000 distinct", rng.integers(-12, 13, size=(3000, dim)).astype(np.float32)),
                       ("5 prototypes x 128", protos[np.arange(640) % 5])]:
        nlist = cent.shape[0]
        n = 8 * nlist
        base = (cent[rng.integers(0, nlist, size=n)] + rng.integers(-1, 2, size=(n, dim))).astype(np.float32)
        queries = (cent[rng.integers(0, nlist, size=nq)] + rng.integers(-1, 2, size=(nq, dim))).astype(np.float32)
        with harness.default_pool(tri, slots=16, max_dim=dim, max_nlist=nlist, max_total_lists=nlist) as pool:
            idx = pool.build_index(base, dim, nlist, tri.TRI_F32, tri.TRI_L2, 0, centroids=cent)
            oidx = harness.oracle_index(tri, idx, base)
            with tpq.PQ(pool, idx, 4, train_iters=1, seed=2) as pq:
                qt = torch.from_numpy(queries).cuda()
                for nprobe in (1, 7, 32, 64, 128, 129, 200):
                    for metric in (0, 1):
                        ids, dist, n_out, probes = _to_host(*pq.search(qt, 5, nprobe, metric))
                        pq.sync()
                        for i in range(nq):
                            want = oracle.probe_set(oracle.coarse_scores(oidx, queries[i], metric), nprobe, metric)
                            assert np.array_equal(probes[i], want), f"{name}: nprobe {nprobe} metric {metric} query {i}"
        _say(f"pq probe lists, {name}: exactly the oracle's for nprobe 1..200, both metrics")


def test_lookup_rate_probe():
    """The measurement helper returns a plausible rate (between a thousandth of and the LDS's 128 bytes per clock and
    compute unit at 4 bytes a look-up) and rejects what it documents."""
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    rate = tpq.lds_gather_rate(96, rounds=50)
    assert 256 * 32 * 2.4e9 * 1e-3 < rate < 256 * 32 * 2.4e9 * 1.1
    for bad in (0, 6, 128):
        with pytest.raises(tri.TriError) as ei:
            tpq.lds_gather_rate(bad)
        assert ei.value.status == tri.TRI_EINVAL
    _say(f"pq look-up rate probe: {rate / 1e12:.2f} T look-ups/s with 96 tables")


def test_training_is_reproducible():
    """Training keeps no sum in an order that depends on timing: two builds with the same parameters give the same
    codebooks and codes bit for bit (a sample that does not fill the last of the runs the rows are dealt out in)."""
    tri = harness.lib()
    from paper_2512_02281_amd import pq as tpq
    n, d, nlist, m = 9000, 64, 12, 16
    rng, base, pool, idx, oidx, torch = _setup(tri, "f32", n, d, nlist, seed=31)
    with pool:
        got = []
        for _ in range(2):
            with tpq.PQ(pool, idx, m, train_iters=5, train_rows=4100, seed=9) as pq:
                got.append(pq.export(n, d))
        assert np.array_equal(got[0][0].view(np.uint32), got[1][0].view(np.uint32))
        assert np.array_equal(got[0][1], got[1][1])
        assert np.all(np.isfinite(got[0][0]))
