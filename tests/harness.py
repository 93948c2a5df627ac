"""Shared plumbing of the GPU parity tests: drive the library through its C ABI binding, export
the index it built, run the CPU oracle on the same bytes, compare with the tie-aware checker."""
from __future__ import annotations

import numpy as np

import oracle
from oracle import index as oindex
from tests import checker


PYTEST_CONFIG = None     # set by conftest.py


def say(msg):
    """A progress line that reaches the terminal (and the log of whoever runs the tests) even for a passing
    test: names the case before each long GPU step and carries the parity reports."""
    capman = PYTEST_CONFIG.pluginmanager.get_plugin("capturemanager") if PYTEST_CONFIG is not None else None
    if capman is None:
        print(msg, flush=True)
        return
    with capman.global_and_fixture_disabled():
        print(f"\n    {msg}", end="", flush=True)


def lib():
    import paper_2512_02281_amd as tri
    return tri


def default_pool(tri, **over):
    cfg = dict(slots=256, items_per_step=8192, lists_per_query_step=0, kmax=128, nprobe_max=128,
               max_indexes=2, max_total_lists=8192, max_nlist=4096, max_dim=768, max_outstanding=4096,
               coarse_rows=0, flags=tri.TRI_FLAG_KEEP_PROBES, score_capacity=0)
    cfg.update(over)
    return tri.Pool(**cfg)


def run_all(tri, pool, queries, max_steps=100000, submit_chunks=None, between_steps=None):
    """Submit `queries` (QUERY_DTYPE array), step until everything is finished, poll.

    submit_chunks: None = submit everything first; else a list of chunk sizes, one chunk submitted
    before each step (the rest after the list is exhausted goes in with the last chunk) -- queries
    then arrive mid-stream.  between_steps: called after every search_step (e.g. to synchronise or to run
    other GPU work).  Returns (ids [n, kmax], dist [n, kmax], n_out [n], probes list, stats list).
    """
    n = queries.shape[0]
    kmax = int(queries["k"].max()) if n else 1
    tickets = np.zeros(n, dtype=np.uint64)
    pos = 0
    stats = []
    chunks = list(submit_chunks) if submit_chunks else [n]
    ci = 0
    steps = 0
    while True:
        if pos < n:
            take = chunks[ci] if ci < len(chunks) else n - pos
            if ci == len(chunks) - 1:
                take = n - pos
            ci += 1
            take = min(take, n - pos)
            t, rc = tri.search_submit_batch(pool.handle, queries[pos:pos + take])
            assert rc == tri.TRI_OK and t.shape[0] == take
            tickets[pos:pos + take] = t
            pos += take
        st = tri.search_step(pool.handle)
        stats.append((st.admitted, st.retired, st.running, st.items))
        if between_steps:
            between_steps()
        steps += 1
        assert steps < max_steps, "search_step loop did not drain"
        if pos >= n and st.running == 0 and st.pending_high == 0 and st.pending_low == 0 and st.items == 0:
            break
    tri.search_sync(pool.handle)
    probes = []
    if pool.cfg.flags & tri.TRI_FLAG_KEEP_PROBES:
        for i in range(n):
            probes.append(tri.search_probes(pool.handle, int(tickets[i]), int(queries["nprobe"][i])))
    ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, kmax)
    assert np.all(status == tri.TRI_OK), f"poll status {status[status != 0][:5]}"
    return ids, dist, n_out, probes, stats


def oracle_index(tri, index_handle, base_np):
    cent, off, ids = tri.ivf_export(index_handle)
    return oracle.Index(base_np, cent, off, ids)


def _settled_by_the_batch_oracle(oidx, base_np, vecs, k, nprobe, metric, ids, dist, n_out, probes, rows, tol):
    """Rows whose result is the oracle's own, found with one multi-threaded oracle.search_batch call over `rows`:
    same probe list as a set, same n_out, the same ids in the same order, every score within the tolerance of the
    oracle's for that id.  Such a result meets every condition of the tie-aware checker (nothing is missing, nothing
    is worse than the k-th score), so only the other rows need the checker's candidate-by-candidate comparison.
    Returns the settled rows as a set."""
    rows = np.asarray(list(rows), dtype=np.int64)
    settled = set()
    if rows.size == 0:
        return settled
    want = oracle.search_batch(oidx, vecs[rows], k[rows], nprobe[rows], metric[rows])
    for j, i in enumerate(rows.tolist()):
        kk, npb, m = int(k[i]), int(nprobe[i]), int(metric[i])
        n = int(want["n"][j])
        if int(n_out[i]) != n or probes[i] is None:
            continue
        if set(probes[i].tolist()) != set(want["probe"][j, :npb].tolist()) or len(probes[i]) != npb:
            continue
        if not np.array_equal(np.asarray(ids[i, :kk]), want["ids"][j, :kk]):
            continue
        got, o = np.asarray(dist[i, :n], dtype=np.float64), want["dist"][j, :n]
        q = vecs[i].astype(np.float64)
        qn2 = float((q * q).sum())
        xn2 = (base_np[want["ids"][j, :n]].astype(np.float64) ** 2).sum(axis=1)
        scale = qn2 + xn2 if m == 0 else np.sqrt(qn2 * xn2)
        pad = np.inf if m == 0 else -np.inf
        if np.all(np.abs(got - o) <= checker.score_allowance(m, tol, o, scale)) and \
                np.all(np.asarray(dist[i, n:kk], dtype=np.float64) == pad):
            settled.add(i)
    return settled


def compare_with_oracle(oidx, base_np, vecs, k, nprobe, metric, ids, dist, n_out, probes, strict=False,
                        sample=None, batch_first=False):
    """Check every (or every sampled) query's result against the oracle.  Returns a small report.

    batch_first: the oracle side of all rows is computed first in one multi-threaded call; rows whose result is
    exactly the oracle's are settled by that (see _settled_by_the_batch_oracle), the others -- ties ordered
    differently, near-ties at the coarse boundary, anything wrong -- go through the tie-aware checker below."""
    nq = vecs.shape[0]
    k = np.broadcast_to(np.asarray(k), (nq,))
    nprobe = np.broadcast_to(np.asarray(nprobe), (nq,))
    metric = np.broadcast_to(np.asarray(metric), (nq,))
    tol = 0.0 if strict else checker.tolerance_for(oidx.dtype)
    rows = range(nq) if sample is None else sample
    report = dict(checked=0, coarse_near_tie=0, tie_positions=0)
    if batch_first and probes and not strict:
        settled = _settled_by_the_batch_oracle(oidx, base_np, vecs, k, nprobe, metric, ids, dist, n_out, probes, rows, tol)
        report["checked"] = report["settled_by_batch"] = len(settled)
        rows = [i for i in rows if i not in settled]
    for i in rows:
        q = vecs[i]
        m, kk, npb = int(metric[i]), int(k[i]), int(nprobe[i])
        coarse = oracle.coarse_scores(oidx, q, m)
        want_probe = oracle.probe_set(coarse, npb, m)
        use_probe = want_probe
        if probes:
            got_probe = probes[i]
            assert got_probe is not None and got_probe.shape[0] == npb
            assert len(set(got_probe.tolist())) == npb, "duplicate lists in the probe set"
            if not np.array_equal(got_probe, want_probe):
                # allowed only among centroids whose coarse scores tie within tolerance at the boundary
                # (or anywhere, for the ORDER of the list, which does not change the candidate set)
                if set(got_probe.tolist()) != set(want_probe.tolist()):
                    qn2 = float((q.astype(np.float64) ** 2).sum())
                    cn2 = float((oidx.centroids.astype(np.float64) ** 2).sum(axis=1).max())
                    eps = checker.ABS_EPS * (qn2 + cn2 if m == 0 else np.sqrt(qn2 * cn2))
                    ptol = checker.tolerance_for(oidx.dtype)   # centroids are means: coarse scores are never exact
                    assert checker.probe_sets_equivalent(got_probe, want_probe, coarse, m, ptol, eps), \
                        f"query {i}: probe set differs beyond a boundary near-tie"
                    report["coarse_near_tie"] += 1
                    use_probe = got_probe
        _, _, _, cand_ids, cand_sc = oracle.scan(oidx, q, use_probe, kk, m, all_candidates=True)
        got_ids = np.r_[ids[i, :kk]]
        got_dist = np.r_[dist[i, :kk]]
        report["tie_positions"] += checker.check_result(q, base_np, m, kk, got_ids, got_dist, int(n_out[i]),
                                                        cand_ids, cand_sc, tol, strict=strict)
        report["checked"] += 1
    return report
