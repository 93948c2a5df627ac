#!/usr/bin/env python3
"""Benchmark of the batched IVF search path on one MI355X.

A "step" is one pass of the whole hot path (admit -> coarse assignment -> pack -> list scan ->
top-k merge -> retire) over one batch of synthetic queries whose vectors are already resident in
HBM.  Default workload: configuration 4 (10M x 768 fp16, inner product, nlist 16384, batches of
4096 queries, nprobe 64, k 100).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload config4|config2|config1|config3]

--workload config3 runs the stream of configuration 3 instead (two resident indexes, Poisson arrivals,
the library's native serving loop): saturation throughput with all queries offered at once, then
open-loop runs at fractions of it with p50 / p99 latency per class.
"""
from __future__ import annotations

import argparse
import contextlib
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E bandwidth
# (The HBM traffic per launch -- rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE -- cannot be measured from inside this
# script: it is read from the summaries under profiles/, see traffic_from_profile.)


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


@contextlib.contextmanager
def one_omp_thread():
    """Hold the OpenMP runtime the CPU oracle runs on to one thread (the oracle itself is not touched)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_get_max_threads.restype = ctypes.c_int
    before = omp.omp_get_max_threads()
    omp.omp_set_num_threads(1)
    try:
        yield
    finally:
        omp.omp_set_num_threads(before)


def traffic_from_profile(name, sources):
    """The measured HBM traffic per launch that a rocprofv3 summary under profiles/ records, valid only while the
    kernel sources it was measured on are unchanged: the summary carries the SHA-256 of those sources, and a
    mismatch (a kernel was edited after the counters were collected) makes the figure null instead of stale.
    Returns (bytes or None, provenance dict)."""
    import hashlib
    path = os.path.join(ROOT, "profiles", name)
    prov = {"file": f"profiles/{name}"}
    if not os.path.exists(path):
        prov["status"] = "no such summary"
        return None, prov
    fields = {}
    for line in open(path):
        if line.startswith("@"):                      # machine-readable lines: "@key = value"
            key, _, val = line[1:].partition("=")
            fields[key.strip()] = val.strip()
    h = hashlib.sha256()
    for src in sources:
        h.update(open(os.path.join(ROOT, "paper_2512_02281_amd", "csrc", src), "rb").read())
    prov["profiled_commit"] = fields.get("profiled_commit")
    prov["profiled_on"] = fields.get("profiled_on")
    if fields.get("sources_sha256") != h.hexdigest():
        prov["status"] = "stale: the kernel sources changed after these counters were collected"
        return None, prov
    prov["status"] = "current: the kernel sources are the profiled ones"
    return float(fields["traffic_bytes_per_launch"]), prov


def batch_config(number, args, tri, workloads, torch, headline):
    """One batch configuration (0, 1, 2 or 4): build its index, time the step loop, recall, CPU oracle.
    headline: the full measurement (configuration 4 by default); otherwise a shorter one whose result is nested
    under "configs" of the headline's line."""
    cfg = workloads.CONFIGS[number]
    if args.queries_per_step and headline:
        import dataclasses
        cfg = dataclasses.replace(cfg, n_queries=args.queries_per_step)
    t_start = time.time()
    log(f"workload {cfg.name}: generating {cfg.n_base} x {cfg.dim}")
    if number in (0, 1):
        base_np, queries_np, rows = workloads.make_config01(cfg)
        base_t = torch.from_numpy(base_np).cuda()
        queries_t = torch.from_numpy(queries_np).cuda()
        dtype, metric, tdtype = tri.TRI_F32, tri.TRI_L2, "f32"
        k = np.full(cfg.n_queries, cfg.k, dtype=np.uint32)
        nprobe = np.full(cfg.n_queries, cfg.nprobe, dtype=np.uint32)
    else:
        base_t, queries_t, rows = workloads.make_config_f16(cfg, device="cuda")
        dtype, metric, tdtype = tri.TRI_F16, tri.TRI_IP, "f16"
        if number == 2:
            k, nprobe = workloads.hetero_params(cfg.n_queries, cfg.seed_params)
        else:
            k = np.full(cfg.n_queries, cfg.k, dtype=np.uint32)
            nprobe = np.full(cfg.n_queries, cfg.nprobe, dtype=np.uint32)
    torch.cuda.synchronize()
    Q = cfg.n_queries
    kmax = int(k.max())
    items = int(nprobe.sum())
    steps = args.steps if headline else max(20, args.steps)
    warmup = args.warmup if headline else 5

    pool = tri.Pool(slots=Q, items_per_step=items, lists_per_query_step=0, kmax=max(kmax, 16),
                    nprobe_max=int(nprobe.max()), max_indexes=1, max_total_lists=cfg.nlist, max_nlist=cfg.nlist,
                    max_dim=cfg.dim, max_outstanding=Q * 8, coarse_rows=Q, flags=tri.TRI_FLAG_PROFILE_SCAN,
                    score_capacity=Q * 16384, own_stream=True)
    log("building the index (untimed)")
    t_b = time.time()
    init = base_t[torch.from_numpy(rows).cuda()].float().cpu().numpy()
    index = pool.build_index(base_t, cfg.dim, cfg.nlist, dtype, metric, cfg.train_iters, centroids=init)
    info = tri.ivf_info(index)
    log(f"index built in {time.time() - t_b:.1f}s; longest list {info['max_list_len']}")
    metric_arr = np.full(Q, metric, dtype=np.uint32)
    es = 2 if dtype == tri.TRI_F16 else 4
    qptr, pitch = queries_t.data_ptr(), cfg.dim * es
    queries_host = np.ascontiguousarray(queries_t.cpu().numpy())
    host_q = tri.make_queries(index, queries_host, k, nprobe, metric_arr)

    def one_batch(from_host):
        if from_host:
            tickets, rc = tri.search_submit_batch(pool.handle, host_q)
        else:
            tickets, rc = tri.search_submit_batch_dev(pool.handle, index, qptr, pitch, Q, k, nprobe, metric_arr)
        assert rc == tri.TRI_OK and tickets.shape[0] == Q
        launches = 0
        while True:
            st = tri.search_step(pool.handle)
            launches += st.items > 0
            if st.running == st.retired and st.pending_low == 0 and st.pending_high == 0:
                break                         # every running query retires in the step just enqueued
            assert launches < 10000
        return tickets, launches

    def drain(tickets):
        ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, kmax)
        assert np.all(status == tri.TRI_OK), "a query of a finished batch was not pollable"
        return ids, dist, n_out

    if args.copy_calibration_mib and headline:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads and writes copy_calibration_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    # context beside the vendor's peak: what a bare streaming read of the same base vectors achieves here (best of a few
    # launch shapes, plain or non-temporal loads)
    stream_gbs = tri.tri_stream_read_bandwidth(base_t, 3) if base_t.numel() * base_t.element_size() >= (1 << 20) else None
    if stream_gbs:
        log(f"bare streaming read of the base ({base_t.numel() * base_t.element_size() / 1e9:.2f} GB): {stream_gbs:.0f} GB/s")
    # Settling, untimed and independent of --warmup: the first few hundred milliseconds under load run about
    # 7 % slower than the steady state (clocks ramping up), whatever is executed.
    log("settling 0.6 s under load")
    t_settle = time.perf_counter()
    while time.perf_counter() - t_settle < 0.6:
        tickets, launches_per_batch = one_batch(args.host_queries)
        tri.search_sync(pool.handle)
        drain(tickets)
    log(f"warmup {warmup}")
    last = None
    for _ in range(max(warmup, 1)):
        tickets, launches_per_batch = one_batch(args.host_queries)
        tri.search_sync(pool.handle)
        last = drain(tickets)
    tri.tri_pool_kernel_times(pool.handle, reset=True)

    def timed(n_steps, from_host):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        inflight = []
        for i in range(n_steps):
            tickets, _ = one_batch(from_host)
            inflight.append(tickets)
            if len(inflight) > 2:                 # results of two batches ago are pollable by now or very soon
                t_old = inflight.pop(0)
                ids, dist, n_out, status = tri.search_poll_batch(pool.handle, t_old, kmax)
                pending = t_old[status == tri.TRI_EAGAIN]
                if pending.size:
                    inflight.insert(0, pending)
        tri.search_sync(pool.handle)
        for t_old in inflight:
            drain(t_old)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def repetitions(n_reps, from_host):
        """One batch at a time, first submit to last result on the host, a synchronisation between repetitions:
        the per-batch end-to-end time (median and minimum over the repetitions)."""
        out = []
        for _ in range(n_reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            tickets, _ = one_batch(from_host)
            tri.search_sync(pool.handle)
            drain(tickets)
            out.append((time.perf_counter() - t0) * 1e3)
        out = np.asarray(out)
        return {"repetitions": n_reps, "median_ms": round(float(np.median(out)), 4), "min_ms": round(float(out.min()), 4),
                "queries_per_s_at_median": round(Q / float(np.median(out)) * 1e3, 1)}

    # The timed region: exactly `steps` steps between synchronisations, batches pipelined (results of a batch are
    # polled while later ones run).  The three launches of the list scan of every step are bracketed by HIP events
    # on the pool's stream (their durations for the roofline figure); the other stages are not.
    log(f"timing {steps} steps")
    total_s = timed(steps, args.host_queries)
    ms_per_step = total_s * 1e3 / steps
    qps = Q * steps / total_s
    kt = tri.tri_pool_kernel_times(pool.handle)
    # the same loop with the query vectors submitted from host memory: the PCIe-inclusive rate (never `value`)
    timed(3, not args.host_queries)
    other_s = timed(steps, not args.host_queries)
    host_s, dev_s = (total_s, other_s) if args.host_queries else (other_s, total_s)
    # one batch at a time: median and minimum of the end-to-end time of a batch
    reps_dev = repetitions(max(20, steps // 2), False)
    reps_host = repetitions(max(20, steps // 2), True)
    # stage breakdown: a short run afterwards with every stage bracketed
    tri.tri_pool_set_profiling(pool.handle, tri.TRI_FLAG_PROFILE)
    tri.tri_pool_kernel_times(pool.handle, reset=True)
    timed(10, args.host_queries)
    ks = tri.tri_pool_kernel_times(pool.handle)
    step_launch = None
    if headline:
        # the same loop with the step replayed from its recording (Sec. 3.2), then kernel by kernel, both unprofiled
        tri.tri_pool_set_profiling(pool.handle, 0)
        tri.tri_pool_set_replay(pool.handle, True)
        timed(5, args.host_queries)
        n_cmp = max(10, steps // 4)
        replay_ms = timed(n_cmp, args.host_queries) * 1e3 / n_cmp
        tri.tri_pool_set_replay(pool.handle, False)
        timed(5, args.host_queries)
        eager_ms = timed(n_cmp, args.host_queries) * 1e3 / n_cmp
        log(f"step replayed from its recording: {replay_ms:.3f} ms/step; kernel by kernel, no events: {eager_ms:.3f} ms/step")
        step_launch = {"replayed_graph_ms_per_step": round(replay_ms, 4), "kernel_by_kernel_ms_per_step": round(eager_ms, 4),
                       "note": "same loop, unprofiled"}
    tri.tri_pool_set_profiling(pool.handle, tri.TRI_FLAG_PROFILE_SCAN)
    nl = max(kt.scan_launches, 1)
    sample_ms, thr_ms, main_ms = kt.sample_ms / nl, kt.threshold_ms / nl, kt.scan_ms / nl
    main_b, list_b, tile_b = kt.scan_unique_bytes / nl, kt.scan_list_bytes / nl, kt.scan_vector_bytes / nl
    row_bytes = -(-cfg.dim * es // 128) * 128
    stage_ms = sample_ms + thr_ms + main_ms
    achieved = list_b / (stage_ms * 1e-3) / 1e9 if stage_ms > 0 else 0.0
    main_achieved = main_b / (main_ms * 1e-3) / 1e9 if main_ms > 0 else 0.0
    sample_b = list_b - main_b
    log(f"{ms_per_step:.3f} ms/step, {qps:.0f} q/s; scan stage {stage_ms:.3f} ms (sample {sample_ms:.3f} + thresholds {thr_ms:.3f} + main "
        f"{main_ms:.3f}) for {list_b / 1e9:.2f} GB -> {achieved:.0f} GB/s; main launch alone {main_achieved:.0f} GB/s; stages ms/step (extra run): "
        f"admit {ks.admit_ms / ks.steps:.3f} coarse {ks.coarse_ms / ks.steps:.3f} pack {ks.pack_ms / ks.steps:.3f} sample {ks.sample_ms / ks.steps:.3f} "
        f"thresholds {ks.threshold_ms / ks.steps:.3f} scan {ks.scan_ms / ks.steps:.3f} select {ks.select_ms / ks.steps:.3f}")

    # ---- recall of the returned lists against exact search (torch matmul on the GPU, harness only)
    recall = None
    if args.recall_sample:
        ids, dist, n_out = last
        rs = np.random.default_rng(77).choice(Q, size=min(args.recall_sample, Q), replace=False)
        qs = queries_t[torch.from_numpy(rs).cuda()]
        hits = tot = 0
        for j, qi in enumerate(rs):
            kk = int(k[qi])
            if metric == tri.TRI_IP:
                sc = (base_t @ qs[j]).float()
                top = torch.topk(sc, kk).indices
            else:
                sc = ((base_t - qs[j]) ** 2).sum(dim=1)
                top = torch.topk(sc, kk, largest=False).indices
            hits += len(set(top.cpu().numpy().tolist()) & set(ids[qi, :kk].tolist()))
            tot += kk
        recall = hits / tot
        log(f"recall@k on {rs.size} queries: {recall:.4f}")

    # ---- the CPU oracle on a bounded sample of the same batch, same box
    cpu = None
    n_cpu = args.cpu_sample if args.cpu_sample >= 0 else {4: 1024, 2: 1024, 1: 1024, 0: 100}[number]
    if not headline:
        n_cpu = min(n_cpu, 512)
    if n_cpu:
        import oracle
        log("exporting the index and copying the base to the host for the CPU oracle")
        cent, off, lids = tri.ivf_export(index)
        base_host = base_t.cpu().numpy()
        oidx = oracle.Index(base_host, cent, off, lids)
        sel = np.arange(0, Q, max(1, Q // n_cpu))[:n_cpu]
        qh = queries_host[sel]
        tc0 = time.perf_counter()
        out = oracle.search_batch(oidx, qh, k[sel], nprobe[sel], metric_arr[sel])
        tc = time.perf_counter() - tc0
        cpu = {"value": round(sel.size / tc, 3), "unit": "queries/s", "cores": out["threads"], "kind": "oracle",
               "sample": f"{sel.size} queries of the same batch (every {max(1, Q // n_cpu)}-th), {tc:.1f} s of wall time"}
        if headline:
            # the same oracle held to one thread, on a smaller sample sized from the rate just measured
            n_one = int(min(sel.size, max(8, 6.0 * sel.size / tc / max(1, out["threads"]))))
            one = sel[:: max(1, sel.size // n_one)][:n_one]
            with one_omp_thread():
                t1 = time.perf_counter()
                out1 = oracle.search_batch(oidx, queries_host[one], k[one], nprobe[one], metric_arr[one])
                t1 = time.perf_counter() - t1
            if out1["threads"] == 1:
                cpu["one_core"] = {"value": round(one.size / t1, 3), "unit": "queries/s",
                                   "sample": f"{one.size} of those queries, {t1:.1f} s"}
        log(f"cpu oracle: {cpu}")
        del base_host, oidx

    traffic, traffic_prov = (None, None)
    if number == 4 and not args.queries_per_step:
        traffic, traffic_prov = traffic_from_profile("scan_kernel_config4.txt", ["scan.hip", "select.hip", "tri_common.h", "tri_mfma.h"])
    cache_note = None
    if list_b < 4e9:
        cache_note = ("the probed lists of a step are %.2f GB, small enough to stay in the 256 MB last-level cache in part and re-read "
                      "per 32-query tile: cache-assisted, not an HBM figure" % (list_b / 1e9))
    rescans = tri.tri_pool_candidate_rescans(pool.handle)
    log(f"queries whose candidate region was too small (re-scored by the merge kernel) since the pool was created: {rescans}")
    result = {
        "metric": "queries/sec at recall@k>=0.9 (1 GPU) + list-scan HBM GB/s as % of peak",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": tdtype, "data": "synthetic", "settle_s": 0.6,
        "config": {"workload": f"configs[{number}] {cfg.name}: {cfg.n_base} x {cfg.dim} {tdtype}, nlist {cfg.nlist}, "
                               f"{Q} queries/step, nprobe {int(nprobe.max()) if number != 2 else 'U{8..128}'}, "
                               f"k {kmax if number != 2 else 'U{1,10,100}'}",
                   "queries_per_step": Q, "items_per_step": items, "launches_per_step": launches_per_batch,
                   "recall_at_k": None if recall is None else round(recall, 4),
                   "recall_sample": min(args.recall_sample, Q),
                   "longest_list": info["max_list_len"], "candidate_region_rescans": rescans,
                   "query_vectors": "host memory (PCIe-inclusive side measurement)" if args.host_queries else "device-resident"},
        # PCIe-inclusive: query vectors copied from host memory at submit and fetched over the bus by the admitting
        # step; results land in pinned host memory either way.  Never `value`.
        "value_host_queries": {"value": round(Q * steps / host_s, 1), "unit": "queries/s", "ms_per_step": round(host_s * 1e3 / steps, 4),
                               "device_resident_same_run": round(Q * steps / dev_s, 1)},
        "per_batch_end_to_end": {"device_resident_queries": reps_dev, "host_queries": reps_host},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_prov,
                     "kernel": "list-scan stage: scan_wave_kernel sample launch + slot_threshold_kernel + scan_wave_kernel main launch; "
                               "every probed list once over the HIP-event time of the three",
                     "avg_launch_ms": round(stage_ms, 4), "algorithmic_bytes_per_launch": int(list_b),
                     "scan_stage": {"sample_ms": round(sample_ms, 4), "threshold_ms": round(thr_ms, 4), "main_ms": round(main_ms, 4),
                                    "bytes_all_lists": int(list_b), "frac_whole": round(achieved / HBM_PEAK_GBS, 4)},
                     "main_launch": {"kernel": "scan_wave_kernel (main launch)", "avg_launch_ms": round(main_ms, 4),
                                     "algorithmic_bytes_per_launch": int(main_b), "achieved": round(main_achieved, 1),
                                     "frac": round(main_achieved / HBM_PEAK_GBS, 4)},
                     "sample_launch": {"avg_launch_ms": round(sample_ms, 4), "algorithmic_bytes_per_launch": int(sample_b),
                                       "achieved": round(sample_b / (sample_ms * 1e-3) / 1e9, 1) if sample_ms > 0 else None},
                     "streaming_read_GBs": None if stream_gbs is None else round(stream_gbs, 1),
                     "tile_bytes_per_launch": int(tile_b),
                     "items_per_launch": int(kt.scan_items / nl), "row_bytes": row_bytes, "note": cache_note},
        "stages_ms_per_step": {"admit": round(ks.admit_ms / ks.steps, 4), "coarse": round(ks.coarse_ms / ks.steps, 4),
                               "pack": round(ks.pack_ms / ks.steps, 4), "sample": round(ks.sample_ms / ks.steps, 4),
                               "thresholds": round(ks.threshold_ms / ks.steps, 4),
                               "scan": round(ks.scan_ms / ks.steps, 4), "select": round(ks.select_ms / ks.steps, 4),
                               "note": "10 more steps, every stage bracketed"},
        "step_launch": step_launch,
        "cpu_baseline": cpu,
        "wall_s_total": round(time.time() - t_start, 1),
    }
    pool.close()
    del base_t, queries_t, pool
    torch.cuda.empty_cache()
    return result


def rowclass_bench(args, tri, torch):
    """Side measurement: the list-scan stage for every kind of scan kernel -- row lengths of 512, 1024, 1536 and
    2048 bytes in fp16 and fp32 (register-resident kernels where they exist, the LDS kernel elsewhere) and two
    lengths only the LDS kernel's generic path serves.  2M unit-norm vectors each, nlist 2048, 2048 queries per
    step, nprobe 32, k 10, inner product: every list is probed by about 32 queries, i.e. one full tile."""
    t_start = time.time()
    n, nlist, Q, nprobe, k = 2_000_000, 2048, 2048, 32, 10
    rows = []
    for tdtype, dim in (("f16", 256), ("f16", 512), ("f16", 768), ("f16", 1024), ("f32", 128), ("f32", 256), ("f32", 384),
                        ("f32", 512), ("f16", 320), ("f32", 200)):
        g = torch.Generator(device="cuda").manual_seed(5000 + dim)
        centres = torch.nn.functional.normalize(torch.randn(nlist, dim, generator=g, device="cuda"), dim=1)
        tt = torch.float16 if tdtype == "f16" else torch.float32
        base = torch.empty(n, dim, dtype=tt, device="cuda")
        for s0 in range(0, n, 1 << 18):
            m = min(1 << 18, n - s0)
            c = torch.randint(0, nlist, (m,), generator=g, device="cuda")
            base[s0:s0 + m] = torch.nn.functional.normalize(centres[c] + 0.05 * torch.randn(m, dim, generator=g, device="cuda"), dim=1).to(tt)
        c = torch.randint(0, nlist, (Q,), generator=g, device="cuda")
        queries = torch.nn.functional.normalize(centres[c] + 0.05 * torch.randn(Q, dim, generator=g, device="cuda"), dim=1).to(tt).contiguous()
        dtype = tri.TRI_F16 if tdtype == "f16" else tri.TRI_F32
        es = 2 if tdtype == "f16" else 4
        pool = tri.Pool(slots=Q, items_per_step=Q * nprobe, lists_per_query_step=0, kmax=16, nprobe_max=nprobe, max_indexes=1,
                        max_total_lists=nlist, max_nlist=nlist, max_dim=dim, max_outstanding=Q * 8, coarse_rows=Q,
                        flags=tri.TRI_FLAG_PROFILE_SCAN, score_capacity=Q * 16384, own_stream=True)
        index = pool.build_index(base, dim, nlist, dtype, tri.TRI_IP, 4, centroids=centres.float().cpu().numpy())
        kk = np.full(Q, k, dtype=np.uint32)
        pp = np.full(Q, nprobe, dtype=np.uint32)
        mm = np.full(Q, tri.TRI_IP, dtype=np.uint32)

        def one():
            t, rc = tri.search_submit_batch_dev(pool.handle, index, queries.data_ptr(), dim * es, Q, kk, pp, mm)
            assert rc == tri.TRI_OK
            st = tri.search_step(pool.handle)
            assert st.retired == Q
            tri.search_sync(pool.handle)
            tri.search_poll_batch(pool.handle, t, k)

        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.3:
            one()
        tri.tri_pool_kernel_times(pool.handle, reset=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            one()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        kt = tri.tri_pool_kernel_times(pool.handle)
        nl = max(kt.scan_launches, 1)
        row_bytes = -(-dim * es // 128) * 128
        kind = ("register-resident, one wavefront per tile" if (row_bytes in (512, 1024) or (tdtype == "f16" and row_bytes in (1536, 2048)))
                else "LDS kernel, pipelined" if row_bytes in (1536, 2048) else "LDS kernel, generic")
        r = {"dtype": tdtype, "dim": dim, "row_bytes": row_bytes, "kernel": kind, "ms_per_step_synchronous": round(ms, 4),
             "sample_ms": round(kt.sample_ms / nl, 4), "threshold_ms": round(kt.threshold_ms / nl, 4), "main_ms": round(kt.scan_ms / nl, 4),
             "lists_GB": round(kt.scan_list_bytes / nl / 1e9, 3),
             "main_launch_GBs": round(kt.scan_unique_bytes / max(kt.scan_ms, 1e-9) / 1e6, 1),
             "scan_stage_GBs": round(kt.scan_list_bytes / max(kt.sample_ms + kt.threshold_ms + kt.scan_ms, 1e-9) / 1e6, 1),
             "rescans": tri.tri_pool_candidate_rescans(pool.handle)}
        log(str(r))
        rows.append(r)
        pool.close()
        del base, queries, pool
        torch.cuda.empty_cache()
    best = max(rows, key=lambda r: r["scan_stage_GBs"])
    print(json.dumps({
        "metric": "queries/sec at recall@k>=0.9 (1 GPU) + list-scan HBM GB/s as % of peak", "value": None, "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": 0, "ms_per_step": None, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16/f32", "data": "synthetic",
        "config": {"workload": f"side measurement: the scan stage per row-length class, {n} unit-norm vectors, nlist {nlist}, {Q} queries/step, "
                               f"nprobe {nprobe}, k {k}, inner product"},
        "roofline": {"bound": "hbm", "achieved": best["scan_stage_GBs"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(best["scan_stage_GBs"] / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "best class: " + best["kernel"]},
        "row_classes": rows, "cpu_baseline": None, "wall_s_total": round(time.time() - t_start, 1)}), flush=True)


def pq_bench(args, tri, workloads, torch):
    """Side measurement: IVF search over product-quantised lists (include/trinity_pq.h) on configuration 2's data --
    1M x 768 fp16 unit-norm, inner product, nlist 4096 -- with m = 96 sub-spaces (96 bytes per vector instead of 1536),
    batches of 2048 queries, nprobe 32, k 10; by table scores alone and with the 100 / 256 best of them re-ranked by
    exact scores read from the tri_pq's own row-major copy of the vectors (pq_params.refine_rows: re-ranking gathers
    whole rows by id, which the index's interleaved blocks, laid out for the list scan, serve badly).  Recall is
    against exact search over the stored vectors; `value` is the fastest mode that reaches
    0.9 (the table-score mode if none does)."""
    from paper_2512_02281_amd import pq as tpq
    t_start = time.time()
    cfg = workloads.CONFIGS[2]
    m, nq, nprobe, k = 96, 2048, 32, 10
    log(f"workload pq on {cfg.name}: generating {cfg.n_base} x {cfg.dim}")
    base_t, queries_t, rows = workloads.make_config_f16(cfg, device="cuda")
    queries_t = queries_t[:nq].contiguous()
    pool = tri.Pool(slots=64, items_per_step=4096, lists_per_query_step=0, kmax=16, nprobe_max=32, max_indexes=1,
                    max_total_lists=cfg.nlist, max_nlist=cfg.nlist, max_dim=cfg.dim, max_outstanding=256, coarse_rows=64,
                    flags=0, score_capacity=0, own_stream=True)
    index = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 4, centroids=base_t[torch.from_numpy(rows.astype(np.int64)).cuda()].float().cpu().numpy())
    t0 = time.perf_counter()
    pq = tpq.PQ(pool, index, m, train_iters=8, train_rows=65536, seed=1, refine_rows=True)
    build_s = time.perf_counter() - t0
    ws = pq.workspace(nq)
    out = pq.search(queries_t, k, nprobe, tri.TRI_IP, ws=ws)
    pq.sync()
    rs = min(args.recall_sample, nq) if args.recall_sample else 0
    exact = torch.topk(queries_t[:rs].float() @ base_t.float().T, k, dim=1).indices.cpu().numpy() if rs else None
    modes = []
    for k_adc in (0, 100, 256):
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.3:
            pq.search(queries_t, k, nprobe, tri.TRI_IP, ws=ws, out=out, k_adc=k_adc)
            pq.sync()
        for _ in range(args.warmup):
            pq.search(queries_t, k, nprobe, tri.TRI_IP, ws=ws, out=out, k_adc=k_adc)
        pq.sync()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pq.search(queries_t, k, nprobe, tri.TRI_IP, ws=ws, out=out, k_adc=k_adc)
        pq.sync()
        torch.cuda.synchronize()
        ms_mode = (time.perf_counter() - t0) * 1e3 / args.steps
        got = out[0].cpu().numpy().view(np.uint32).astype(np.int64)
        rec = float(np.mean([len(set(got[i].tolist()) & set(exact[i].tolist())) / k for i in range(rs)])) if rs else None
        modes.append({"k_adc": k_adc, "ms_per_batch": round(ms_mode, 4), "qps": round(nq / ms_mode * 1e3, 1), "recall_at_k": rec})
        log(f"pq: short list {k_adc or 'none'}: {ms_mode:.3f} ms per batch = {nq / ms_mode * 1e3:.0f} q/s, recall@{k} {rec}")
    good = [x for x in modes if x["recall_at_k"] is not None and x["recall_at_k"] >= 0.9]
    head = max(good, key=lambda x: x["qps"]) if good else modes[0]
    ms, recall = head["ms_per_batch"], head["recall_at_k"]
    out = pq.search(queries_t, k, nprobe, tri.TRI_IP, ws=ws, out=out, k_adc=0)          # (the table-score result, for the oracle comparison below)
    pq.sync()
    ids = out[0].cpu().numpy().view(np.uint32).astype(np.int64)
    probes = out[3].cpu().numpy().view(np.uint32).astype(np.int64)
    # what the batch scans: codes of the probed lists per query (look-ups = m per code), distinct lists once (bytes)
    cent, list_off, list_ids = tri.ivf_export(index)
    lens = np.diff(list_off.astype(np.int64))
    codes_scanned = int(lens[probes].sum())
    lookups = codes_scanned * m
    unique_bytes = int(lens[np.unique(probes)].sum()) * m
    cpu = None
    cs = 64 if args.cpu_sample < 0 else args.cpu_sample
    if cs:
        import oracle
        from oracle import pq as opq
        cb, codes = pq.export(cfg.n_base, cfg.dim)
        oidx = oracle.Index(base_t.cpu().numpy(), cent, list_off, list_ids)
        qh = queries_t[:cs].cpu().numpy()
        t0 = time.perf_counter()
        same = 0
        for i in range(cs):
            _, oid, _, _ = opq.search(oidx, codes, cb, qh[i], k, nprobe, 1)
            same += int(np.array_equal(oid, ids[i]))
        dt = time.perf_counter() - t0
        cpu = {"value": round(cs / dt, 3), "unit": "queries/s", "cores": 1, "kind": "oracle",
               "sample": f"{cs} queries of the same batch, {dt:.1f} s of wall time; {same} of them returned exactly the GPU's ids"}
    lds_peak = 256 * 128 * 2.4          # GB/s: 256 compute units x 128 bytes of LDS per clock x 2.4 GHz
    achieved = lookups * 4 / (modes[0]["ms_per_batch"] * 1e-3) / 1e9          # (the table-score pass alone)
    # what byte-indexed look-ups on random codes can reach at all: the scan's inner loop alone, measured now
    bare = tpq.lds_gather_rate(m, rounds=5000) * 4 / 1e9          # (35 ms: its start-up no longer shows)
    log(f"pq: {ms:.3f} ms per batch of {nq} = {nq / ms * 1e3:.0f} q/s, recall@{k} {recall}, {codes_scanned} codes x {m} look-ups "
        f"-> {achieved:.0f} GB/s of LDS reads (a bare loop of such look-ups: {bare:.0f} GB/s); build {build_s:.1f} s")
    result = {
        "metric": "queries/sec at recall@k>=0.9 (1 GPU) + list-scan HBM GB/s as % of peak", "value": round(nq / ms * 1e3, 1), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32 tables over u8 codes of f16 vectors", "data": "synthetic",
        "config": {"workload": f"side measurement: IVF over product-quantised lists on configs[2]'s data ({cfg.n_base} x {cfg.dim} f16, nlist {cfg.nlist}), "
                               f"m {m} sub-spaces of {cfg.dim // m}, {nq} queries per batch, nprobe {nprobe}, k {k}, inner product",
                   "queries_per_step": nq, "recall_at_k": recall, "recall_sample": rs, "bytes_per_vector": m,
                   "short_list_for_exact_reranking": head["k_adc"], "rows_for_reranking": "row-major copy by id (refine_rows)", "modes": modes,
                   "codes_scanned_per_batch": codes_scanned, "pq_build_s": round(build_s, 2), "query_vectors": "device-resident"},
        "roofline": {"bound": "lds", "achieved": round(achieved, 1), "peak": lds_peak, "unit": "GB/s", "frac": round(achieved / lds_peak, 4),
                     "traffic": None, "kernel": "pq_scan_kernel + the batch's four other launches (whole batch time)",
                     "lookups_per_batch": lookups, "unique_code_bytes_per_batch": unique_bytes,
                     "bare_lookup_loop": {"achieved": round(bare, 1), "unit": "GB/s", "frac_of_it": round(achieved / bare, 4),
                                          "note": "the scan's inner loop alone (random bytes, m tables in LDS, one 1024-thread workgroup per "
                                                  "compute unit), measured in this run: random indices collide on LDS banks"},
                     "note": "m 4-byte LDS look-ups per scanned code; peak = 256 compute units x 128 B of LDS per clock x 2.4 GHz; "
                             "the codes themselves (96 MB in all) are cache-resident"},
        "cpu_baseline": cpu, "wall_s_total": round(time.time() - t_start, 1)}
    pq.close()
    pool.close()
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="config4", choices=["config4", "config2", "config1", "config0", "config3", "graph", "graph-stream", "rowclasses", "pq"])
    ap.add_argument("--only-headline", action="store_true",
                    help="config4: skip the shorter measurements of configurations 0-3 that the default run nests under \"configs\"")
    ap.add_argument("--graph-n", type=int, default=1_000_000, help="graph workload: database rows")
    ap.add_argument("--graph-slots", type=int, default=8192, help="graph workload: requests advanced per step")
    ap.add_argument("--graph-topm", type=int, default=128, help="graph workload: length of a request's candidate list")
    ap.add_argument("--graph-parents", type=int, default=4, help="graph workload: parents expanded per extend")
    ap.add_argument("--graph-groups", type=int, default=3, help="graph workload: slot groups stepped in turn (1..4)")
    ap.add_argument("--graph-seeds", type=int, default=64, help="graph workload: entry points")
    ap.add_argument("--queries-per-step", type=int, default=0,
                    help="config1/2/4: queries per batch instead of the configuration's own number (a side measurement of how "
                         "the path scales when more queries share each list read; never the headline value)")
    ap.add_argument("--stream-queries", type=int, default=100_000, help="config3: queries in the stream")
    ap.add_argument("--cpu-sample", type=int, default=-1, help="queries timed on the CPU oracle (0 = skip)")
    ap.add_argument("--recall-sample", type=int, default=256, help="queries checked against exact search (graph workload: as many)")
    ap.add_argument("--host-queries", action="store_true",
                    help="submit the query vectors of the timed region from host memory (adds their PCIe transfer to every step; "
                         "a side measurement, never the headline value)")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="run one plain device copy of this many MiB before timing (a kernel of known traffic, "
                         "to scale profiler byte counters)")
    args = ap.parse_args()
    t_run_start = time.time()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path does not shard in this round); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    lib_path = os.path.join(ROOT, "paper_2512_02281_amd", "libtrinity_ivf.so")
    if not os.path.exists(lib_path):
        from paper_2512_02281_amd.build import build_library  # the only case in which bench builds
        build_library()
    import torch
    import paper_2512_02281_amd as tri
    import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(3)
    if args.workload == "graph":
        print(json.dumps(graph_bench(args, tri, torch)), flush=True)
        return
    if args.workload == "graph-stream":
        return graph_stream_bench(args, tri, torch)
    if args.workload == "rowclasses":
        return rowclass_bench(args, tri, torch)
    if args.workload == "pq":
        print(json.dumps(pq_bench(args, tri, workloads, torch)), flush=True)
        return
    number = int(args.workload[-1])
    if number == 3:
        print(json.dumps(stream_bench(args, tri, workloads, torch, brief=False)), flush=True)
        return
    result = batch_config(number, args, tri, workloads, torch, headline=True)
    if number == 4 and not args.only_headline and not args.queries_per_step and not args.host_queries:
        # the other configurations, shorter, in the same run: absolute queries/s, recall and the CPU oracle beside
        # each; one compact record per configuration in the line, the full record of each on stderr
        others = {}
        for other in (0, 1, 2):
            r = batch_config(other, args, tri, workloads, torch, headline=False)
            log("full record of configs[%d]: %s" % (other, json.dumps(r)))
            e2e = r["per_batch_end_to_end"]
            others[str(other)] = {
                "qps": r["value"], "ms_per_step": r["ms_per_step"], "launches_per_step": r["config"]["launches_per_step"],
                "recall_at_k": r["config"]["recall_at_k"], "qps_host_queries": r["value_host_queries"]["value"],
                "batch_ms_median_min": [e2e["device_resident_queries"]["median_ms"], e2e["device_resident_queries"]["min_ms"]],
                "batch_ms_median_min_host_queries": [e2e["host_queries"]["median_ms"], e2e["host_queries"]["min_ms"]],
                "scan_stage_GBs": r["roofline"]["achieved"], "scan_lists_GB": round(r["roofline"]["algorithmic_bytes_per_launch"] / 1e9, 3),
                "cache_assisted": r["roofline"]["note"] is not None,
                "cpu_oracle_qps": r["cpu_baseline"]["value"] if r["cpu_baseline"] else None,
                "cpu_cores": r["cpu_baseline"]["cores"] if r["cpu_baseline"] else None,
                "cpu_sample": int(r["cpu_baseline"]["sample"].split()[0]) if r["cpu_baseline"] else None}
        r = stream_bench(args, tri, workloads, torch, brief=True)
        log("full record of configs[3]: %s" % json.dumps(r))
        runs = r["stream"]
        others["3"] = {"saturation_qps": r["value"], "queries": args.stream_queries, "slots": 4096, "lists_per_query_step": 8,
                       "query_vectors": "host memory",
                       "open_loop": [{"offered_qps": x["offered_qps"], "qps": x["throughput_qps"],
                                      "p50_p99_ms": x["latency_ms_p50_p99"]["all"],
                                      "p50_p99_ms_cache_high_class": x["latency_ms_p50_p99"]["cache_high_class"]} for x in runs[1:4]],
                       "cpu_oracle_qps": r["cpu_baseline"]["value"] if r["cpu_baseline"] else None,
                       "cpu_cores": r["cpu_baseline"]["cores"] if r["cpu_baseline"] else None}
        result["configs"] = others
        # the two other engines, as compact records too (their own workloads print the full ones); a failure there is
        # recorded, never allowed to take the headline with it
        engines = {}
        for name, run in (("graph", lambda: graph_bench(args, tri, torch)), ("pq", lambda: pq_bench(args, tri, workloads, torch))):
            try:
                r = run()
                log("full record of the %s engine: %s" % (name, json.dumps(r)))
                rec = {"workload": r["config"]["workload"], "qps": r["value"], "ms_per_step": r["ms_per_step"],
                       "recall_at_k": r["config"]["recall_at_k"], "bound": r["roofline"]["bound"],
                       "achieved": r["roofline"]["achieved"], "unit": r["roofline"]["unit"], "frac": r["roofline"]["frac"],
                       "cpu_oracle_qps": r["cpu_baseline"]["value"] if r["cpu_baseline"] else None}
                if name == "pq":
                    rec["modes"] = r["config"]["modes"]
                    rec["frac_of_bare_lookup_loop"] = r["roofline"]["bare_lookup_loop"]["frac_of_it"]
                engines[name] = rec
            except Exception as e:          # noqa: BLE001 (whatever it is, the headline stands)
                engines[name] = {"error": "%s: %s" % (type(e).__name__, e)}
        result["engines"] = engines
        result["wall_s_run"] = round(time.time() - t_run_start, 1)          # (the whole run: every configuration and engine)
    print(json.dumps(result), flush=True)


def stream_bench(args, tri, workloads, torch, brief):
    """Configuration 3: 70 % RAG queries (k ~ U{10..100}, nprobe 32, low class) over the 1M x 768 index,
    30 % prompt-cache lookups (k 1, nprobe 8, high class) over the 200k x 768 index, 4096 slots, 8 lists
    per query and step.  brief: saturation and the three open-loop rates only (the summary the default run
    nests under "configs"); otherwise also the static-batch scheme, the step-boundary policies and the
    replayed step.  Returns the result."""
    t_start = time.time()
    rag_cfg, cache_cfg = workloads.CONFIGS[2], workloads.CACHE_INDEX
    n, slots, p = args.stream_queries, 4096, 8
    log(f"workload config3: generating 2 bases and {n} queries")
    w = workloads.make_config3(n, "cuda", rag_cfg, cache_cfg)
    torch.cuda.synchronize()
    queries = np.ascontiguousarray(w["queries"].cpu().numpy())
    pool = tri.Pool(slots=slots, items_per_step=slots * p, lists_per_query_step=p, kmax=128, nprobe_max=32,
                    max_indexes=2, max_total_lists=rag_cfg.nlist + cache_cfg.nlist, max_nlist=rag_cfg.nlist,
                    max_dim=768, max_outstanding=n, coarse_rows=0, flags=tri.TRI_FLAG_PROFILE,
                    score_capacity=256 << 20, own_stream=True)
    log("building the two indexes (untimed)")
    init_r = w["rag_base"][torch.from_numpy(w["rag_rows"]).cuda()].float().cpu().numpy()
    init_c = w["cache_base"][torch.from_numpy(w["cache_rows"]).cuda()].float().cpu().numpy()
    ir = pool.build_index(w["rag_base"], rag_cfg.dim, rag_cfg.nlist, tri.TRI_F16, tri.TRI_IP, rag_cfg.train_iters, centroids=init_r)
    ic = pool.build_index(w["cache_base"], cache_cfg.dim, cache_cfg.nlist, tri.TRI_F16, tri.TRI_IP, cache_cfg.train_iters, centroids=init_c)
    index_of = np.where(w["is_rag"], ir, ic).astype(np.uint64)
    q = tri.make_queries(index_of, queries, w["k"], w["nprobe"], tri.TRI_IP, w["klass"])
    is_rag = w["is_rag"]

    def run(arrival, label, qq=None, **policy):
        qq = q if qq is None else qq
        tri.search_set_policy(pool.handle, **policy)
        tri.tri_pool_kernel_times(pool.handle, reset=True)
        ids, dist, n_out, done_s, st, _ = tri.search_run_stream(pool.handle, qq, arrival, 100, depth=2)
        lat = (done_s - arrival) * 1e3
        kt = tri.tri_pool_kernel_times(pool.handle)
        pct = lambda a: [round(float(np.percentile(a, x)), 3) for x in (50, 99)]
        r = {"label": label, "offered_qps": None if arrival[-1] == 0 else round(n / arrival[-1], 1),
             "throughput_qps": round(n / st.wall_s, 1), "steps": int(st.steps),
             "mean_items_per_step": round(st.items / max(st.steps, 1), 1),
             "padding_fraction": round(1 - st.items / max(st.capacity, 1), 4),
             "mean_running_slots": round(st.running / max(st.steps, 1), 1), "longest_queue": int(st.max_pending),
             "latency_ms_p50_p99": {"all": pct(lat), "rag_low_class": pct(lat[is_rag]), "cache_high_class": pct(lat[~is_rag])},
             "cache_hit_rate": round(float((dist[~is_rag, 0] >= 0.95).mean()), 4),
             "host_s": {"wall": round(st.wall_s, 4), "submit": round(st.submit_s, 4), "search_step": round(st.step_s, 4),
                        "collect": round(st.collect_s, 4)},
             "scan_ms_per_step": round(kt.scan_ms / max(kt.scan_launches, 1), 4),
             "scan_unique_GBs": round(kt.scan_unique_bytes / max(kt.scan_ms, 1e-9) / 1e6, 1)}
        log(str(r))
        return r, kt, st

    log("warmup")
    run(np.zeros(n), "warmup")
    sat, kt, st = run(np.zeros(n), "closed loop: all queries offered at t = 0")
    t_sat = sat["throughput_qps"]
    runs = [sat]
    for frac in (0.5, 0.8):
        runs.append(run(workloads.poisson_arrivals(n, frac * t_sat, 4003), f"Poisson arrivals at {frac} x saturation")[0])
    runs.append(run(workloads.poisson_arrivals(n, 1.0e5, 4003), "Poisson arrivals at 100,000 / s")[0])
    if not brief:
        more_stream_runs(runs, run, tri, pool, workloads, n, q, is_rag, t_sat)
    return finish_stream(args, tri, pool, w, ir, ic, queries, is_rag, n, slots, p, runs, t_sat, kt, st, t_start)


def more_stream_runs(runs, run, tri, pool, workloads, n, q, is_rag, t_sat):
    # the scheme continuous batching replaces (Sec. 3.2): a batch must drain before the next is admitted
    runs.append(run(np.zeros(n), "closed loop, static batches", static_batches=True)[0])
    for frac in (0.5, 0.8):
        runs.append(run(workloads.poisson_arrivals(n, frac * t_sat, 4003), f"Poisson arrivals at {frac} x saturation, static batches",
                        static_batches=True)[0])
    # the step-boundary policy (Sec. 3.3) where slots are scarce -- a burst, everything offered at once:
    # one queue, two classes with the cache lookups first, a reserved share, and least-slack order with
    # a budget on the cache lookups
    burst = np.zeros(n)
    q_one = q.copy()
    q_one["klass"] = tri.TRI_CLASS_LOW
    q_ddl = q.copy()
    q_ddl["deadline_ns"] = np.where(is_rag, 0, 20_000_000)
    runs.append(run(burst, "burst, one class (first-in first-out only)", qq=q_one)[0])
    runs.append(run(burst, "burst, two classes, high class first (share 1)")[0])
    runs.append(run(burst, "burst, two classes, reserved share 0.3", high_share=0.3)[0])
    runs.append(run(burst, "burst, reserved share 0.3, least slack first, 20 ms budget on cache lookups",
                    qq=q_ddl, high_share=0.3, order_high=tri.TRI_ORDER_SLACK)[0])
    tri.search_set_policy(pool.handle)
    # launch overhead of a step (Sec. 3.2: the captured fixed-shape step): the same streams unprofiled,
    # kernel by kernel and replayed from the recording
    tri.tri_pool_set_profiling(pool.handle, 0)
    low = workloads.poisson_arrivals(n, 1.0e5, 4003)
    for replay in (False, True):
        tri.tri_pool_set_replay(pool.handle, replay)
        how = "replayed recording" if replay else "kernel by kernel"
        run(burst, f"warmup ({how})")
        runs.append(run(burst, f"closed loop, no profiling events, {how}")[0])
        runs.append(run(low, f"Poisson arrivals at 100,000 / s, no profiling events, {how}")[0])
    tri.tri_pool_set_replay(pool.handle, False)
    tri.tri_pool_set_profiling(pool.handle, tri.TRI_FLAG_PROFILE)


def finish_stream(args, tri, pool, w, ir, ic, queries, is_rag, n, slots, p, runs, t_sat, kt, st, t_start):
    import torch
    cpu = None
    n_cpu = args.cpu_sample if args.cpu_sample >= 0 else 512
    if n_cpu:
        import oracle
        log("CPU oracle on a sample of the stream")
        sel = np.arange(0, n, max(1, n // n_cpu))[:n_cpu]
        tc = 0.0
        threads = 0
        for idx, base_t, mask in ((ir, w["rag_base"], is_rag[sel]), (ic, w["cache_base"], ~is_rag[sel])):
            cent, off, lids = tri.ivf_export(idx)
            oidx = oracle.Index(base_t.cpu().numpy(), cent, off, lids)
            ss = sel[mask]
            t0 = time.perf_counter()
            out = oracle.search_batch(oidx, queries[ss], w["k"][ss], w["nprobe"][ss], np.ones(ss.size, dtype=np.uint32))
            tc += time.perf_counter() - t0
            threads = out["threads"]
        cpu = {"value": round(sel.size / tc, 3), "unit": "queries/s", "cores": threads, "kind": "oracle",
               "sample": f"{sel.size} queries of the same stream (every {max(1, n // n_cpu)}-th), {tc:.1f} s of wall time"}
        log(f"cpu oracle: {cpu}")
    scan_ms = kt.scan_ms / max(kt.scan_launches, 1)
    unique_b = kt.scan_unique_bytes / max(kt.scan_launches, 1)
    achieved = unique_b / (scan_ms * 1e-3) / 1e9 if scan_ms > 0 else 0.0
    result = {
        "metric": "queries/sec at recall@k>=0.9 (1 GPU) + list-scan HBM GB/s as % of peak",
        "value": t_sat, "unit": "queries/s", "n_gpus": 1, "steps": int(st.steps), "warmup": 1,
        "ms_per_step": round(st.wall_s * 1e3 / max(st.steps, 1), 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"configs[3] stream: {n} queries, 70% RAG (1M x 768 fp16, nlist 4096, nprobe 32, k U{{10..100}}) + "
                               f"30% cache lookups (200k x 768, nlist 512, nprobe 8, k 1), {slots} slots, {p} lists per query and step",
                   "query_vectors": "host memory (copied at submit, uploaded by the admitting step)"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "kernel": "scan_kernel",
                     "avg_launch_ms": round(scan_ms, 4), "algorithmic_bytes_per_launch": int(unique_b),
                     "note": "at most 1.84 GB of lists per step, smaller than the 256 MB cache only in part: cache-assisted, not an HBM figure"},
        "stream": runs,
        "cpu_baseline": cpu,
        "wall_s_total": round(time.time() - t_start, 1),
    }
    pool.close()
    torch.cuda.empty_cache()
    return result


def graph_bench(args, tri, torch):
    """The paper's own engine (Sec. 3.2) on a config-2-sized corpus: n x 768 fp16 unit-norm points near a
    12-dimensional subspace, inner product, a degree-32 neighbour graph (24 nearest + 8 random rows), 64
    entry points, topM 64, 4 parents per extend, at most 64 extends, k 10.  One bench step = one batch of
    4 * slots device-resident queries from submission to the last result."""
    import graph_inputs
    from paper_2512_02281_amd import graph as tg
    t_start = time.time()
    n, dim, latent, D, n_rand, M, p, iters, k = args.graph_n, 768, 12, 32, 8, args.graph_topm, args.graph_parents, 64, 10
    S = args.graph_slots
    Q = 4 * S
    log(f"workload graph: generating {n} x {dim} fp16 and its degree-{D} neighbour list (untimed)")
    X, Z = graph_inputs.make_points(n, dim, latent, np.float16, graph_inputs.SEED_POINTS, device="cuda")
    Qv, _ = graph_inputs.make_points(Q, dim, latent, np.float16, graph_inputs.SEED_QUERIES, device="cuda")
    G = graph_inputs.make_graph(Z, D, n_rand, graph_inputs.SEED_EDGES, block=1024).to(torch.int32)
    seeds = graph_inputs.entry_points(n, args.graph_seeds)
    torch.cuda.synchronize()
    log(f"inputs ready after {time.time() - t_start:.1f} s")
    pool = tg.GraphPool(X, G, seeds, tri.TRI_F16, slots=S, topm=M, parents=p, max_iters=iters, max_outstanding=2 * Q,
                        groups=args.graph_groups, flags=tri.TRI_FLAG_PROFILE, own_stream=True)
    kk = np.full(Q, k, dtype=np.uint32)
    mm = np.full(Q, tri.TRI_IP, dtype=np.uint32)

    def one_batch():
        return pool.run_all(Qv, kk, mm)

    if args.copy_calibration_mib:
        src = torch.ones(args.copy_calibration_mib << 18, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads and writes copy_calibration_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    log("settling and warm-up")
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < 0.6:
        one_batch()
    for _ in range(args.warmup):
        one_batch()
    pool.kernel_times(reset=True)
    torch.cuda.synchronize()
    log(f"timing {args.steps} batches of {Q} queries")
    t0 = time.perf_counter()
    launches = 0
    for _ in range(args.steps):
        ids, dist, n_out, it, ev, steps = one_batch()
        launches += steps
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    qps = Q * args.steps / total_s
    # The step kernel's own duration: with several groups their launches overlap in time on the GPU, so it is
    # measured on a second pool that steps all slots as one group (same index, same queries, two batches).
    kt_groups = pool.kernel_times()
    pool.close()
    pool = tg.GraphPool(X, G, seeds, tri.TRI_F16, slots=S, topm=M, parents=p, max_iters=iters, max_outstanding=2 * Q,
                        groups=1, flags=tri.TRI_FLAG_PROFILE, own_stream=True)
    one_batch()
    pool.kernel_times(reset=True)
    ids, dist, n_out, it, ev, _ = one_batch()
    kt = pool.kernel_times()
    dist_ms = kt.step_kernel_ms / max(kt.steps, 1)
    bytes_per_launch = kt.tasks * kt.row_bytes / max(kt.steps, 1)
    achieved = bytes_per_launch / (dist_ms * 1e-3) / 1e9 if dist_ms > 0 else 0.0
    log(f"{total_s * 1e3 / args.steps:.3f} ms/batch, {qps:.0f} q/s; {launches / args.steps:.1f} extend steps per batch, "
        f"{total_s * 1e6 / launches:.1f} us per step; step kernel {dist_ms * 1e3:.1f} us/launch for "
        f"{kt.tasks / max(kt.steps, 1):.0f} rows of {kt.row_bytes} B -> {achieved:.0f} GB/s; mean extends {it.mean():.1f}, "
        f"mean distance evaluations {ev.mean():.0f} per query")
    recall = None
    if args.recall_sample:
        rs = np.random.default_rng(77).choice(Q, size=min(args.recall_sample, Q), replace=False)
        hits = 0
        for qi in rs:
            top = torch.topk((X @ Qv[int(qi)]).float(), k).indices.cpu().numpy().tolist()
            hits += len(set(top) & set(ids[qi, :k].tolist()))
        recall = hits / (k * rs.size)
        log(f"recall@{k} on {rs.size} queries: {recall:.4f}")
    cpu = None
    n_cpu = args.cpu_sample if args.cpu_sample >= 0 else 4096
    if n_cpu:
        from oracle import graph_search as gs
        log("CPU oracle (one request at a time, one core) on a sample of the batch")
        Xh, Gh = X.cpu().numpy(), G.cpu().numpy().astype(np.uint32)
        sel = np.arange(0, Q, max(1, Q // n_cpu))[:n_cpu]
        Qh = Qv.cpu().numpy()[sel]
        tc0 = time.perf_counter()
        same = 0
        for j, qi in enumerate(sel):
            r = gs.search(Xh, Gh, seeds, Qh[j], k, M, p, iters, gs.METRIC_IP)
            same += np.array_equal(r["ids"], ids[qi, :k])
        tc = time.perf_counter() - tc0
        cpu = {"value": round(sel.size / tc, 3), "unit": "queries/s", "cores": 1, "kind": "oracle",
               "sample": f"{sel.size} queries of the same batch (every {max(1, Q // n_cpu)}-th), {tc:.1f} s of wall time; "
                         f"{same} of them returned exactly the GPU's ids"}
        log(f"cpu oracle: {cpu}")
    graph_traffic, graph_traffic_prov = (None, None)
    if n == 1_000_000 and S == 8192:
        graph_traffic, graph_traffic_prov = traffic_from_profile("graph_step_kernel.txt", ["graph_engine.hip"])
    result = {
        "metric": "queries/sec at recall@k>=0.9 (1 GPU) + list-scan HBM GB/s as % of peak",
        "value": round(qps, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(total_s * 1e3 / args.steps, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"graph engine (paper Sec. 3.2): {n} x {dim} fp16 near a {latent}-dim subspace, inner product, "
                               f"degree {D} ({D - n_rand} nearest + {n_rand} random), {seeds.size} entry points, topM {M}, {p} parents per "
                               f"extend, at most {iters} extends, k {k}; {S} slots in {args.graph_groups} groups, batches of {Q} queries",
                   "queries_per_step": Q, "extend_steps_per_batch": round(launches / args.steps, 1),
                   "us_per_extend_step": round(total_s * 1e6 / launches, 2),
                   "mean_extends_per_query": round(float(it.mean()), 2), "mean_evaluations_per_query": round(float(ev.mean()), 1),
                   "recall_at_k": None if recall is None else round(recall, 4), "query_vectors": "device-resident"},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": graph_traffic, "traffic_source": graph_traffic_prov, "kernel": "gx_step_kernel",
                     "avg_launch_ms": round(dist_ms, 5), "measured": "all slots stepped as one group (launches do not overlap)",
                     "avg_launch_ms_in_timed_region": round(kt_groups.step_kernel_ms / max(kt_groups.steps, 1), 5),
                     "algorithmic_bytes_per_launch": int(bytes_per_launch),
                     "rows_per_launch": int(kt.tasks / max(kt.steps, 1)), "row_bytes": int(kt.row_bytes),
                     "note": "gathered rows: every distance task reads one 1536-byte row once; the kernel also merges and extends; "
                             "1.5 GB of rows against 256 MB of last-level cache and entry-point rows shared by all requests: "
                             "partly cache-assisted"},
        "cpu_baseline": cpu,
        "wall_s_total": round(time.time() - t_start, 1),
    }
    pool.close()
    return result


def graph_stream_bench(args, tri, torch):
    """The graph engine under arrivals (Sec. 3.2's claim: continuous batching against batches that must drain):
    the graph workload's index, --stream-queries host-resident queries, first all offered at once (saturation),
    then Poisson arrivals at 0.5 x and 0.8 x of the continuous scheme's saturation rate -- each with continuous
    batching and with static batches (a group of slots admits only when all of it has finished)."""
    import graph_inputs
    import workloads
    from paper_2512_02281_amd import graph as tg
    t_start = time.time()
    n, dim, latent, D, n_rand, M, p, iters, k = args.graph_n, 768, 12, 32, 8, args.graph_topm, args.graph_parents, 64, 10
    S, nq = args.graph_slots, args.stream_queries
    log(f"workload graph-stream: generating {n} x {dim} fp16, its degree-{D} neighbour list and {nq} queries (untimed)")
    X, Z = graph_inputs.make_points(n, dim, latent, np.float16, graph_inputs.SEED_POINTS, device="cuda")
    Qv, _ = graph_inputs.make_points(nq, dim, latent, np.float16, graph_inputs.SEED_QUERIES, device="cuda")
    G = graph_inputs.make_graph(Z, D, n_rand, graph_inputs.SEED_EDGES, block=1024).to(torch.int32)
    seeds = graph_inputs.entry_points(n, args.graph_seeds)
    Qh = np.ascontiguousarray(Qv.cpu().numpy())
    torch.cuda.synchronize()
    pool = tg.GraphPool(X, G, seeds, tri.TRI_F16, slots=S, topm=M, parents=p, max_iters=iters, max_outstanding=nq + S,
                        groups=args.graph_groups, own_stream=True)
    pct = lambda a: [round(float(np.percentile(a, x)), 3) for x in (50, 95, 99)]

    def run(arrival, static, label):
        ids, dist, n_out, done_s, st = pool.run_stream(Qh, arrival, k, tri.TRI_IP, static_batches=static)
        lat = (done_s - arrival) * 1e3
        r = {"label": label, "batching": "static batches" if static else "continuous",
             "offered_qps": None if arrival[-1] == 0 else round(nq / arrival[-1], 1),
             "throughput_qps": round(nq / st.wall_s, 1), "steps": int(st.steps),
             "mean_running_slots": round(st.running / max(st.steps, 1), 1), "longest_queue": int(st.max_pending),
             "latency_ms_p50_p95_p99": pct(lat)}
        log(str(r))
        return r, ids

    log("warm-up")
    run(np.zeros(nq), False, "warm-up")
    runs = []
    sat, ids_ref = run(np.zeros(nq), False, "all queries offered at t = 0")
    runs.append(sat)
    r, ids_s = run(np.zeros(nq), True, "all queries offered at t = 0")
    runs.append(r)
    assert np.array_equal(ids_ref, ids_s), "the batching scheme changed a result"
    for frac in (0.5, 0.8):
        arr = workloads.poisson_arrivals(nq, frac * sat["throughput_qps"], 4005)
        for static in (False, True):
            r, ids_x = run(arr, static, f"Poisson arrivals at {frac} x the continuous scheme's saturation rate")
            runs.append(r)
            assert np.array_equal(ids_ref, ids_x), "the batching scheme changed a result"
    result = {
        "metric": "queries/sec at recall@k>=0.9 (1 GPU) + list-scan HBM GB/s as % of peak",
        "value": sat["throughput_qps"], "unit": "queries/s", "n_gpus": 1, "steps": sat["steps"], "warmup": 1,
        "ms_per_step": round(1e3 * nq / sat["throughput_qps"] / max(sat["steps"], 1), 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {"workload": f"graph engine stream: {nq} host-resident queries over {n} x {dim} fp16 (degree {D}, topM {M}, "
                               f"{p} parents per extend, k {k}), {S} slots in {args.graph_groups} groups",
                   "query_vectors": "host memory (copied at arrival, read by the admitting step)"},
        "roofline": None, "stream": runs, "cpu_baseline": None, "wall_s_total": round(time.time() - t_start, 1),
    }
    pool.close()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
