"""GPU tests of the boundary's memory and failure contracts: whose memory a pool and a build use,
how long device-submitted query rows must live, and what a pool is worth after a step failed."""
import ctypes

import numpy as np
import pytest

import workloads
from tests import harness

pytestmark = pytest.mark.gpu


def _small_f16(tri, n_queries=160):
    import torch
    cfg = workloads.CONFIGS[2].scaled(n_base=20_000, n_components=64, nlist=64, n_queries=n_queries)
    base_t, queries_t, rows = workloads.make_config_f16(cfg, device="cuda")
    torch.cuda.synchronize()
    return cfg, base_t, queries_t, base_t.cpu().numpy(), queries_t.cpu().numpy(), rows


def _search_all(tri, pool, idx, queries, k, nprobe):
    q = tri.make_queries(idx, queries, k, nprobe, tri.TRI_IP)
    return harness.run_all(tri, pool, q)


def test_pinned_memory_and_build_scratch_of_the_caller_or_the_library():
    """The same searches through a pool whose pinned host memory and build scratch are the caller's (torch
    tensors) and through one that lets the library allocate them: identical indexes, identical results;
    memory the device cannot address, or too little of it, is refused."""
    import torch
    tri = harness.lib()
    cfg, base_t, queries_t, base, queries, rows = _small_f16(tri)
    k, nprobe = workloads.hetero_params(cfg.n_queries, cfg.seed_params)
    nprobe = np.minimum(nprobe, 32).astype(np.uint32)
    init = base[rows].astype(np.float32)
    out = {}
    for mode in ("caller", "library"):
        with harness.default_pool(tri, slots=64, lists_per_query_step=8, max_dim=cfg.dim, max_nlist=64, max_total_lists=64,
                                  library_memory=mode == "library") as pool:
            assert (pool._pinned is None) == (mode == "library")
            idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 4, centroids=init)
            exported = tri.ivf_export(idx)
            ids, dist, n_out, probes, _ = _search_all(tri, pool, idx, queries, k, nprobe)
            if mode == "caller":
                oidx = harness.oracle_index(tri, idx, base)
                rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, 1, ids, dist, n_out, probes)
                assert rep["checked"] == cfg.n_queries
            out[mode] = (exported, ids, dist, n_out)
    for a, b in zip(out["caller"][0], out["library"][0]):
        assert np.array_equal(a, b)
    for a, b in zip(out["caller"][1:], out["library"][1:]):
        assert np.array_equal(a, b, equal_nan=True)

    # refused: pageable host memory as pinned_ws; too little pinned memory; too little build scratch
    pcfg = tri.tri_pool_cfg(slots=64, items_per_step=1024, lists_per_query_step=0, kmax=16, nprobe_max=16, max_indexes=1,
                            max_total_lists=64, max_nlist=64, max_dim=cfg.dim, max_outstanding=128, coarse_rows=0, flags=0,
                            score_capacity=0, hip_stream=torch.cuda.current_stream().cuda_stream)
    dev_bytes, pinned_bytes = tri.tri_pool_workspace_bytes(pcfg)
    ws = torch.empty(dev_bytes + 256, dtype=torch.uint8, device="cuda")
    pageable = np.zeros(pinned_bytes + 256, dtype=np.uint8)
    with pytest.raises(tri.TriError) as ei:
        tri.tri_pool_create(pcfg, tri._aligned(ws), dev_bytes, (pageable.ctypes.data + 255) // 256 * 256, pinned_bytes)
    assert ei.value.status == tri.TRI_EINVAL
    pinned = torch.empty(pinned_bytes + 256, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(tri.TriError) as ei:
        tri.tri_pool_create(pcfg, tri._aligned(ws), dev_bytes, tri._aligned(pinned), pinned_bytes - 256)
    assert ei.value.status == tri.TRI_ENOMEM
    with pytest.raises(tri.TriError) as ei:
        tri.tri_pool_create(pcfg, tri._aligned(ws), dev_bytes, tri._aligned(pinned) + 8, pinned_bytes)
    assert ei.value.status == tri.TRI_EINVAL
    handle = tri.tri_pool_create(pcfg, tri._aligned(ws), dev_bytes, tri._aligned(pinned), pinned_bytes)
    try:
        params = tri.ivf_params(cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 2, 0)
        need, tmp_need = tri.ivf_build_bytes(params, cfg.n_base), tri.ivf_build_tmp_bytes(params, cfg.n_base, False)
        mem = torch.empty(need + 256, dtype=torch.uint8, device="cuda")
        tmp = torch.empty(tmp_need + 256, dtype=torch.uint8, device="cuda")
        with pytest.raises(tri.TriError) as ei:
            tri.ivf_build(handle, params, base_t.data_ptr(), cfg.n_base, init, tri._aligned(mem), need, tri._aligned(tmp), tmp_need - 256)
        assert ei.value.status == tri.TRI_ENOMEM
        idx = tri.ivf_build(handle, params, base_t.data_ptr(), cfg.n_base, init, tri._aligned(mem), need, tri._aligned(tmp), tmp_need)
        tri.ivf_destroy(idx)
    finally:
        tri.tri_pool_destroy(handle)


def test_device_submitted_rows_may_be_overwritten_once_the_stream_has_passed_the_submit():
    """search_submit_batch_dev copies the rows with a kernel of the pool's stream: work enqueued on that stream
    afterwards may overwrite them.  The free tickets are fragmented first, so the copy runs over many runs of
    store rows, and the source has a pitch wider than a row."""
    import torch
    tri = harness.lib()
    cfg, base_t, queries_t, base, queries, rows = _small_f16(tri, n_queries=300)
    with harness.default_pool(tri, slots=64, lists_per_query_step=4, max_dim=cfg.dim, max_nlist=64, max_total_lists=64,
                              max_outstanding=512) as pool:
        idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 4, centroids=base[rows].astype(np.float32))
        oidx = harness.oracle_index(tri, idx, base)
        # fragment the free tickets: queue 400 host queries, cancel all but every third, drain the rest
        filler = np.ascontiguousarray(np.tile(queries[:100], (4, 1)))
        t, rc = tri.search_submit_batch(pool.handle, tri.make_queries(idx, filler, 1, 1, tri.TRI_IP))
        assert rc == tri.TRI_OK
        for i, tk in enumerate(t):
            if i % 3:
                tri.search_cancel(pool.handle, int(tk))
        keep = t[::3]
        while True:
            st = tri.search_step(pool.handle)
            if st.running == 0 and st.pending_low == 0 and st.items == 0:
                break
        tri.search_sync(pool.handle)
        _, _, _, status = tri.search_poll_batch(pool.handle, keep[::2], 1)      # every other of those stays alive
        assert np.all(status == tri.TRI_OK)
        # the device rows, with a pitch of dim + 24 elements
        wide = torch.zeros(cfg.n_queries, cfg.dim + 24, dtype=torch.float16, device="cuda")
        wide[:, :cfg.dim] = queries_t
        wide[:, cfg.dim:] = 7.0                                                  # must never be read as part of a row
        k = np.full(cfg.n_queries, 10, dtype=np.uint32)
        nprobe = np.full(cfg.n_queries, 8, dtype=np.uint32)
        tickets, rc = tri.search_submit_batch_dev(pool.handle, idx, wide.data_ptr(), (cfg.dim + 24) * 2, cfg.n_queries, k, nprobe,
                                                  tri.TRI_IP)
        assert rc == tri.TRI_OK and tickets.shape[0] == cfg.n_queries
        assert np.any(np.diff(np.sort(tickets & 0xFFFFFFFF).astype(np.int64)) > 1), "the tickets were meant to be fragmented"
        wide.fill_(float("nan"))                                                 # same stream as the pool's: ordered after the copy
        while True:
            st = tri.search_step(pool.handle)
            if st.running == 0 and st.pending_low == 0 and st.items == 0:
                break
        tri.search_sync(pool.handle)
        probes = [tri.search_probes(pool.handle, int(tk), 8) for tk in tickets]
        ids, dist, n_out, status = tri.search_poll_batch(pool.handle, tickets, 10)
        assert np.all(status == tri.TRI_OK)
        rep = harness.compare_with_oracle(oidx, base, queries, k, nprobe, 1, ids, dist, n_out, probes)
        assert rep["checked"] == cfg.n_queries
        # more rows than free tickets: the first ones are queued, TRI_EAGAIN says so
        many = torch.zeros(600, cfg.dim, dtype=torch.float16, device="cuda")
        tickets, rc = tri.search_submit_batch_dev(pool.handle, idx, many.data_ptr(), cfg.dim * 2, 600, 1, 1, tri.TRI_IP)
        assert rc == tri.TRI_EAGAIN and 0 < tickets.shape[0] < 600
        for tk in tickets:
            tri.search_cancel(pool.handle, int(tk))


def test_a_step_that_fails_half_way_marks_the_pool_failed():
    """A failure after admission leaves host and GPU out of step: from then on every call reports the failure,
    and the pool can still be torn down (forced from the host: no kernel misbehaves)."""
    tri = harness.lib()
    cfg, base_t, queries_t, base, queries, rows = _small_f16(tri, n_queries=40)
    with harness.default_pool(tri, slots=16, lists_per_query_step=4, max_dim=cfg.dim, max_nlist=64, max_total_lists=64) as pool:
        idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 2, centroids=base[rows].astype(np.float32))
        q = tri.make_queries(idx, queries, 5, 8, tri.TRI_IP)
        tickets, rc = tri.search_submit_batch(pool.handle, q)
        assert rc == tri.TRI_OK
        tri.search_step(pool.handle)                         # a healthy step first
        tri.tri_pool_inject_failure(pool.handle)
        with pytest.raises(tri.TriError) as ei:
            tri.search_step(pool.handle)
        assert ei.value.status == tri.TRI_EHIP and "injected" in str(ei.value)
        for call in (lambda: tri.search_step(pool.handle), lambda: tri.search_sync(pool.handle),
                     lambda: tri.search_submit_batch(pool.handle, q[:1]),
                     lambda: tri.search_poll(pool.handle, int(tickets[0]), 5),
                     lambda: tri.search_poll_batch(pool.handle, tickets[:2], 5),
                     lambda: pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 0, centroids=base[rows].astype(np.float32))):
            with pytest.raises(tri.TriError) as ei:
                call()
            assert ei.value.status == tri.TRI_EHIP and "failed earlier" in str(ei.value) and "injected" in str(ei.value)
    # (leaving the block destroyed the index and the pool without an error)
    assert pool.handle is None


def test_a_pool_on_its_own_stream_is_not_written_by_work_pending_on_another():
    """The binding takes a pool's device memory as memory of the pool's stream.  Taken on torch's current stream
    instead, a block that a temporary of still-pending kernels had just given back could be handed out, cleared by
    the library on the pool's stream and then written by those kernels: state that starts at zero (the count of
    candidate-region rescans is such a word) would hold their data."""
    import torch
    tri = harness.lib()
    cfg, base_t, queries_t, base, queries, rows = _small_f16(tri, n_queries=64)
    for _ in range(3):
        x = torch.randn(1 << 24, device="cuda")
        for _ in range(8):
            x = x * 1.0001 + 0.04          # every line frees a 64 MiB temporary while its kernel is still queued
        del x
        with harness.default_pool(tri, slots=64, lists_per_query_step=8, max_dim=cfg.dim, max_nlist=64, max_total_lists=64,
                                  own_stream=True) as pool:
            torch.cuda.synchronize()
            assert tri.tri_pool_candidate_rescans(pool.handle) == 0
            idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 2, centroids=base[rows].astype(np.float32))
            ids, dist, n_out, probes, _ = _search_all(tri, pool, idx, queries, 10, 8)
            oidx = harness.oracle_index(tri, idx, base)
            rep = harness.compare_with_oracle(oidx, base, queries, 10, 8, 1, ids, dist, n_out, probes)
            assert rep["checked"] == cfg.n_queries
            assert tri.tri_pool_candidate_rescans(pool.handle) == 0
