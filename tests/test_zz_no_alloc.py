"""tri_pool_create_static -- the pool whose device workspace is the library's own static array, for callers
that cannot allocate device memory -- against tri_pool_create: the same index, the same queries, bit-identical
results, on two pools in a row in the same array, the second one smaller (fewer slots, a shorter task array,
fewer queries), so that it runs over what the first one left behind."""
import numpy as np
import pytest

import workloads
from tests import harness

pytestmark = pytest.mark.gpu


def _run(tri, static, cfg_over, base_t, base, rows, cfg, queries, k, nprobe):
    with harness.default_pool(tri, static_workspace=static, **cfg_over) as pool:
        idx = pool.build_index(base_t, cfg.dim, cfg.nlist, tri.TRI_F16, tri.TRI_IP, 3, centroids=base[rows].astype(np.float32))
        exported = tri.ivf_export(idx)
        q = tri.make_queries(idx, queries, k, nprobe, tri.TRI_IP)
        ids, dist, n_out, probes, stats = harness.run_all(tri, pool, q)
        oidx = harness.oracle_index(tri, idx, base) if static else None
    return exported, ids, dist, n_out, probes, len(stats), oidx


def test_static_workspace_pool_matches_a_pool_in_caller_memory_twice_in_a_row():
    import torch
    tri = harness.lib()
    cfg = workloads.CONFIGS[2].scaled(n_base=20_000, n_components=64, nlist=64, n_queries=240)
    base_t, queries_t, rows = workloads.make_config_f16(cfg, device="cuda")
    torch.cuda.synchronize()
    base, queries = base_t.cpu().numpy(), queries_t.cpu().numpy()
    k, nprobe = workloads.hetero_params(cfg.n_queries, cfg.seed_params)
    nprobe = np.minimum(nprobe, 32).astype(np.uint32)
    first = dict(slots=64, items_per_step=2048, lists_per_query_step=8, kmax=128, nprobe_max=32, max_indexes=1,
                 max_total_lists=64, max_nlist=64, max_dim=cfg.dim, max_outstanding=1024, score_capacity=4 << 20)
    second = dict(first, slots=24, items_per_step=512, lists_per_query_step=4, max_outstanding=256, score_capacity=1 << 20)
    for over, nq in ((first, 240), (second, 90)):
        got = _run(tri, True, over, base_t, base, rows, cfg, queries[:nq], k[:nq], nprobe[:nq])
        want = _run(tri, False, over, base_t, base, rows, cfg, queries[:nq], k[:nq], nprobe[:nq])
        for a, b in zip(got[0], want[0]):
            assert np.array_equal(a, b), "the two pools built different indexes"
        assert got[5] == want[5]                                     # the same number of steps
        assert np.array_equal(got[1], want[1]), "ids differ"
        assert np.array_equal(got[2], want[2], equal_nan=True), "scores differ"
        assert np.array_equal(got[3], want[3])
        for a, b in zip(got[4], want[4]):
            assert np.array_equal(a, b), "probe lists differ"
        # and both are right: the static pool's results against the oracle
        rep = harness.compare_with_oracle(got[6], base, queries[:nq], k[:nq], nprobe[:nq], 1, got[1], got[2], got[3], got[4])
        assert rep["checked"] == nq


def test_static_workspace_limits_are_reported():
    import torch
    tri = harness.lib()
    small = dict(slots=16, items_per_step=256, lists_per_query_step=0, kmax=16, nprobe_max=16, max_indexes=1, max_total_lists=64,
                 max_nlist=64, max_dim=128, max_outstanding=64, coarse_rows=0, flags=0, score_capacity=1 << 18,
                 hip_stream=torch.cuda.current_stream().cuda_stream)
    cfg = tri.tri_pool_cfg(**small)
    _, pinned_bytes = tri.tri_pool_workspace_bytes(cfg)
    pinned = torch.empty(pinned_bytes + 256, dtype=torch.uint8, pin_memory=True)
    # a configuration beyond the static array: refused with its size, nothing created
    big = tri.tri_pool_cfg(**dict(small, score_capacity=32 << 20))
    need, big_pinned = tri.tri_pool_workspace_bytes(big)
    assert need > tri.TRI_STATIC_WS_BYTES
    big_pin = torch.empty(big_pinned + 256, dtype=torch.uint8, pin_memory=True)
    with pytest.raises(tri.TriError) as ei:
        tri.tri_pool_create_static(big, tri._aligned(big_pin), big_pinned)
    assert ei.value.status == tri.TRI_ENOMEM and str(need) in str(ei.value)
    # no pinned memory, no pool: this call never allocates any
    with pytest.raises(tri.TriError) as ei:
        tri.tri_pool_create_static(cfg, None, 0)
    assert ei.value.status == tri.TRI_EINVAL
    # one pool at a time per device
    a = tri.tri_pool_create_static(cfg, tri._aligned(pinned), pinned_bytes)
    try:
        pinned2 = torch.empty(pinned_bytes + 256, dtype=torch.uint8, pin_memory=True)
        with pytest.raises(tri.TriError) as ei:
            tri.tri_pool_create_static(cfg, tri._aligned(pinned2), pinned_bytes)
        assert ei.value.status == tri.TRI_EAGAIN
    finally:
        tri.tri_pool_destroy(a)
    b = tri.tri_pool_create_static(cfg, tri._aligned(pinned), pinned_bytes)      # free again after the destroy
    tri.tri_pool_destroy(b)
