"""CPU-only checks of the C-ABI library: it loads, exports every function the header declares,
its structs have the layout the binding assumes, and the host-only entry points validate their
arguments.  No GPU work is launched here."""
import ctypes
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "trinity_ivf.h")


@pytest.fixture(scope="module")
def tri():
    lib_path = os.path.join(ROOT, "paper_2512_02281_amd", "libtrinity_ivf.so")
    if not os.path.exists(lib_path):
        from paper_2512_02281_amd.build import build_library
        build_library()
    import paper_2512_02281_amd as tri
    return tri


def _declared_functions(header=HEADER):
    text = open(header).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*\s*|int\s+)(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_library_exports_every_declared_function(tri):
    declared = _declared_functions()
    assert len(declared) >= 20
    lib = ctypes.CDLL(tri.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    assert sorted(tri.EXPORTS) == declared, "binding and header disagree on the entry points"
    for name in ("ivf_build", "search_submit", "search_step", "search_poll"):
        assert name in declared
    assert "gfx950" in tri.tri_version()


def test_struct_layouts_match_the_header(tri):
    prog = r'''
#include <stdio.h>
#include <stddef.h>
#include "trinity_ivf.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu\n", sizeof(tri_pool_cfg), sizeof(ivf_params), sizeof(tri_query),
         sizeof(tri_step_stats), sizeof(tri_kernel_times));
  printf("%zu %zu %zu\n", sizeof(tri_policy), sizeof(tri_stream_stats), offsetof(tri_policy, flush_timeout_high_s));
  printf("%zu %zu %zu %zu ", sizeof(tri_feedback_cfg), sizeof(tri_feedback_signals), offsetof(tri_feedback_cfg, period_s),
         offsetof(tri_feedback_signals, wait_p95_s));
  printf("%zu %zu %zu %zu\n", offsetof(tri_pool_cfg, score_capacity), offsetof(tri_pool_cfg, hip_stream),
         offsetof(ivf_params, seed), offsetof(tri_query, deadline_ns));
  return 0;
}'''
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "a.c"), os.path.join(tmp, "a.out")
        open(src, "w").write(prog)
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", exe, src])
        out = subprocess.check_output([exe]).decode().split()
    sizes = [int(v) for v in out]
    assert sizes[:5] == [ctypes.sizeof(tri.tri_pool_cfg), ctypes.sizeof(tri.ivf_params), ctypes.sizeof(tri.tri_query),
                         ctypes.sizeof(tri.tri_step_stats), ctypes.sizeof(tri.tri_kernel_times)]
    assert sizes[5:8] == [ctypes.sizeof(tri.tri_policy), ctypes.sizeof(tri.tri_stream_stats),
                          tri.tri_policy.flush_timeout_high_s.offset]
    assert sizes[8:12] == [ctypes.sizeof(tri.tri_feedback_cfg), ctypes.sizeof(tri.tri_feedback_signals),
                           tri.tri_feedback_cfg.period_s.offset, tri.tri_feedback_signals.wait_p95_s.offset]
    assert sizes[12:] == [tri.tri_pool_cfg.score_capacity.offset, tri.tri_pool_cfg.hip_stream.offset,
                         tri.ivf_params.seed.offset, tri.tri_query.deadline_ns.offset]


def _cfg(tri, **over):
    base = dict(slots=64, items_per_step=1024, lists_per_query_step=0, kmax=100, nprobe_max=64, max_indexes=2,
                max_total_lists=2048, max_nlist=1024, max_dim=768, max_outstanding=256, coarse_rows=0, flags=0,
                score_capacity=0)
    base.update(over)
    return tri.tri_pool_cfg(**base)


def test_workspace_size_and_config_validation(tri):
    small, small_pinned = tri.tri_pool_workspace_bytes(_cfg(tri))
    big, big_pinned = tri.tri_pool_workspace_bytes(_cfg(tri, slots=4096, items_per_step=1 << 18, max_outstanding=8192))
    assert 0 < small < big and small % 256 == 0
    # the candidate buffer by default: 1024 pairs per slot and 32 per work item, 8 bytes each
    assert big > (4096 * 1024 + (1 << 18) * 32) * 8
    # pinned host memory: result blocks of the four steps that may be in flight (ids and scores of every slot's
    # kmax results) and a padded row (fp32 rows of max_dim are the widest) per outstanding ticket
    assert small_pinned % 256 == 0 and small_pinned >= 4 * 64 * 2 * 100 * 4 + 256 * 768 * 4
    assert big_pinned >= 4 * 4096 * 2 * 100 * 4 + 8192 * 768 * 4 and big_pinned < 2 * (4 * 4096 * 2 * 100 * 4 + 8192 * 768 * 4) + (64 << 20)
    for bad in (dict(slots=0), dict(items_per_step=0), dict(kmax=0), dict(kmax=2000), dict(nprobe_max=0),
                dict(nprobe_max=5000), dict(max_indexes=0), dict(max_nlist=0), dict(max_total_lists=10),
                dict(max_dim=0), dict(max_dim=4096), dict(max_outstanding=8)):
        with pytest.raises(tri.TriError) as ei:
            tri.tri_pool_workspace_bytes(_cfg(tri, **bad))
        assert ei.value.status == tri.TRI_EINVAL and tri.tri_last_error()


def test_index_size_and_parameter_validation(tri):
    p = tri.ivf_params(768, 1024, tri.TRI_F16, tri.TRI_IP, 10, 1)
    n = 100_000
    got = tri.ivf_build_bytes(p, n)
    assert got >= n * 768 * 2 + n * 8 + 1024 * 768 * 2           # vectors + norms + ids + centroids
    assert got < (n + 32 * 1024) * 768 * 2 * 1.02 + (1 << 20)     # (every list in whole blocks of 32 vectors)
    p32 = tri.ivf_params(100, 16, tri.TRI_F32, tri.TRI_L2, 0, 0)   # dim 100 fp32 pads to 128 elements
    assert tri.ivf_build_bytes(p32, 1000) >= 1000 * 128 * 4
    # temporary memory of a build: a padded copy of the training rows dominates (all rows when n <= 256 nlist),
    # a host-resident base adds its device copy, no training leaves the score block and the assignment tables
    t_dev = tri.ivf_build_tmp_bytes(p, n, False)
    t_host = tri.ivf_build_tmp_bytes(p, n, True)
    p0 = tri.ivf_params(768, 1024, tri.TRI_F16, tri.TRI_IP, 0, 1)
    assert t_dev % 256 == 0 and t_dev >= n * 768 * 2 + n * 4 and 0 <= t_host - t_dev - n * 768 * 2 < 512
    assert tri.ivf_build_tmp_bytes(p0, n, False) <= t_dev - n * 768 * 2
    for bad, nn in ((tri.ivf_params(0, 4, 0, 0, 0, 0), 10), (tri.ivf_params(8, 0, 0, 0, 0, 0), 10),
                    (tri.ivf_params(8, 4, 7, 0, 0, 0), 10), (tri.ivf_params(8, 4, 0, 0, 0, 0), 0),
                    (tri.ivf_params(8, 40, 0, 0, 0, 0), 10), (tri.ivf_params(5000, 4, 1, 0, 0, 0), 10),
                    (tri.ivf_params(8, 4, 0, 0, 0, 0), 1 << 33)):
        with pytest.raises(tri.TriError) as ei:
            tri.ivf_build_bytes(bad, nn)
        assert ei.value.status == tri.TRI_EINVAL
        with pytest.raises(tri.TriError) as ei:
            tri.ivf_build_tmp_bytes(bad, nn, False)
        assert ei.value.status == tri.TRI_EINVAL


def test_admission_split_properties(tri):
    """The reserved-share rule of the step boundary (paper Sec. 3.3): the buffer is filled whenever the two
    queues together can fill it, the high class gets at least its reserved share when it has that many
    waiting, what one class cannot use goes to the other, and nothing is admitted that is not waiting."""
    import numpy as np
    rng = np.random.default_rng(5)
    cases = [(rng.integers(0, 50), rng.integers(0, 80), rng.integers(0, 80), float(rng.choice([0, 0.1, 0.25, 0.5, 0.9, 1])))
             for _ in range(3000)]
    cases += [(10, 100, 100, 0.3), (10, 2, 100, 0.3), (10, 100, 3, 0.3), (0, 5, 5, 0.5), (7, 0, 0, 0.5), (7, 3, 2, 0.5)]
    for n, nh, nl, r in cases:
        n, nh, nl = int(n), int(nh), int(nl)
        th, tl = tri.tri_policy_split(n, nh, nl, r)
        assert th <= nh and tl <= nl and th + tl == min(n, nh + nl)
        reserved = min(n, int(np.ceil(float(np.float32(r)) * n - 1e-4)))
        assert th >= min(nh, reserved)                      # the reserved share, when the high class can use it
        assert tl >= min(nl, n - reserved)                  # the rest, when the low class can use it
    assert tri.tri_policy_split(10, 100, 100, 0.3) == (3, 7)
    assert tri.tri_policy_split(10, 2, 100, 0.3) == (2, 8)      # unused reserved share goes to the low class
    assert tri.tri_policy_split(10, 100, 3, 0.3) == (7, 3)      # unused rest goes to the high class
    assert tri.tri_policy_split(10, 100, 100, 1.0) == (10, 0)   # the default: high class first
    assert tri.tri_policy_split(10, 100, 100, 0.0) == (0, 10)
    with pytest.raises(tri.TriError):
        tri.tri_policy_split(10, 1, 1, 1.5)


def test_slack_order_properties(tri):
    """Least slack first, slack = deadline - (now + steps left * step time): equal step counts reduce to
    earliest deadline first; a later deadline with many steps left can be more urgent; no deadline comes
    last in arrival order; ties keep arrival order."""
    import numpy as np
    none = np.iinfo(np.int64).max
    now, step = 1_000_000, 2_000
    ddl = np.array([now + 50_000, now + 10_000, none, now + 30_000, none, now + 10_000], dtype=np.int64)
    same = np.full(6, 4, dtype=np.uint32)
    assert tri.tri_policy_slack_order(ddl, same, now, step).tolist() == [1, 5, 3, 0, 2, 4]
    # query 0 (deadline +50 us) needs 25 steps of 2 us -> slack 0; query 3 (deadline +30 us) needs 1 -> slack 28 us
    left = np.array([25, 4, 1, 1, 1, 4], dtype=np.uint32)
    assert tri.tri_policy_slack_order(ddl, left, now, step).tolist() == [0, 1, 5, 3, 2, 4]
    # against a plain restatement on random inputs
    rng = np.random.default_rng(8)
    for _ in range(200):
        n = int(rng.integers(1, 40))
        d = np.where(rng.random(n) < 0.2, none, now + rng.integers(-5_000, 100_000, size=n)).astype(np.int64)
        e = rng.integers(1, 30, size=n).astype(np.uint32)
        got = tri.tri_policy_slack_order(d, e, now, step)
        slack = [float("inf") if d[i] == none else int(d[i]) - (now + int(e[i]) * step) for i in range(n)]
        full = sorted(range(n), key=lambda i: (slack[i], i))
        assert got.tolist() == full
        m = int(rng.integers(0, n + 1))                     # only the m most urgent in slack order, the rest by arrival
        assert tri.tri_policy_slack_order(d, e, now, step, m).tolist() == full[:m] + sorted(full[m:])
    assert tri.tri_policy_slack_order(np.zeros(0, np.int64), np.zeros(0, np.uint32), now, step).shape == (0,)


def test_streaming_read_probe_rejects_bad_arguments(tri):
    lib = ctypes.CDLL(tri.LIB_PATH)
    lib.tri_stream_read_bandwidth.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                              ctypes.POINTER(ctypes.c_double)]
    out = ctypes.c_double(0.0)
    assert lib.tri_stream_read_bandwidth(None, 1 << 20, None, None, 1, ctypes.byref(out)) == tri.TRI_EINVAL
    assert lib.tri_stream_read_bandwidth(ctypes.c_void_p(4096), 100, ctypes.c_void_p(4096), None, 1, ctypes.byref(out)) == tri.TRI_EINVAL
    assert lib.tri_stream_read_bandwidth(ctypes.c_void_p(4096), 1 << 20, ctypes.c_void_p(4096), None, 0, ctypes.byref(out)) == tri.TRI_EINVAL
    assert lib.tri_stream_read_bandwidth(ctypes.c_void_p(4100), 1 << 20, ctypes.c_void_p(4096), None, 1, ctypes.byref(out)) == tri.TRI_EINVAL
    assert "aligned" in tri.tri_last_error()


def test_graph_header_exports_layouts_and_validation(tri):
    """include/trinity_graph.h: every declared function is exported and bound, the structs have the layout the
    binding assumes, and the size query validates its arguments (no GPU needed)."""
    from paper_2512_02281_amd import graph as tg
    header = os.path.join(ROOT, "include", "trinity_graph.h")
    declared = _declared_functions(header)
    assert sorted(tg.GRAPH_EXPORTS) == declared
    lib = ctypes.CDLL(tri.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    prog = r'''
#include <stdio.h>
#include <stddef.h>
#include "trinity_graph.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu %u %u\n", sizeof(tri_graph_cfg), sizeof(tri_graph_step_stats), sizeof(tri_graph_times),
         offsetof(tri_graph_cfg, hip_stream), offsetof(tri_graph_times, row_bytes), TRI_GRAPH_TOPM_LIMIT, TRI_GRAPH_TASK_LIMIT);
  return 0;
}'''
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "a.c"), os.path.join(tmp, "a.out")
        open(src, "w").write(prog)
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", exe, src])
        out = [int(v) for v in subprocess.check_output([exe]).decode().split()]
    assert out == [ctypes.sizeof(tg.tri_graph_cfg), ctypes.sizeof(tg.tri_graph_step_stats), ctypes.sizeof(tg.tri_graph_times),
                   tg.tri_graph_cfg.hip_stream.offset, tg.tri_graph_times.row_bytes.offset, tg.TRI_GRAPH_TOPM_LIMIT,
                   tg.TRI_GRAPH_TASK_LIMIT]
    size = ctypes.c_size_t(0)
    ok = tg.tri_graph_cfg(64, 64, 4, 32, 256, 0, 0, 0, None)
    assert lib.graph_pool_bytes(ctypes.byref(ok), 100000, 768, 32, tri.TRI_F16, ctypes.byref(size)) == tri.TRI_OK
    # rows (padded to 256 B), |x|^2, neighbour list and 64 visited tables are in there
    assert size.value >= 100000 * (1536 + 4 + 32 * 4) + 64 * (100000 // 8)
    for bad in (tg.tri_graph_cfg(0, 64, 4, 32, 256, 0, 0, 0, None), tg.tri_graph_cfg(64, 257, 4, 32, 256, 0, 0, 0, None),
                tg.tri_graph_cfg(64, 64, 9, 32, 256, 0, 0, 0, None), tg.tri_graph_cfg(64, 64, 4, 32, 32, 0, 0, 0, None),
                tg.tri_graph_cfg(64, 64, 4, 32, 256, 5, 0, 0, None)):   # groups > 4
        assert lib.graph_pool_bytes(ctypes.byref(bad), 100000, 768, 32, tri.TRI_F16, ctypes.byref(size)) == tri.TRI_EINVAL
    assert lib.graph_pool_bytes(ctypes.byref(ok), 0, 768, 32, tri.TRI_F16, ctypes.byref(size)) == tri.TRI_EINVAL
    assert lib.graph_pool_bytes(ctypes.byref(ok), 1000, 5000, 32, tri.TRI_F16, ctypes.byref(size)) == tri.TRI_EINVAL


def test_feedback_period_matches_the_oracle_rule(tri):
    """tri_policy_feedback (the library's control-loop period, host only) against oracle/control.py on random
    signals, unknown ones included, and its argument checks."""
    import numpy as np
    from oracle import control
    ocfg = control.Config(r_min=0.1, r_max=0.8, r_step=0.05, tau_factor=2.0, tau_min_s=1e-4, tau_max_s=8e-3,
                          u_kv_target=0.9, u_kv_band=0.05, stall_target=0.1, wait_p95_budget_s=2e-3)
    ccfg = tri.tri_feedback_cfg(ocfg.r_min, ocfg.r_max, ocfg.r_step, ocfg.tau_factor, ocfg.tau_min_s, ocfg.tau_max_s,
                                ocfg.u_kv_target, ocfg.u_kv_band, ocfg.stall_target, 0.0, ocfg.wait_p95_budget_s, 0.3)
    rng = np.random.default_rng(5)
    nan = float("nan")
    pick = lambda hi: float(rng.choice([nan, float(np.float32(rng.uniform(0, hi))), 0.0, hi]))
    seen = set()
    for _ in range(3000):
        r, tau = float(np.float32(rng.uniform(0, 1))), float(rng.uniform(0, 1e-2))
        u, st, stp, w = pick(1.0), pick(1.0), pick(1.0), pick(6e-3)
        want_r, want_tau, want_rules = control.period(ocfg, r, tau, u, st, stp, w)
        pol, rules = tri.tri_policy_feedback(ccfg, tri.tri_feedback_signals(u, st, stp, 0.0, w),
                                             tri.tri_policy(r, tri.TRI_ORDER_SLACK, 1e-3, tau))
        assert float(pol.high_share) == want_r and pol.flush_timeout_high_s == want_tau, (r, tau, u, st, stp, w)
        assert {i + 1 for i in range(4) if rules >> i & 1} == want_rules
        assert pol.order_high == tri.TRI_ORDER_SLACK and pol.flush_timeout_s == 1e-3      # untouched
        seen |= want_rules
    assert seen == {1, 2, 3, 4}
    bad = tri.tri_feedback_cfg(0.5, 0.4, 0.05, 2.0, 1e-4, 8e-3, 0.9, 0.05, 0.1, 0.0, 2e-3, 0.3)
    with pytest.raises(Exception):
        tri.tri_policy_feedback(bad, tri.tri_feedback_signals(0.5, 0.1, 0.1, 0.0, 1e-3), tri.tri_policy(0.5, 0, 0.0, 1e-3))


def test_product_path_never_touches_the_oracle():
    """The library sources and the binding must not reference the oracle (no CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2512_02281_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2512_02281_amd" not in text and "trinity_ivf" not in text


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits before touching a device."""
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_pq_header_exports_and_layout(tri):
    """include/trinity_pq.h: every declared function is exported and bound, the parameter struct has the layout the
    binding assumes (no GPU needed: the calls themselves need a resident index)."""
    from paper_2512_02281_amd import pq as tpq
    header = os.path.join(ROOT, "include", "trinity_pq.h")
    declared = _declared_functions(header)
    assert sorted(tpq.PQ_EXPORTS) == declared
    lib = ctypes.CDLL(tri.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in the header but not exported"
    prog = r'''
#include <stdio.h>
#include <stddef.h>
#include "trinity_pq.h"
int main(void) {
  printf("%zu %zu %zu %u %u %u %u\n", sizeof(pq_params), offsetof(pq_params, train_rows), offsetof(pq_params, seed),
         TRI_PQ_KSUB, TRI_PQ_KMAX, TRI_PQ_NPROBE_MAX, TRI_PQ_DSUB_MAX);
  return 0;
}'''
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "a.c"), os.path.join(tmp, "a.out")
        open(src, "w").write(prog)
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", exe, src])
        out = [int(v) for v in subprocess.check_output([exe]).decode().split()]
    assert out == [ctypes.sizeof(tpq.pq_params), tpq.pq_params.train_rows.offset, tpq.pq_params.seed.offset, tpq.TRI_PQ_KSUB,
                   tpq.TRI_PQ_KMAX, tpq.TRI_PQ_NPROBE_MAX, tpq.TRI_PQ_DSUB_MAX]
    size = ctypes.c_size_t(0)
    assert lib.pq_build_bytes(None, None, ctypes.byref(size), ctypes.byref(size)) == tri.TRI_EINVAL
    assert lib.pq_search_bytes(None, 4, ctypes.byref(size)) == tri.TRI_EINVAL
