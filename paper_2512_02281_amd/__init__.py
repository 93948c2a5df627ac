"""Thin Python binding of the MI355X vector-search pool library (argument marshalling only).

Every function here has the name of the C entry point it forwards to (include/trinity_ivf.h);
every step of the search path runs in the library's HIP kernels.  PyTorch appears only as the
owner of device memory (workspaces, index storage) and of the stream.  There is no fallback: if
the shared library has not been built, importing this package raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

TRI_OK, TRI_EINVAL, TRI_ENOMEM, TRI_EAGAIN, TRI_EHIP, TRI_ENOENT = 0, -1, -2, -3, -4, -5
TRI_L2, TRI_IP = 0, 1
TRI_F32, TRI_F16 = 0, 1
TRI_CLASS_HIGH, TRI_CLASS_LOW = 0, 1
TRI_FLAG_PROFILE, TRI_FLAG_KEEP_PROBES, TRI_FLAG_PROFILE_SCAN, TRI_FLAG_GRAPH, TRI_FLAG_STREAM_LISTS = 1, 2, 4, 8, 16
TRI_ORDER_FIFO, TRI_ORDER_SLACK = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtrinity_ivf.so")


class TriError(RuntimeError):
    def __init__(self, status: int, where: str, text: str):
        super().__init__(f"{where} -> status {status}: {text}")
        self.status = status


class tri_pool_cfg(ctypes.Structure):
    _fields_ = [("slots", ctypes.c_uint32), ("items_per_step", ctypes.c_uint32),
                ("lists_per_query_step", ctypes.c_uint32), ("kmax", ctypes.c_uint32),
                ("nprobe_max", ctypes.c_uint32), ("max_indexes", ctypes.c_uint32),
                ("max_total_lists", ctypes.c_uint32), ("max_nlist", ctypes.c_uint32),
                ("max_dim", ctypes.c_uint32), ("max_outstanding", ctypes.c_uint32),
                ("coarse_rows", ctypes.c_uint32), ("flags", ctypes.c_uint32),
                ("score_capacity", ctypes.c_uint64), ("hip_stream", ctypes.c_void_p)]


class ivf_params(ctypes.Structure):
    _fields_ = [("dim", ctypes.c_uint32), ("nlist", ctypes.c_uint32), ("dtype", ctypes.c_uint32),
                ("build_metric", ctypes.c_uint32), ("train_iters", ctypes.c_uint32),
                ("seed", ctypes.c_uint64)]


class tri_query(ctypes.Structure):
    _fields_ = [("index", ctypes.c_void_p), ("vec", ctypes.c_void_p), ("k", ctypes.c_uint32),
                ("nprobe", ctypes.c_uint32), ("metric", ctypes.c_uint32), ("klass", ctypes.c_uint32),
                ("deadline_ns", ctypes.c_uint64), ("user_tag", ctypes.c_uint64)]


# numpy view of the same struct, for building many queries without a Python loop
QUERY_DTYPE = np.dtype([("index", np.uint64), ("vec", np.uint64), ("k", np.uint32), ("nprobe", np.uint32),
                        ("metric", np.uint32), ("klass", np.uint32), ("deadline_ns", np.uint64),
                        ("user_tag", np.uint64)], align=True)
assert QUERY_DTYPE.itemsize == ctypes.sizeof(tri_query)


class tri_step_stats(ctypes.Structure):
    _fields_ = [("step", ctypes.c_uint64), ("admitted", ctypes.c_uint32), ("retired", ctypes.c_uint32),
                ("running", ctypes.c_uint32), ("items", ctypes.c_uint32), ("capacity", ctypes.c_uint32),
                ("pending_high", ctypes.c_uint32), ("pending_low", ctypes.c_uint32),
                ("finished", ctypes.c_uint32)]


class tri_kernel_times(ctypes.Structure):
    _fields_ = [("steps", ctypes.c_uint64), ("admit_ms", ctypes.c_double), ("coarse_ms", ctypes.c_double),
                ("pack_ms", ctypes.c_double), ("sample_ms", ctypes.c_double), ("threshold_ms", ctypes.c_double),
                ("scan_ms", ctypes.c_double), ("select_ms", ctypes.c_double),
                ("scan_launches", ctypes.c_uint64), ("scan_vector_bytes", ctypes.c_uint64),
                ("scan_unique_bytes", ctypes.c_uint64), ("scan_items", ctypes.c_uint64), ("scan_list_bytes", ctypes.c_uint64)]


class tri_policy(ctypes.Structure):
    _fields_ = [("high_share", ctypes.c_float), ("order_high", ctypes.c_uint32),
                ("flush_timeout_s", ctypes.c_double), ("flush_timeout_high_s", ctypes.c_double),
                ("static_batches", ctypes.c_uint32), ("pad_", ctypes.c_uint32)]


class tri_feedback_cfg(ctypes.Structure):
    _fields_ = [("r_min", ctypes.c_float), ("r_max", ctypes.c_float), ("r_step", ctypes.c_float),
                ("tau_factor", ctypes.c_float), ("tau_min_s", ctypes.c_double), ("tau_max_s", ctypes.c_double),
                ("u_kv_target", ctypes.c_float), ("u_kv_band", ctypes.c_float), ("stall_target", ctypes.c_float),
                ("pad_", ctypes.c_float), ("wait_p95_budget_s", ctypes.c_double), ("period_s", ctypes.c_double)]


class tri_feedback_signals(ctypes.Structure):
    _fields_ = [("u_kv", ctypes.c_float), ("decode_stall", ctypes.c_float), ("decode_stall_prev", ctypes.c_float),
                ("pad_", ctypes.c_float), ("wait_p95_s", ctypes.c_double)]


class tri_stream_stats(ctypes.Structure):
    _fields_ = [("wall_s", ctypes.c_double), ("steps", ctypes.c_uint64), ("items", ctypes.c_uint64),
                ("capacity", ctypes.c_uint64), ("running", ctypes.c_uint64), ("max_pending", ctypes.c_uint64),
                ("submit_s", ctypes.c_double), ("step_s", ctypes.c_double), ("collect_s", ctypes.c_double)]


EXPORTS = ["tri_pool_workspace_bytes", "tri_pool_create", "tri_pool_create_static", "tri_pool_destroy", "ivf_build_bytes", "ivf_build_tmp_bytes", "ivf_build",
           "ivf_export", "ivf_info", "ivf_destroy", "search_submit", "search_submit_batch", "search_submit_batch_dev",
           "search_step", "search_poll", "search_poll_batch", "search_probes", "search_cancel", "search_sync",
           "search_run_stream", "search_set_policy", "search_get_policy", "tri_policy_split", "tri_policy_slack_order",
           "tri_policy_feedback", "search_set_feedback", "search_report_signals", "search_get_feedback",
           "tri_pool_kernel_times", "tri_pool_set_profiling", "tri_pool_set_replay", "tri_stream_read_bandwidth",
           "tri_pool_inject_failure", "tri_pool_set_candidate_reserve", "tri_pool_candidate_rescans", "tri_last_error", "tri_version"]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'); "
                          "this package has no fallback path")
    # PyTorch supplies the device memory and the stream this library works on, so both must talk to the
    # same HIP runtime instance: let torch load its runtime first, the library then binds to that one.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t
    P = ctypes.POINTER
    lib.tri_pool_workspace_bytes.argtypes = [P(tri_pool_cfg), P(sz), P(sz)]
    lib.tri_pool_create.argtypes = [P(tri_pool_cfg), vp, sz, vp, sz, P(vp)]
    lib.tri_pool_create_static.argtypes = [P(tri_pool_cfg), vp, sz, P(vp)]
    lib.tri_pool_inject_failure.argtypes = [vp]
    lib.tri_pool_set_candidate_reserve.argtypes = [vp, u32]
    lib.tri_pool_candidate_rescans.argtypes = [vp, P(u64)]
    lib.tri_pool_destroy.argtypes = [vp]
    lib.ivf_build_bytes.argtypes = [P(ivf_params), u64, P(sz)]
    lib.ivf_build_tmp_bytes.argtypes = [P(ivf_params), u64, ctypes.c_int, P(sz)]
    lib.ivf_build.argtypes = [vp, P(ivf_params), vp, u64, vp, vp, sz, vp, sz, P(vp)]
    lib.ivf_export.argtypes = [vp, vp, vp, vp]
    lib.ivf_info.argtypes = [vp, P(u64), P(u32), P(u32), P(u32), P(u32)]
    lib.ivf_destroy.argtypes = [vp]
    lib.search_submit.argtypes = [vp, P(tri_query), P(u64)]
    lib.search_submit_batch.argtypes = [vp, vp, u32, vp, P(u32)]
    lib.search_submit_batch_dev.argtypes = [vp, vp, vp, u64, u32, vp, vp, vp, vp, vp, P(u32)]
    lib.search_step.argtypes = [vp, P(tri_step_stats)]
    lib.search_poll.argtypes = [vp, u64, P(u32), vp, vp]
    lib.search_poll_batch.argtypes = [vp, vp, u32, u32, vp, vp, vp, vp]
    lib.search_probes.argtypes = [vp, u64, vp, P(u32)]
    lib.search_cancel.argtypes = [vp, u64]
    lib.search_sync.argtypes = [vp]
    lib.search_run_stream.argtypes = [vp, vp, vp, u32, u32, u32, vp, vp, vp, vp, vp, P(tri_stream_stats)]
    lib.search_set_policy.argtypes = [vp, P(tri_policy)]
    lib.search_get_policy.argtypes = [vp, P(tri_policy), P(ctypes.c_double)]
    lib.tri_policy_split.argtypes = [u32, u32, u32, ctypes.c_float, P(u32), P(u32)]
    lib.tri_policy_slack_order.argtypes = [u32, vp, vp, ctypes.c_int64, ctypes.c_int64, u32, vp]
    lib.tri_policy_feedback.argtypes = [P(tri_feedback_cfg), P(tri_feedback_signals), P(tri_policy), P(u32)]
    lib.search_set_feedback.argtypes = [vp, P(tri_feedback_cfg)]
    lib.search_report_signals.argtypes = [vp, ctypes.c_float, ctypes.c_float]
    lib.search_get_feedback.argtypes = [vp, P(u64), P(tri_feedback_signals)]
    lib.tri_pool_kernel_times.argtypes = [vp, P(tri_kernel_times), ctypes.c_int]
    lib.tri_pool_set_profiling.argtypes = [vp, u32]
    lib.tri_pool_set_replay.argtypes = [vp, ctypes.c_int]
    lib.tri_stream_read_bandwidth.argtypes = [vp, sz, vp, vp, u32, P(ctypes.c_double)]
    lib.tri_last_error.restype = ctypes.c_char_p
    lib.tri_version.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name not in ("tri_last_error", "tri_version"):
            getattr(lib, name).restype = ctypes.c_int
    return lib


_lib = _load()


def tri_last_error() -> str:
    return _lib.tri_last_error().decode()


def tri_version() -> str:
    return _lib.tri_version().decode()


def _check(rc: int, where: str, ok=(TRI_OK,)) -> int:
    if rc not in ok:
        raise TriError(rc, where, tri_last_error())
    return rc


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


# ------------------------------------------------------------------------------------------- pool
def tri_pool_workspace_bytes(cfg: tri_pool_cfg):
    """(device workspace bytes, pinned host bytes) a pool with this configuration needs."""
    dev, pinned = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(_lib.tri_pool_workspace_bytes(ctypes.byref(cfg), ctypes.byref(dev), ctypes.byref(pinned)), "tri_pool_workspace_bytes")
    return int(dev.value), int(pinned.value)


def tri_pool_create(cfg: tri_pool_cfg, dev_ws_ptr: int, dev_ws_bytes: int, pinned_ptr: Optional[int] = None,
                    pinned_bytes: int = 0) -> int:
    """pinned_ptr None: the library allocates the pinned host memory itself."""
    out = ctypes.c_void_p(None)
    _check(_lib.tri_pool_create(ctypes.byref(cfg), ctypes.c_void_p(dev_ws_ptr), dev_ws_bytes, ctypes.c_void_p(pinned_ptr),
                                pinned_bytes, ctypes.byref(out)), "tri_pool_create")
    return out.value


TRI_STATIC_WS_BYTES = 64 << 20


def tri_pool_create_static(cfg: tri_pool_cfg, pinned_ptr: int, pinned_bytes: int) -> int:
    """A pool whose device workspace is the library's own static array (no device allocation anywhere)."""
    out = ctypes.c_void_p(None)
    _check(_lib.tri_pool_create_static(ctypes.byref(cfg), ctypes.c_void_p(pinned_ptr), pinned_bytes, ctypes.byref(out)),
           "tri_pool_create_static")
    return out.value


def tri_pool_set_candidate_reserve(pool: int, pairs: int) -> None:
    _check(_lib.tri_pool_set_candidate_reserve(ctypes.c_void_p(pool), pairs), "tri_pool_set_candidate_reserve")


def tri_pool_candidate_rescans(pool: int) -> int:
    out = ctypes.c_uint64(0)
    _check(_lib.tri_pool_candidate_rescans(ctypes.c_void_p(pool), ctypes.byref(out)), "tri_pool_candidate_rescans")
    return int(out.value)


def tri_pool_inject_failure(pool: int) -> None:
    _check(_lib.tri_pool_inject_failure(ctypes.c_void_p(pool)), "tri_pool_inject_failure")


def tri_pool_destroy(pool: int) -> None:
    _check(_lib.tri_pool_destroy(ctypes.c_void_p(pool)), "tri_pool_destroy")


def tri_pool_set_profiling(pool: int, flags: int) -> None:
    _check(_lib.tri_pool_set_profiling(ctypes.c_void_p(pool), flags), "tri_pool_set_profiling")


def tri_stream_read_bandwidth(buf, repeats: int = 10) -> float:
    """GB/s of a plain streaming read of the torch cuda tensor `buf` (on the current stream)."""
    import torch
    sink = torch.zeros(1, dtype=torch.int32, device=buf.device)
    out = ctypes.c_double(0.0)
    torch.cuda.synchronize()
    _check(_lib.tri_stream_read_bandwidth(ctypes.c_void_p(buf.data_ptr()), buf.numel() * buf.element_size(),
                                          ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream),
                                          repeats, ctypes.byref(out)), "tri_stream_read_bandwidth")
    return float(out.value)


def tri_pool_set_replay(pool: int, on: bool) -> None:
    _check(_lib.tri_pool_set_replay(ctypes.c_void_p(pool), 1 if on else 0), "tri_pool_set_replay")


def tri_pool_kernel_times(pool: int, reset: bool = False) -> tri_kernel_times:
    out = tri_kernel_times()
    _check(_lib.tri_pool_kernel_times(ctypes.c_void_p(pool), ctypes.byref(out), int(reset)), "tri_pool_kernel_times")
    return out


# ------------------------------------------------------------------------------------------- index
def ivf_build_bytes(params: ivf_params, n: int) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib.ivf_build_bytes(ctypes.byref(params), n, ctypes.byref(out)), "ivf_build_bytes")
    return int(out.value)


def ivf_build_tmp_bytes(params: ivf_params, n: int, base_on_host: bool) -> int:
    out = ctypes.c_size_t(0)
    _check(_lib.ivf_build_tmp_bytes(ctypes.byref(params), n, int(base_on_host), ctypes.byref(out)), "ivf_build_tmp_bytes")
    return int(out.value)


def ivf_build(pool: int, params: ivf_params, base_ptr: int, n: int, centroids: Optional[np.ndarray],
              dev_mem_ptr: int, dev_mem_bytes: int, tmp_ptr: Optional[int] = None, tmp_bytes: int = 0) -> int:
    """base_ptr: host or device address of the row-major n x dim base (of params.dtype).  tmp_ptr None: the
    library allocates (and frees) its temporary device memory itself."""
    if centroids is not None:
        centroids = np.ascontiguousarray(centroids, dtype=np.float32)
        assert centroids.shape == (params.nlist, params.dim)
    out = ctypes.c_void_p(None)
    _check(_lib.ivf_build(ctypes.c_void_p(pool), ctypes.byref(params), ctypes.c_void_p(base_ptr), n,
                          _np_ptr(centroids), ctypes.c_void_p(dev_mem_ptr), dev_mem_bytes, ctypes.c_void_p(tmp_ptr), tmp_bytes,
                          ctypes.byref(out)),
           "ivf_build")
    return out.value


def ivf_info(index: int) -> dict:
    n, dim, nlist, dtype, mx = ctypes.c_uint64(), ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint32(), ctypes.c_uint32()
    _check(_lib.ivf_info(ctypes.c_void_p(index), ctypes.byref(n), ctypes.byref(dim), ctypes.byref(nlist),
                         ctypes.byref(dtype), ctypes.byref(mx)), "ivf_info")
    return dict(n=int(n.value), dim=int(dim.value), nlist=int(nlist.value), dtype=int(dtype.value),
                max_list_len=int(mx.value))


def ivf_export(index: int):
    """(centroids fp32 [nlist, dim], list_off uint64 [nlist+1], list_ids int64 [n])."""
    info = ivf_info(index)
    cent = np.empty((info["nlist"], info["dim"]), dtype=np.float32)
    off = np.empty(info["nlist"] + 1, dtype=np.uint64)
    ids = np.empty(info["n"], dtype=np.int64)
    _check(_lib.ivf_export(ctypes.c_void_p(index), _np_ptr(cent), _np_ptr(off), _np_ptr(ids)), "ivf_export")
    return cent, off, ids


def ivf_destroy(index: int) -> None:
    _check(_lib.ivf_destroy(ctypes.c_void_p(index)), "ivf_destroy")


# ------------------------------------------------------------------------------------------- search
def search_submit(pool: int, index: int, vec: np.ndarray, k: int, nprobe: int, metric: int,
                  klass: int = TRI_CLASS_LOW, deadline_ns: int = 0, user_tag: int = 0) -> int:
    vec = np.ascontiguousarray(vec)
    q = tri_query(index, vec.ctypes.data, k, nprobe, metric, klass, deadline_ns, user_tag)
    out = ctypes.c_uint64(0)
    _check(_lib.search_submit(ctypes.c_void_p(pool), ctypes.byref(q), ctypes.byref(out)), "search_submit")
    return int(out.value)


def make_queries(index, vecs: np.ndarray, k, nprobe, metric, klass=TRI_CLASS_LOW, deadline_ns=0) -> np.ndarray:
    """An array of tri_query records over the rows of `vecs` (which must stay alive until submitted).
    index / k / nprobe / metric / klass: scalars or per-row arrays."""
    assert vecs.flags["C_CONTIGUOUS"] and vecs.ndim == 2
    n = vecs.shape[0]
    q = np.zeros(n, dtype=QUERY_DTYPE)
    q["index"] = index
    q["vec"] = vecs.ctypes.data + np.arange(n, dtype=np.uint64) * np.uint64(vecs.strides[0])
    q["k"], q["nprobe"], q["metric"], q["klass"] = k, nprobe, metric, klass
    q["deadline_ns"] = deadline_ns
    return q


def search_submit_batch(pool: int, queries: np.ndarray):
    """queries: array of QUERY_DTYPE.  Returns (tickets uint64 [n_done], status).  status TRI_EAGAIN
    means only the first n_done were queued."""
    assert queries.dtype == QUERY_DTYPE and queries.flags["C_CONTIGUOUS"]
    n = queries.shape[0]
    tickets = np.zeros(n, dtype=np.uint64)
    done = ctypes.c_uint32(0)
    rc = _lib.search_submit_batch(ctypes.c_void_p(pool), _np_ptr(queries), n, _np_ptr(tickets), ctypes.byref(done))
    _check(rc, "search_submit_batch", ok=(TRI_OK, TRI_EAGAIN))
    return tickets[:done.value], rc


def search_submit_batch_dev(pool: int, index: int, vecs_ptr: int, pitch_bytes: int, n: int, k, nprobe, metric,
                            klass=TRI_CLASS_LOW):
    """Queries whose vectors already live in device memory (vecs_ptr: device address of n rows).
    k / nprobe / metric / klass: scalars or arrays of n.  Returns (tickets, status)."""
    arrs = [np.ascontiguousarray(np.broadcast_to(np.asarray(a, dtype=np.uint32), (n,))) for a in (k, nprobe, metric, klass)]
    tickets = np.zeros(n, dtype=np.uint64)
    done = ctypes.c_uint32(0)
    rc = _lib.search_submit_batch_dev(ctypes.c_void_p(pool), ctypes.c_void_p(index), ctypes.c_void_p(vecs_ptr),
                                      pitch_bytes, n, _np_ptr(arrs[0]), _np_ptr(arrs[1]), _np_ptr(arrs[2]),
                                      _np_ptr(arrs[3]), _np_ptr(tickets), ctypes.byref(done))
    _check(rc, "search_submit_batch_dev", ok=(TRI_OK, TRI_EAGAIN))
    return tickets[:done.value], rc


def search_step(pool: int, stats: Optional[tri_step_stats] = None) -> tri_step_stats:
    st = stats if stats is not None else tri_step_stats()
    _check(_lib.search_step(ctypes.c_void_p(pool), ctypes.byref(st)), "search_step")
    return st


def search_poll(pool: int, ticket: int, k: int):
    """None while the query is not finished, else (ids int64 [k], dist fp32 [k], n_out)."""
    ids = np.empty(k, dtype=np.int64)
    dist = np.empty(k, dtype=np.float32)
    n = ctypes.c_uint32(0)
    rc = _lib.search_poll(ctypes.c_void_p(pool), ticket, ctypes.byref(n), _np_ptr(ids), _np_ptr(dist))
    if rc == TRI_EAGAIN:
        return None
    _check(rc, "search_poll")
    return ids, dist, int(n.value)


def search_poll_batch(pool: int, tickets: np.ndarray, stride: int):
    """(ids int64 [n, stride], dist fp32 [n, stride], n_out uint32 [n], status int32 [n])."""
    tickets = np.ascontiguousarray(tickets, dtype=np.uint64)
    n = tickets.shape[0]
    ids = np.full((n, stride), -1, dtype=np.int64)          # entries past a query's own k stay -1 / nan
    dist = np.full((n, stride), np.nan, dtype=np.float32)
    n_out = np.zeros(n, dtype=np.uint32)
    status = np.zeros(n, dtype=np.int32)
    rc = _lib.search_poll_batch(ctypes.c_void_p(pool), _np_ptr(tickets), n, stride, _np_ptr(n_out), _np_ptr(ids),
                                _np_ptr(dist), _np_ptr(status))
    if rc < 0:
        _check(rc, "search_poll_batch")
    return ids, dist, n_out, status


def search_probes(pool: int, ticket: int, nprobe: int) -> Optional[np.ndarray]:
    lists = np.empty(nprobe, dtype=np.uint32)
    n = ctypes.c_uint32(0)
    rc = _lib.search_probes(ctypes.c_void_p(pool), ticket, _np_ptr(lists), ctypes.byref(n))
    if rc == TRI_EAGAIN:
        return None
    _check(rc, "search_probes")
    return lists[:n.value]


def search_cancel(pool: int, ticket: int) -> None:
    _check(_lib.search_cancel(ctypes.c_void_p(pool), ticket), "search_cancel")


def search_sync(pool: int) -> None:
    _check(_lib.search_sync(ctypes.c_void_p(pool)), "search_sync")


def search_set_policy(pool: int, high_share: float = 1.0, order_high: int = TRI_ORDER_FIFO,
                      flush_timeout_s: float = 0.0, flush_timeout_high_s: float = 0.0, static_batches: bool = False) -> None:
    pol = tri_policy(high_share, order_high, flush_timeout_s, flush_timeout_high_s, 1 if static_batches else 0, 0)
    _check(_lib.search_set_policy(ctypes.c_void_p(pool), ctypes.byref(pol)), "search_set_policy")


def search_get_policy(pool: int):
    """(tri_policy, mean step duration in seconds)."""
    pol, t = tri_policy(), ctypes.c_double(0.0)
    _check(_lib.search_get_policy(ctypes.c_void_p(pool), ctypes.byref(pol), ctypes.byref(t)), "search_get_policy")
    return pol, float(t.value)


def tri_policy_feedback(cfg: tri_feedback_cfg, signals: tri_feedback_signals, policy: tri_policy):
    """One period of the control loop: returns (new tri_policy, bit mask of the rules that applied)."""
    out = tri_policy(policy.high_share, policy.order_high, policy.flush_timeout_s, policy.flush_timeout_high_s,
                     policy.static_batches, 0)
    rules = ctypes.c_uint32(0)
    _check(_lib.tri_policy_feedback(ctypes.byref(cfg), ctypes.byref(signals), ctypes.byref(out), ctypes.byref(rules)),
           "tri_policy_feedback")
    return out, int(rules.value)


def search_set_feedback(pool: int, cfg: Optional[tri_feedback_cfg]) -> None:
    _check(_lib.search_set_feedback(ctypes.c_void_p(pool), ctypes.byref(cfg) if cfg is not None else None),
           "search_set_feedback")


def search_report_signals(pool: int, u_kv: float, decode_stall: float) -> None:
    _check(_lib.search_report_signals(ctypes.c_void_p(pool), u_kv, decode_stall), "search_report_signals")


def search_get_feedback(pool: int):
    """(periods applied, tri_feedback_signals of the last period)."""
    n, last = ctypes.c_uint64(0), tri_feedback_signals()
    _check(_lib.search_get_feedback(ctypes.c_void_p(pool), ctypes.byref(n), ctypes.byref(last)), "search_get_feedback")
    return int(n.value), last


def tri_policy_split(free_slots: int, n_high: int, n_low: int, high_share: float):
    """(take_high, take_low): the admission split search_step applies at a step boundary."""
    a, b = ctypes.c_uint32(0), ctypes.c_uint32(0)
    _check(_lib.tri_policy_split(free_slots, n_high, n_low, high_share, ctypes.byref(a), ctypes.byref(b)), "tri_policy_split")
    return int(a.value), int(b.value)


def tri_policy_slack_order(deadline_ns, steps_left, now_ns: int, step_ns: int, m: Optional[int] = None) -> np.ndarray:
    """The m (default: all) indices of least slack by ascending slack (deadline INT64_MAX = none), then the
    other indices ascending: the order search_step applies when it admits m high-class queries."""
    deadline_ns = np.ascontiguousarray(deadline_ns, dtype=np.int64)
    steps_left = np.ascontiguousarray(steps_left, dtype=np.uint32)
    order = np.zeros(deadline_ns.shape[0], dtype=np.uint32)
    n = deadline_ns.shape[0]
    _check(_lib.tri_policy_slack_order(n, _np_ptr(deadline_ns), _np_ptr(steps_left), now_ns, step_ns,
                                       n if m is None else m, _np_ptr(order)), "tri_policy_slack_order")
    return order


def search_run_stream(pool: int, queries: np.ndarray, arrival_s: np.ndarray, stride: int, depth: int = 0,
                      nprobe_max: int = 0):
    """Drive the pool through a stream (queries: QUERY_DTYPE array, arrival_s: seconds, not decreasing).
    Returns (ids int64 [n, stride], dist fp32 [n, stride], n_out uint32 [n], done_s float64 [n], stats,
    probes uint32 [n, nprobe_max] or None -- asked for by passing the pool's nprobe_max)."""
    assert queries.dtype == QUERY_DTYPE and queries.flags["C_CONTIGUOUS"]
    arrival_s = np.ascontiguousarray(arrival_s, dtype=np.float64)
    n = queries.shape[0]
    assert arrival_s.shape == (n,)
    ids = np.full((n, stride), -1, dtype=np.int64)
    dist = np.full((n, stride), np.nan, dtype=np.float32)
    n_out = np.zeros(n, dtype=np.uint32)
    done_s = np.zeros(n, dtype=np.float64)
    stats = tri_stream_stats()
    probes = np.zeros((n, nprobe_max), dtype=np.uint32) if nprobe_max else None
    _check(_lib.search_run_stream(ctypes.c_void_p(pool), _np_ptr(queries), _np_ptr(arrival_s), n, depth, stride,
                                  _np_ptr(n_out), _np_ptr(ids), _np_ptr(dist), _np_ptr(done_s), _np_ptr(probes),
                                  ctypes.byref(stats)),
           "search_run_stream")
    return ids, dist, n_out, done_s, stats, probes


# ------------------------------------------------------------------------------------------- holders
def _aligned(t, align=256):
    return (t.data_ptr() + align - 1) // align * align


class Pool:
    """Owns the torch tensors that back a pool: its device workspace, its pinned host memory and its
    indexes' storage (the library allocates no device memory; library_memory=True lets it allocate
    the pinned host memory and the temporary memory of index builds itself; static_workspace=True
    makes the pool with tri_pool_create_static, in the library's own static device array)."""

    def __init__(self, **cfg_fields):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the search path has no CPU fallback")
        # (a step can only be recorded for replay on a stream of its own, never on the default stream)
        own_stream = bool(cfg_fields.pop("own_stream", False))
        self.library_memory = bool(cfg_fields.pop("library_memory", False))
        self.static_workspace = bool(cfg_fields.pop("static_workspace", False))
        self.cfg = tri_pool_cfg(**cfg_fields)
        self._stream = torch.cuda.Stream() if own_stream or self.cfg.flags & TRI_FLAG_GRAPH else torch.cuda.current_stream()
        self.cfg.hip_stream = self._stream.cuda_stream
        nbytes, pinned_bytes = tri_pool_workspace_bytes(self.cfg)
        self._pinned = None
        self._index_mem = {}
        if self.static_workspace:
            self._ws = None
            self._pinned = torch.empty(pinned_bytes + 256, dtype=torch.uint8, pin_memory=True)
            self.handle = tri_pool_create_static(self.cfg, _aligned(self._pinned), pinned_bytes)
            return
        self._ws = self._device_bytes(nbytes)
        if self.library_memory:
            self.handle = tri_pool_create(self.cfg, _aligned(self._ws), nbytes)
        else:
            self._pinned = torch.empty(pinned_bytes + 256, dtype=torch.uint8, pin_memory=True)
            self.handle = tri_pool_create(self.cfg, _aligned(self._ws), nbytes, _aligned(self._pinned), pinned_bytes)

    def _device_bytes(self, nbytes: int):
        """Device memory the pool's stream will work in, allocated as that stream's: torch's allocator hands a
        freed block to a new tensor of the same stream without waiting, so memory taken on another stream could
        still be written by that stream's pending kernels (a temporary of theirs) after the library has cleared it."""
        import torch
        with torch.cuda.stream(self._stream):
            return torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")

    def build_index(self, base, dim: int, nlist: int, dtype: int, build_metric: int, train_iters: int,
                    centroids: Optional[np.ndarray] = None, seed: int = 0) -> int:
        """base: torch tensor (cpu or cuda) or numpy array, row-major [n, dim] of the index dtype."""
        import torch
        params = ivf_params(dim, nlist, dtype, build_metric, train_iters, seed)
        n = int(base.shape[0])
        nbytes = ivf_build_bytes(params, n)
        mem = self._device_bytes(nbytes)
        if isinstance(base, np.ndarray):
            base = np.ascontiguousarray(base)
            base_ptr, on_host = base.ctypes.data, True
        else:
            base = base.contiguous()
            base_ptr, on_host = base.data_ptr(), not base.is_cuda
        torch.cuda.current_stream().synchronize()
        if self.library_memory:
            index = ivf_build(self.handle, params, base_ptr, n, centroids, _aligned(mem), nbytes)
        else:
            tmp_bytes = ivf_build_tmp_bytes(params, n, on_host)
            tmp = self._device_bytes(tmp_bytes)
            index = ivf_build(self.handle, params, base_ptr, n, centroids, _aligned(mem), nbytes, _aligned(tmp), tmp_bytes)
            del tmp
        self._index_mem[index] = mem
        return index

    def destroy_index(self, index: int) -> None:
        ivf_destroy(index)
        self._index_mem.pop(index, None)

    def close(self) -> None:
        if self.handle:
            for index in list(self._index_mem):
                self.destroy_index(index)
            tri_pool_destroy(self.handle)
            self.handle = None
            self._ws = None
            self._pinned = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
