"""ctypes binding of include/trinity_graph.h: the pool worker's graph engine (paper Sec. 3.2, the
continuous-batching extend loop over a fixed-degree neighbour graph).  Argument marshalling only;
every step of the path runs in the library's kernels.  PyTorch owns the device memory and the stream."""
from __future__ import annotations

import ctypes
from typing import Optional

import numpy as np

from . import (TRI_CLASS_LOW, TRI_EAGAIN, TRI_F16, TRI_F32, TRI_FLAG_PROFILE, TRI_OK, TriError, _check, _lib, _np_ptr,
               tri_last_error)

GRAPH_EXPORTS = ["graph_pool_bytes", "graph_pool_create", "graph_pool_destroy", "graph_submit", "graph_step",
                 "graph_poll", "graph_sync", "graph_kernel_times", "graph_run_stream"]
TRI_GRAPH_TOPM_LIMIT = 256
TRI_GRAPH_TASK_LIMIT = 256
TRI_GRAPH_PAD = 0xFFFFFFFF
TRI_GRAPH_VISITED_HASH, TRI_GRAPH_VISITED_BITS = 16, 32


class tri_graph_cfg(ctypes.Structure):
    _fields_ = [("slots", ctypes.c_uint32), ("topm", ctypes.c_uint32), ("parents", ctypes.c_uint32),
                ("max_iters", ctypes.c_uint32), ("max_outstanding", ctypes.c_uint32), ("groups", ctypes.c_uint32),
                ("flags", ctypes.c_uint32), ("pad_", ctypes.c_uint32), ("hip_stream", ctypes.c_void_p)]


class tri_graph_step_stats(ctypes.Structure):
    _fields_ = [("step", ctypes.c_uint64), ("admitted", ctypes.c_uint32), ("running", ctypes.c_uint32),
                ("finished", ctypes.c_uint32), ("pending", ctypes.c_uint32)]


class tri_graph_times(ctypes.Structure):
    _fields_ = [("steps", ctypes.c_uint64), ("tasks", ctypes.c_uint64), ("step_kernel_ms", ctypes.c_double),
                ("row_bytes", ctypes.c_uint32), ("pad_", ctypes.c_uint32)]


class tri_graph_stream_stats(ctypes.Structure):
    _fields_ = [("wall_s", ctypes.c_double), ("steps", ctypes.c_uint64), ("running", ctypes.c_uint64),
                ("max_pending", ctypes.c_uint64)]


def _declare():
    vp, u32, u64, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_size_t
    P = ctypes.POINTER
    _lib.graph_pool_bytes.argtypes = [P(tri_graph_cfg), u64, u32, u32, u32, P(sz)]
    _lib.graph_pool_create.argtypes = [P(tri_graph_cfg), vp, vp, u64, u32, u32, u32, vp, u32, vp, sz, P(vp)]
    _lib.graph_pool_destroy.argtypes = [vp]
    _lib.graph_submit.argtypes = [vp, vp, ctypes.c_int, u64, u32, vp, vp, vp, vp, P(u32)]
    _lib.graph_step.argtypes = [vp, P(tri_graph_step_stats)]
    _lib.graph_poll.argtypes = [vp, vp, u32, u32, vp, vp, vp, vp, vp, vp]
    _lib.graph_sync.argtypes = [vp]
    _lib.graph_run_stream.argtypes = [vp, vp, u64, vp, u32, vp, vp, vp, ctypes.c_int, u32, vp, vp, vp, vp,
                                      P(tri_graph_stream_stats)]
    _lib.graph_kernel_times.argtypes = [vp, P(tri_graph_times), ctypes.c_int]
    for name in GRAPH_EXPORTS:
        getattr(_lib, name).restype = ctypes.c_int


_declare()


def _ptr(a):
    """Address of a numpy array (host) or a torch tensor (host or device)."""
    if isinstance(a, np.ndarray):
        return ctypes.c_void_p(a.ctypes.data)
    return ctypes.c_void_p(a.data_ptr())


class GraphPool:
    """One graph index resident on the GPU and the slot table that serves it."""

    def __init__(self, vectors, neighbors, seeds: np.ndarray, dtype: int, slots: int, topm: int, parents: int,
                 max_iters: int, max_outstanding: int = 0, groups: int = 0, flags: int = 0, own_stream: bool = False):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU: the search path has no CPU fallback")
        n, dim = int(vectors.shape[0]), int(vectors.shape[1])
        degree = int(neighbors.shape[1])
        assert int(neighbors.shape[0]) == n
        self._stream = torch.cuda.Stream() if own_stream else torch.cuda.current_stream()
        self.cfg = tri_graph_cfg(slots, topm, parents, max_iters, max_outstanding or 4 * slots, groups, flags, 0,
                                 self._stream.cuda_stream)
        nbytes = ctypes.c_size_t(0)
        _check(_lib.graph_pool_bytes(ctypes.byref(self.cfg), n, dim, degree, dtype, ctypes.byref(nbytes)), "graph_pool_bytes")
        with torch.cuda.stream(self._stream):       # the pool's stream works in it: allocated as that stream's memory
            self._mem = torch.empty(nbytes.value + 256, dtype=torch.uint8, device="cuda")
        ptr = (self._mem.data_ptr() + 255) // 256 * 256
        vectors = np.ascontiguousarray(vectors) if isinstance(vectors, np.ndarray) else vectors.contiguous()
        neighbors = np.ascontiguousarray(neighbors, dtype=np.uint32) if isinstance(neighbors, np.ndarray) else neighbors.contiguous()
        seeds = np.ascontiguousarray(seeds, dtype=np.uint32)
        torch.cuda.synchronize()
        h = ctypes.c_void_p(0)
        _check(_lib.graph_pool_create(ctypes.byref(self.cfg), _ptr(vectors), _ptr(neighbors), n, dim, degree, dtype,
                                      _np_ptr(seeds), int(seeds.shape[0]), ctypes.c_void_p(ptr), nbytes.value, ctypes.byref(h)),
               "graph_pool_create")
        self.handle = h.value
        self.n, self.dim, self.degree, self.dtype = n, dim, degree, dtype
        self._keep = []

    def submit(self, vecs, k, metric, klass: Optional[np.ndarray] = None):
        """vecs: numpy array (host, copied now) or torch cuda tensor (read at admission: keep it alive), [n, dim].
        Returns (tickets, status)."""
        n = int(vecs.shape[0])
        k = np.ascontiguousarray(np.broadcast_to(np.asarray(k, dtype=np.uint32), (n,)))
        metric = np.ascontiguousarray(np.broadcast_to(np.asarray(metric, dtype=np.uint32), (n,)))
        kl = None if klass is None else np.ascontiguousarray(np.broadcast_to(np.asarray(klass, dtype=np.uint32), (n,)))
        on_device = not isinstance(vecs, np.ndarray)
        if on_device:
            assert vecs.is_cuda and vecs.is_contiguous()
            self._keep.append(vecs)
            pitch = vecs.stride(0) * vecs.element_size()
        else:
            vecs = np.ascontiguousarray(vecs)
            pitch = vecs.strides[0]
        tickets = np.zeros(n, dtype=np.uint64)
        done = ctypes.c_uint32(0)
        rc = _lib.graph_submit(ctypes.c_void_p(self.handle), _ptr(vecs), 1 if on_device else 0, pitch, n, _np_ptr(k),
                               _np_ptr(metric), _np_ptr(kl) if kl is not None else None, _np_ptr(tickets), ctypes.byref(done))
        if rc not in (TRI_OK, TRI_EAGAIN):
            raise TriError(rc, "graph_submit", tri_last_error())
        return tickets[:done.value], rc

    def step(self) -> tri_graph_step_stats:
        st = tri_graph_step_stats()
        _check(_lib.graph_step(ctypes.c_void_p(self.handle), ctypes.byref(st)), "graph_step")
        return st

    def sync(self) -> None:
        _check(_lib.graph_sync(ctypes.c_void_p(self.handle)), "graph_sync")

    def poll(self, tickets: np.ndarray, stride: int):
        """(ids [n, stride] int64, dist [n, stride] fp32, n_out, iters, evals, status)."""
        tickets = np.ascontiguousarray(tickets, dtype=np.uint64)
        n = tickets.shape[0]
        ids = np.full((n, stride), -1, dtype=np.int64)
        dist = np.full((n, stride), np.nan, dtype=np.float32)
        n_out = np.zeros(n, dtype=np.uint32)
        iters = np.zeros(n, dtype=np.uint32)
        evals = np.zeros(n, dtype=np.uint32)
        status = np.full(n, TRI_EAGAIN, dtype=np.int32)
        rc = _lib.graph_poll(ctypes.c_void_p(self.handle), _np_ptr(tickets), n, stride, _np_ptr(n_out), _np_ptr(ids),
                             _np_ptr(dist), _np_ptr(iters), _np_ptr(evals), _np_ptr(status))
        if rc < 0:
            raise TriError(rc, "graph_poll", tri_last_error())
        return ids, dist, n_out, iters, evals, status

    def run_all(self, vecs, k, metric, klass=None, max_steps: int = 1_000_000):
        """Submit everything, step until nothing runs or waits, poll.  Returns (ids, dist, n_out, iters, evals, steps)."""
        tickets, rc = self.submit(vecs, k, metric, klass)
        assert rc == TRI_OK and tickets.shape[0] == vecs.shape[0]
        steps = 0
        while True:
            st = self.step()
            steps += 1
            assert steps < max_steps, "graph_step loop did not drain"
            if st.running == 0 and st.pending == 0:
                break
        self.sync()
        kmax = int(np.max(np.asarray(k))) if vecs.shape[0] else 1
        ids, dist, n_out, iters, evals, status = self.poll(tickets, kmax)
        assert np.all(status == TRI_OK), status[status != 0][:5]
        self._keep.clear()
        return ids, dist, n_out, iters, evals, steps

    def run_stream(self, vecs: np.ndarray, arrival_s: np.ndarray, k, metric, klass=None, static_batches: bool = False):
        """Drive the pool through a stream of host queries.  Returns (ids, dist, n_out, done_s, stats)."""
        n = int(vecs.shape[0])
        vecs = np.ascontiguousarray(vecs)
        arrival_s = np.ascontiguousarray(arrival_s, dtype=np.float64)
        k = np.ascontiguousarray(np.broadcast_to(np.asarray(k, dtype=np.uint32), (n,)))
        metric = np.ascontiguousarray(np.broadcast_to(np.asarray(metric, dtype=np.uint32), (n,)))
        kl = None if klass is None else np.ascontiguousarray(np.broadcast_to(np.asarray(klass, dtype=np.uint32), (n,)))
        stride = int(k.max()) if n else 1
        ids = np.full((n, stride), -1, dtype=np.int64)
        dist = np.full((n, stride), np.nan, dtype=np.float32)
        n_out = np.zeros(n, dtype=np.uint32)
        done_s = np.zeros(n, dtype=np.float64)
        st = tri_graph_stream_stats()
        _check(_lib.graph_run_stream(ctypes.c_void_p(self.handle), _ptr(vecs), vecs.strides[0] if n else 0, _np_ptr(arrival_s), n,
                                     _np_ptr(k), _np_ptr(metric), _np_ptr(kl) if kl is not None else None,
                                     1 if static_batches else 0, stride, _np_ptr(n_out), _np_ptr(ids), _np_ptr(dist),
                                     _np_ptr(done_s), ctypes.byref(st)), "graph_run_stream")
        return ids, dist, n_out, done_s, st

    def kernel_times(self, reset: bool = False) -> tri_graph_times:
        t = tri_graph_times()
        _check(_lib.graph_kernel_times(ctypes.c_void_p(self.handle), ctypes.byref(t), 1 if reset else 0), "graph_kernel_times")
        return t

    def close(self) -> None:
        if self.handle:
            _check(_lib.graph_pool_destroy(ctypes.c_void_p(self.handle)), "graph_pool_destroy")
            self.handle = None
            self._mem = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
