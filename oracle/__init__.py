"""CPU oracle for batched IVF-Flat search -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import this
package; the product path never does, and this package never imports the HIP library.

``ivf_oracle.c`` holds the definition (coarse scores, probe set, full scan of the probed
lists, ordering by (score, id)); this file only marshals numpy arrays into it.
``index.py`` holds the oracle's own plain index construction and the checker for an
index exported by somebody else.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

METRIC_L2 = 0
METRIC_IP = 1
DTYPE_F32 = 0
DTYPE_F16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ivf_oracle.c")
_SO = os.path.join(_HERE, "libivf_oracle.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile ivf_oracle.c with gcc (OpenMP) into a shared object beside it."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"])
    return _SO


def _bind(path: str):
    """Load a compiled oracle and declare its argument types."""
    lib = ctypes.CDLL(path)
    vp, u32, u64, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int
    lib.ivf_oracle_coarse.argtypes = [vp, u32, u32, vp, i32, i32, vp]
    lib.ivf_oracle_probe.argtypes = [vp, u32, u32, i32, vp]
    lib.ivf_oracle_scan.argtypes = [vp, i32, u64, u32, vp, vp, u32, vp, u32, vp, i32, u32,
                                    vp, vp, vp, vp, vp, u64, vp]
    lib.ivf_oracle_search.argtypes = [vp, i32, u64, u32, vp, u32, vp, vp, vp, u32, u32, i32,
                                      vp, vp, vp, vp]
    lib.ivf_oracle_search_batch.argtypes = [vp, i32, u64, u32, vp, u32, vp, vp, vp, u32,
                                            vp, vp, vp, u32, u32, vp, vp, vp, vp, vp]
    lib.ivf_oracle_half_to_double.argtypes = [ctypes.c_uint16]
    lib.ivf_oracle_half_to_double.restype = ctypes.c_double
    for f in (lib.ivf_oracle_coarse, lib.ivf_oracle_probe, lib.ivf_oracle_scan,
              lib.ivf_oracle_search, lib.ivf_oracle_search_batch):
        f.restype = ctypes.c_int
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _bind(build_oracle())
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return DTYPE_F32
    if a.dtype == np.float16:
        return DTYPE_F16
    raise TypeError(f"oracle stores fp32 or fp16 vectors, got {a.dtype}")


class Index:
    """The data an IVF-Flat index consists of, as plain host arrays.

    base: [n, d] fp32 or fp16, original row order.  centroids: [nlist, d] fp32 (the values
    the searched index ranks with, widened).  list_off: [nlist+1] uint64.  list_ids: [n]
    int64 (row numbers, list after list).
    """

    def __init__(self, base, centroids, list_off, list_ids):
        self.base = np.ascontiguousarray(base)
        self.centroids = np.ascontiguousarray(centroids, dtype=np.float32)
        self.list_off = np.ascontiguousarray(list_off, dtype=np.uint64)
        self.list_ids = np.ascontiguousarray(list_ids, dtype=np.int64)
        self.n, self.d = self.base.shape
        self.nlist = self.centroids.shape[0]
        self.dtype = _dtype_code(self.base)
        assert self.centroids.shape == (self.nlist, self.d)
        assert self.list_off.shape == (self.nlist + 1,)
        assert self.list_ids.shape == (self.n,)


def half_to_double(bits: int) -> float:
    return _load().ivf_oracle_half_to_double(int(bits) & 0xFFFF)


def coarse_scores(index: Index, q: np.ndarray, metric: int) -> np.ndarray:
    """Step 1: fp64 score of q against every centroid."""
    q = np.ascontiguousarray(q, dtype=index.base.dtype)
    out = np.empty(index.nlist, dtype=np.float64)
    rc = _load().ivf_oracle_coarse(_ptr(index.centroids), index.nlist, index.d, _ptr(q), index.dtype,
                                   int(metric), _ptr(out))
    if rc:
        raise RuntimeError(f"ivf_oracle_coarse -> {rc}")
    return out


def probe_set(scores: np.ndarray, nprobe: int, metric: int) -> np.ndarray:
    """Step 2: the nprobe best centroid numbers in rank order."""
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    out = np.empty(nprobe, dtype=np.uint32)
    rc = _load().ivf_oracle_probe(_ptr(scores), scores.shape[0], int(nprobe), int(metric), _ptr(out))
    if rc:
        raise RuntimeError(f"ivf_oracle_probe -> {rc}")
    return out


def scan(index: Index, q: np.ndarray, probe: np.ndarray, k: int, metric: int, all_candidates: bool = False):
    """Steps 3-5 for a given probe set.

    Returns (ids[k] int64, dist[k] float64, n_out) and, with all_candidates, also
    (cand_ids, cand_scores): every candidate in final order.
    """
    q = np.ascontiguousarray(q, dtype=index.base.dtype)
    probe = np.ascontiguousarray(probe, dtype=np.uint32)
    ids = np.empty(k, dtype=np.int64)
    dist = np.empty(k, dtype=np.float64)
    n_out = ctypes.c_uint32(0)
    n_cand = ctypes.c_uint64(0)
    cap = 0
    cand_ids = cand_scores = None
    if all_candidates:
        cap = int(sum(int(index.list_off[l + 1] - index.list_off[l]) for l in probe))
        cand_ids = np.empty(max(cap, 1), dtype=np.int64)
        cand_scores = np.empty(max(cap, 1), dtype=np.float64)
    rc = _load().ivf_oracle_scan(_ptr(index.base), index.dtype, index.n, index.d,
                                 _ptr(index.list_off), _ptr(index.list_ids), index.nlist,
                                 _ptr(probe), probe.shape[0], _ptr(q), int(metric), int(k),
                                 _ptr(ids), _ptr(dist), ctypes.byref(n_out),
                                 _ptr(cand_ids), _ptr(cand_scores), cap, ctypes.byref(n_cand))
    if rc:
        raise RuntimeError(f"ivf_oracle_scan -> {rc}")
    if all_candidates:
        m = int(n_cand.value)
        return ids, dist, int(n_out.value), cand_ids[:m], cand_scores[:m]
    return ids, dist, int(n_out.value)


def search(index: Index, q: np.ndarray, k: int, nprobe: int, metric: int):
    """Steps 1-5 for one query: (probe[nprobe], ids[k], dist[k], n_out)."""
    q = np.ascontiguousarray(q, dtype=index.base.dtype)
    probe = np.empty(nprobe, dtype=np.uint32)
    ids = np.empty(k, dtype=np.int64)
    dist = np.empty(k, dtype=np.float64)
    n_out = ctypes.c_uint32(0)
    rc = _load().ivf_oracle_search(_ptr(index.base), index.dtype, index.n, index.d,
                                   _ptr(index.centroids), index.nlist, _ptr(index.list_off),
                                   _ptr(index.list_ids), _ptr(q), int(k), int(nprobe), int(metric),
                                   _ptr(probe), _ptr(ids), _ptr(dist), ctypes.byref(n_out))
    if rc:
        raise RuntimeError(f"ivf_oracle_search -> {rc}")
    return probe, ids, dist, int(n_out.value)


def search_batch(index: Index, queries: np.ndarray, k, nprobe, metric):
    """Independent queries, each with its own k / nprobe / metric (scalars broadcast).

    Returns dict(probe [nq, nprobe_max] uint32, ids [nq, kmax] int64, dist [nq, kmax] float64,
    n [nq] uint32, threads int).  Rows are padded with id -1 and +/-inf.
    """
    queries = np.ascontiguousarray(queries, dtype=index.base.dtype)
    nq = queries.shape[0]
    k = np.ascontiguousarray(np.broadcast_to(np.asarray(k, dtype=np.uint32), (nq,)))
    nprobe = np.ascontiguousarray(np.broadcast_to(np.asarray(nprobe, dtype=np.uint32), (nq,)))
    metric = np.ascontiguousarray(np.broadcast_to(np.asarray(metric, dtype=np.uint32), (nq,)))
    kmax = int(k.max()) if nq else 1
    pmax = int(nprobe.max()) if nq else 1
    probe = np.full((nq, pmax), 0xFFFFFFFF, dtype=np.uint32)
    ids = np.empty((nq, kmax), dtype=np.int64)
    dist = np.empty((nq, kmax), dtype=np.float64)
    n_out = np.zeros(nq, dtype=np.uint32)
    threads = ctypes.c_int(0)
    rc = _load().ivf_oracle_search_batch(_ptr(index.base), index.dtype, index.n, index.d,
                                         _ptr(index.centroids), index.nlist, _ptr(index.list_off),
                                         _ptr(index.list_ids), _ptr(queries), nq,
                                         _ptr(k), _ptr(nprobe), _ptr(metric), kmax, pmax,
                                         _ptr(probe), _ptr(ids), _ptr(dist), _ptr(n_out),
                                         ctypes.byref(threads))
    if rc:
        raise RuntimeError(f"ivf_oracle_search_batch -> {rc}")
    return dict(probe=probe, ids=ids, dist=dist, n=n_out, threads=int(threads.value))
