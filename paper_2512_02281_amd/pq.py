"""ctypes binding of include/trinity_pq.h: IVF search over product-quantised lists.  Argument marshalling only; torch
tensors own the device memory.  There is no CPU fallback."""
from __future__ import annotations

import ctypes
from typing import Optional

import numpy as np

from . import _lib, _check, _np_ptr, TRI_OK   # noqa: F401  (the library is loaded by the package)

PQ_EXPORTS = ["pq_build_bytes", "pq_build", "pq_destroy", "pq_export", "pq_search_bytes", "pq_search_batch", "pq_sync",
              "pq_lds_gather_rate"]
TRI_PQ_KSUB = 256
TRI_PQ_KMAX = 256
TRI_PQ_NPROBE_MAX = 256
TRI_PQ_DSUB_MAX = 32


class pq_params(ctypes.Structure):
    _fields_ = [("m", ctypes.c_uint32), ("train_iters", ctypes.c_uint32), ("train_rows", ctypes.c_uint32),
                ("refine_rows", ctypes.c_uint32), ("seed", ctypes.c_uint64)]


def _bind():
    vp, u32, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_size_t
    P = ctypes.POINTER
    _lib.pq_build_bytes.argtypes = [vp, P(pq_params), P(sz), P(sz)]
    _lib.pq_build.argtypes = [vp, P(pq_params), vp, vp, sz, vp, sz, P(vp)]
    _lib.pq_destroy.argtypes = [vp]
    _lib.pq_export.argtypes = [vp, vp, vp]
    _lib.pq_search_bytes.argtypes = [vp, u32, P(sz)]
    _lib.pq_search_batch.argtypes = [vp, vp, sz, u32, u32, u32, u32, u32, vp, sz, vp, vp, vp, vp]
    _lib.pq_sync.argtypes = [vp]
    _lib.pq_lds_gather_rate.argtypes = [u32, u32, vp, vp, P(ctypes.c_double)]
    for name in PQ_EXPORTS:
        getattr(_lib, name).restype = ctypes.c_int


_bind()


def _aligned(t, align=256):
    return (t.data_ptr() + align - 1) // align * align


def lds_gather_rate(m: int, rounds: int = 200) -> float:
    """Look-ups per second of a bare loop of the scan's byte-indexed LDS look-ups into m tables (current stream)."""
    import torch
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = ctypes.c_double(0.0)
    torch.cuda.synchronize()
    _check(_lib.pq_lds_gather_rate(m, rounds, ctypes.c_void_p(sink.data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream),
                                   ctypes.byref(out)), "pq_lds_gather_rate")
    return float(out.value)


class PQ:
    """Codebooks and codes of an index of a living Pool (the Pool owns the stream; this object the device memory)."""

    def __init__(self, pool, index: int, m: int, train_iters: int = 8, train_rows: int = 0, seed: int = 0,
                 codebooks: Optional[np.ndarray] = None, refine_rows: bool = False):
        import torch
        self.pool, self.index = pool, index
        self.params = pq_params(m, train_iters, train_rows, 1 if refine_rows else 0, seed)
        dev, tmp = ctypes.c_size_t(0), ctypes.c_size_t(0)
        _check(_lib.pq_build_bytes(ctypes.c_void_p(index), ctypes.byref(self.params), ctypes.byref(dev), ctypes.byref(tmp)), "pq_build_bytes")
        self._mem = pool._device_bytes(dev.value)
        tmp_t = pool._device_bytes(tmp.value)
        cb_ptr = None
        if codebooks is not None:
            codebooks = np.ascontiguousarray(codebooks, dtype=np.float32)
            cb_ptr = _np_ptr(codebooks)
        torch.cuda.current_stream().synchronize()
        h = ctypes.c_void_p(0)
        _check(_lib.pq_build(ctypes.c_void_p(index), ctypes.byref(self.params), cb_ptr, ctypes.c_void_p(_aligned(self._mem)), dev.value,
                             ctypes.c_void_p(_aligned(tmp_t)), tmp.value, ctypes.byref(h)), "pq_build")
        self.handle = h.value
        self.m = m
        del tmp_t

    def export(self, n: int, dim: int):
        cb = np.empty((self.m, TRI_PQ_KSUB, dim // self.m), dtype=np.float32)
        codes = np.empty((n, self.m), dtype=np.uint8)
        _check(_lib.pq_export(ctypes.c_void_p(self.handle), _np_ptr(cb), _np_ptr(codes)), "pq_export")
        return cb, codes

    def workspace(self, nq: int):
        ws = ctypes.c_size_t(0)
        _check(_lib.pq_search_bytes(ctypes.c_void_p(self.handle), nq, ctypes.byref(ws)), "pq_search_bytes")
        return self.pool._device_bytes(ws.value), ws.value

    def search(self, queries, k: int, nprobe: int, metric: int, ws=None, keep_probes: bool = True, out=None, k_adc: int = 0):
        """queries: torch cuda tensor [nq, dim] of the index's storage type.  Returns torch tensors (ids int32 as
        uint32 bits, dist, n_out[, probes]) on the device; asynchronous on the pool's stream (sync() waits).
        k_adc >= k: the k_adc best by table sums are re-ranked by their exact scores against the stored vectors."""
        import torch
        nq = int(queries.shape[0])
        if ws is None:
            ws = self.workspace(nq)
        ws_t, ws_bytes = ws
        with torch.cuda.stream(self.pool._stream):
            if out is None:
                ids = torch.empty((nq, k), dtype=torch.int32, device="cuda")
                dist = torch.empty((nq, k), dtype=torch.float32, device="cuda")
                n_out = torch.empty((nq,), dtype=torch.int32, device="cuda")
                probes = torch.empty((nq, nprobe), dtype=torch.int32, device="cuda") if keep_probes else None
            else:
                ids, dist, n_out, probes = out
        _check(_lib.pq_search_batch(ctypes.c_void_p(self.handle), ctypes.c_void_p(queries.data_ptr()),
                                    int(queries.stride(0)) * queries.element_size(), nq, k, k_adc, nprobe, metric,
                                    ctypes.c_void_p(_aligned(ws_t)), ws_bytes, ctypes.c_void_p(ids.data_ptr()),
                                    ctypes.c_void_p(dist.data_ptr()), ctypes.c_void_p(n_out.data_ptr()),
                                    ctypes.c_void_p(probes.data_ptr()) if probes is not None else None), "pq_search_batch")
        return ids, dist, n_out, probes

    def sync(self):
        _check(_lib.pq_sync(ctypes.c_void_p(self.handle)), "pq_sync")

    def close(self):
        if self.handle:
            _check(_lib.pq_destroy(ctypes.c_void_p(self.handle)), "pq_destroy")
            self.handle = None
            self._mem = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
