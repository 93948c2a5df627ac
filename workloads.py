"""Seeded synthetic inputs for the batched-IVF search path.

This module only *draws inputs*: mixtures of points, query parameters, arrival
times and k-means seed rows.  It holds none of the search method's arithmetic
(no distances, no ranking, no clustering) and is the only code that both the
CPU oracle's callers and the HIP path's callers share.

The five workloads mirror the shapes and value distributions of the evaluation
configurations this build is measured on; every one of them is synthetic and
stands in for a public corpus of the same shape (1M x 128 byte-valued
descriptors; 768-d unit-norm text embeddings), which is not available here.

Seeds: data 1000+c, queries 2000+c, k-means seed rows 3000+c, per-query
parameters and arrivals 4000+c, where c is the configuration number.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

METRIC_L2 = 0
METRIC_IP = 1
DTYPE_F32 = 0
DTYPE_F16 = 1
CLASS_HIGH = 0
CLASS_LOW = 1


@dataclasses.dataclass(frozen=True)
class Config:
    """Shape of one evaluation configuration (``scale`` shrinks it for tests)."""
    number: int
    name: str
    n_base: int
    dim: int
    dtype: int
    metric: int
    n_components: int
    nlist: int
    n_queries: int
    nprobe: int          # 0 = heterogeneous (see hetero_params)
    k: int               # 0 = heterogeneous
    train_iters: int = 10

    @property
    def seed_data(self) -> int:
        return 1000 + self.number

    @property
    def seed_queries(self) -> int:
        return 2000 + self.number

    @property
    def seed_kmeans(self) -> int:
        return 3000 + self.number

    @property
    def seed_params(self) -> int:
        return 4000 + self.number

    def scaled(self, n_base: int, n_components: int, nlist: int, n_queries: int,
               dim: Optional[int] = None) -> "Config":
        """Same recipe and seeds at a smaller size (parity-test variant)."""
        return dataclasses.replace(self, n_base=n_base, n_components=n_components,
                                   nlist=nlist, n_queries=n_queries,
                                   dim=self.dim if dim is None else dim)


CONFIGS = {
    0: Config(0, "tiny-gauss-f32-l2", 10_000, 128, DTYPE_F32, METRIC_L2, 64, 64, 100, 8, 10),
    1: Config(1, "bytes1m-f32-l2", 1_000_000, 128, DTYPE_F32, METRIC_L2, 1024, 1024, 1024, 32, 10),
    2: Config(2, "emb1m-f16-ip-hetero", 1_000_000, 768, DTYPE_F16, METRIC_IP, 4096, 4096, 2048, 0, 0),
    # configuration 3 is a stream over two indexes: the RAG index is configuration 2's,
    # the prompt-cache index is described by CACHE_INDEX below.
    4: Config(4, "emb10m-f16-ip", 10_000_000, 768, DTYPE_F16, METRIC_IP, 16384, 16384, 4096, 64, 100),
}
CACHE_INDEX = Config(3, "cache200k-f16-ip", 200_000, 768, DTYPE_F16, METRIC_IP, 512, 512, 0, 8, 1)


# --------------------------------------------------------------------------- config 0
def gaussian_mixture_f32(n: int, dim: int, n_components: int, centre_seed: int, point_seed: int,
                         centre_sigma: float = 2.0, noise_sigma: float = 1.0) -> np.ndarray:
    """Points of a Gaussian mixture: centre ~ N(0, centre_sigma^2 I), point = centre + N(0, noise_sigma^2 I).

    ``centre_seed`` fixes the components, ``point_seed`` the draw; base set and
    queries use the same ``centre_seed`` and different ``point_seed``.
    """
    centres = np.random.default_rng(centre_seed).standard_normal((n_components, dim)) * centre_sigma
    rng = np.random.default_rng(point_seed)
    comp = rng.integers(0, n_components, size=n)
    pts = centres[comp] + rng.standard_normal((n, dim)) * noise_sigma
    return np.ascontiguousarray(pts.astype(np.float32))


# --------------------------------------------------------------------------- config 1
def byte_mixture_f32(n: int, dim: int, n_components: int, centre_seed: int, point_seed: int,
                     sigma: float = 20.0, chunk: int = 131072) -> np.ndarray:
    """Integer-valued fp32 points in [0,255]: round(clip(centre + N(0, sigma^2), 0, 255))."""
    centres = np.random.default_rng(centre_seed).uniform(0.0, 255.0, size=(n_components, dim)).astype(np.float32)
    rng = np.random.default_rng(point_seed)
    out = np.empty((n, dim), dtype=np.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = rng.integers(0, n_components, size=e - s)
        blk = centres[comp] + rng.standard_normal((e - s, dim), dtype=np.float32) * np.float32(sigma)
        np.clip(blk, 0.0, 255.0, out=blk)
        np.rint(blk, out=blk)
        out[s:e] = blk
    return out


# --------------------------------------------------------------------------- configs 2-4
def unit_mixture_f16(n: int, dim: int, n_components: int, centre_seed: int, point_seed: int,
                     noise_sigma: float = 0.05, device: str = "cpu", chunk: int = 262144):
    """Unit-norm embedding-like points, stored fp16 (a torch tensor on ``device``).

    centre = normalised Gaussian; point = normalise(centre + N(0, noise_sigma^2 I)).
    Returns (points fp16 [n, dim], component index int64 [n]).
    """
    import torch
    gc = torch.Generator(device=device)
    gc.manual_seed(centre_seed)
    centres = torch.randn((n_components, dim), generator=gc, device=device, dtype=torch.float32)
    centres /= centres.norm(dim=1, keepdim=True)
    gp = torch.Generator(device=device)
    gp.manual_seed(point_seed)
    out = torch.empty((n, dim), dtype=torch.float16, device=device)
    comp_all = torch.empty((n,), dtype=torch.int64, device=device)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = torch.randint(0, n_components, (e - s,), generator=gp, device=device)
        blk = centres[comp] + noise_sigma * torch.randn((e - s, dim), generator=gp, device=device,
                                                          dtype=torch.float32)
        blk /= blk.norm(dim=1, keepdim=True)
        out[s:e] = blk.to(torch.float16)
        comp_all[s:e] = comp
    return out, comp_all


def perturbed_copies_f16(rows, point_seed: int, noise_sigma: float = 0.005):
    """Near-duplicates of the given fp16 rows: normalise(row + N(0, noise_sigma^2 I)), fp16 (torch)."""
    import torch
    g = torch.Generator(device=rows.device)
    g.manual_seed(point_seed)
    blk = rows.float() + noise_sigma * torch.randn(rows.shape, generator=g, device=rows.device)
    blk /= blk.norm(dim=1, keepdim=True)
    return blk.to(torch.float16)


# --------------------------------------------------------------------------- shared small draws
def kmeans_seed_rows(n_base: int, nlist: int, seed: int) -> np.ndarray:
    """``nlist`` distinct base-row numbers, ascending: the initial centroids are these rows."""
    rows = np.random.default_rng(seed).choice(n_base, size=nlist, replace=False)
    return np.sort(rows).astype(np.int64)


def hetero_params(n_queries: int, seed: int):
    """Per-query k ~ U{1,10,100} and nprobe ~ U{8,16,32,64,128} (configuration 2)."""
    rng = np.random.default_rng(seed)
    k = rng.choice(np.array([1, 10, 100], dtype=np.uint32), size=n_queries)
    nprobe = rng.choice(np.array([8, 16, 32, 64, 128], dtype=np.uint32), size=n_queries)
    return k.astype(np.uint32), nprobe.astype(np.uint32)


def poisson_arrivals(n: int, rate_per_s: float, seed: int) -> np.ndarray:
    """Arrival times in seconds of a Poisson process (exponential gaps), ascending."""
    rng = np.random.default_rng(seed)
    return np.cumsum(rng.exponential(1.0 / rate_per_s, size=n))


def stream_mix(n: int, seed: int, rag_fraction: float = 0.7):
    """Configuration 3's request mix.

    Returns (is_rag bool[n], k uint32[n], nprobe uint32[n], klass uint32[n],
    cache_is_near_duplicate bool[n]).  RAG: k ~ U{10..100}, nprobe 32, low class.
    Cache lookup: k 1, nprobe 8, high class; half of them are near-duplicates of a
    stored cache vector (expected hit), the rest fresh mixture draws (expected miss).
    """
    rng = np.random.default_rng(seed)
    is_rag = rng.random(n) < rag_fraction
    k = np.where(is_rag, rng.integers(10, 101, size=n), 1).astype(np.uint32)
    nprobe = np.where(is_rag, 32, 8).astype(np.uint32)
    klass = np.where(is_rag, CLASS_LOW, CLASS_HIGH).astype(np.uint32)
    near_dup = (~is_rag) & (rng.random(n) < 0.5)
    return is_rag, k, nprobe, klass, near_dup


# --------------------------------------------------------------------------- whole configs
def make_config01(cfg: Config):
    """(base fp32 [n,d], queries fp32 [q,d], k-means seed rows) for configurations 0 and 1."""
    if cfg.number == 0:
        base = gaussian_mixture_f32(cfg.n_base, cfg.dim, cfg.n_components, cfg.seed_data, cfg.seed_data + 500)
        queries = gaussian_mixture_f32(cfg.n_queries, cfg.dim, cfg.n_components, cfg.seed_data, cfg.seed_queries)
    elif cfg.number == 1:
        base = byte_mixture_f32(cfg.n_base, cfg.dim, cfg.n_components, cfg.seed_data, cfg.seed_data + 500)
        queries = byte_mixture_f32(cfg.n_queries, cfg.dim, cfg.n_components, cfg.seed_data, cfg.seed_queries)
    else:
        raise ValueError("make_config01 serves configurations 0 and 1")
    return base, queries, kmeans_seed_rows(cfg.n_base, cfg.nlist, cfg.seed_kmeans)


def make_config_f16(cfg: Config, device: str = "cpu"):
    """(base fp16 torch [n,d], queries fp16 torch [q,d], k-means seed rows) for configurations 2-4."""
    base, _ = unit_mixture_f16(cfg.n_base, cfg.dim, cfg.n_components, cfg.seed_data, cfg.seed_data + 500,
                               device=device)
    queries, _ = unit_mixture_f16(max(cfg.n_queries, 1), cfg.dim, cfg.n_components, cfg.seed_data,
                                  cfg.seed_queries, device=device)
    return base, queries[:cfg.n_queries], kmeans_seed_rows(cfg.n_base, cfg.nlist, cfg.seed_kmeans)


def make_config3(n_queries: int, device: str = "cpu", rag_cfg: Optional[Config] = None,
                 cache_cfg: Optional[Config] = None):
    """Configuration 3: a stream over two indexes (torch tensors on ``device``).

    RAG index = configuration 2's base; prompt-cache index = CACHE_INDEX.  Query i is a RAG query
    (fresh draw from the RAG mixture) or a cache lookup: a near-duplicate of a stored cache vector
    (cosine about 0.99: an expected hit) or a fresh draw from the cache mixture (an expected miss).
    Returns a dict: rag_base, cache_base, rag_rows, cache_rows (k-means seed rows), queries fp16 [n, d]
    in arrival order, is_rag, k, nprobe, klass, near_dup, dup_of (cache row a near-duplicate copies, else -1).
    """
    import torch
    rag_cfg = rag_cfg or CONFIGS[2]
    cache_cfg = cache_cfg or CACHE_INDEX
    rag_base, _ = unit_mixture_f16(rag_cfg.n_base, rag_cfg.dim, rag_cfg.n_components, rag_cfg.seed_data,
                                   rag_cfg.seed_data + 500, device=device)
    cache_base, _ = unit_mixture_f16(cache_cfg.n_base, cache_cfg.dim, cache_cfg.n_components, cache_cfg.seed_data,
                                     cache_cfg.seed_data + 500, device=device)
    is_rag, k, nprobe, klass, near_dup = stream_mix(n_queries, 4003)
    n_rag, n_dup = int(is_rag.sum()), int(near_dup.sum())
    n_fresh = n_queries - n_rag - n_dup
    queries = torch.empty((n_queries, rag_cfg.dim), dtype=torch.float16, device=device)
    if n_rag:
        qr, _ = unit_mixture_f16(n_rag, rag_cfg.dim, rag_cfg.n_components, rag_cfg.seed_data, 2003, device=device)
        queries[torch.from_numpy(np.flatnonzero(is_rag)).to(device)] = qr
    fresh = (~is_rag) & (~near_dup)
    if n_fresh:
        qf, _ = unit_mixture_f16(n_fresh, cache_cfg.dim, cache_cfg.n_components, cache_cfg.seed_data, 2004,
                                 device=device)
        queries[torch.from_numpy(np.flatnonzero(fresh)).to(device)] = qf
    dup_of = np.full(n_queries, -1, dtype=np.int64)
    if n_dup:
        src = np.random.default_rng(4004).integers(0, cache_cfg.n_base, size=n_dup)
        dup_of[near_dup] = src
        qd = perturbed_copies_f16(cache_base[torch.from_numpy(src).to(device)], 2005)
        queries[torch.from_numpy(np.flatnonzero(near_dup)).to(device)] = qd
    return dict(rag_base=rag_base, cache_base=cache_base,
                rag_rows=kmeans_seed_rows(rag_cfg.n_base, rag_cfg.nlist, rag_cfg.seed_kmeans),
                cache_rows=kmeans_seed_rows(cache_cfg.n_base, cache_cfg.nlist, cache_cfg.seed_kmeans),
                queries=queries, is_rag=is_rag, k=k, nprobe=nprobe, klass=klass, near_dup=near_dup, dup_of=dup_of)
