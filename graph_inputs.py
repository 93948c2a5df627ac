"""Seeded synthetic inputs for the graph engine: points, queries, entry points and a fixed-degree
neighbour graph.

The engine takes the neighbour graph as an INPUT (the paper keeps "a fixed-degree neighbor list G"
resident and says nothing about how it is made; it cites a GPU graph-index library for that), so
making one here is input preparation, like drawing the points: nearest neighbours by one matrix
product per block of rows plus a few pseudo-random long edges.  Nothing of the search method (topM,
visited, the extend loop, its stop rule) is in this module; the oracle and the HIP path both receive
the arrays made here.

Points lie near a random low-dimensional subspace of the embedding space (then normalised), the kind
of data on which greedy search over a nearest-neighbour graph is meaningful; this stands in for a
768-d text-embedding corpus, which is not available here.  `integer=True` rounds the coordinates to
small integers so that every sum the search forms is exact in fp32 in any order (bit-exact parity).
"""
from __future__ import annotations

import numpy as np

SEED_POINTS, SEED_QUERIES, SEED_EDGES, SEED_ENTRY = 1005, 2005, 3005, 4005


def make_points(n: int, dim: int, latent: int, np_dtype, seed: int, integer: bool = False, device: str = "cpu"):
    """(points [n, dim] of np_dtype as a torch tensor on `device`, latent coordinates [n, latent] fp32 tensor)."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    ga = torch.Generator(device=device)
    ga.manual_seed(SEED_POINTS * 7919 + dim * 31 + latent)         # the subspace is the same for points and queries
    A = torch.randn(latent, dim, generator=ga, device=device) / latent ** 0.5
    out = torch.empty(n, dim, dtype=torch.float16 if np_dtype == np.float16 else torch.float32, device=device)
    Z = torch.empty(n, latent, dtype=torch.float32, device=device)
    for a in range(0, n, 65536):
        b = min(n, a + 65536)
        z = torch.randn(b - a, latent, generator=g, device=device)
        x = z @ A + 0.02 * torch.randn(b - a, dim, generator=g, device=device)
        x = x / x.norm(dim=1, keepdim=True)
        if integer:
            x = torch.clamp(torch.round(x * (4.0 * dim ** 0.5)), -15, 15)    # entries of size ~1/sqrt(dim) -> a few units
        out[a:b] = x.to(out.dtype)
        Z[a:b] = z
    return out, Z


def make_graph(coords, degree: int, n_random: int, seed: int, block: int = 2048) -> "torch.Tensor":
    """Neighbour list [n, degree] uint32 (as int64 torch tensor on coords' device, values < n): the
    degree - n_random nearest rows by squared L2 on `coords` (self excluded, ties by torch.topk's order),
    then n_random pseudo-random rows."""
    import torch
    n = coords.shape[0]
    knn = degree - n_random
    assert 0 < knn < n
    c = coords.float()
    sq = (c * c).sum(1)
    G = torch.empty(n, degree, dtype=torch.int64, device=c.device)
    for a in range(0, n, block):
        b = min(n, a + block)
        d = sq[None, :] - 2.0 * (c[a:b] @ c.T)                    # + |row|^2, the same for a whole row of d
        d[torch.arange(b - a, device=c.device), torch.arange(a, b, device=c.device)] = float("inf")
        G[a:b, :knn] = torch.topk(d, knn, dim=1, largest=False).indices
    if n_random:
        g = torch.Generator(device=c.device)
        g.manual_seed(seed)
        G[:, knn:] = torch.randint(0, n, (n, n_random), generator=g, device=c.device)
    return G


def entry_points(n: int, count: int, seed: int = SEED_ENTRY) -> np.ndarray:
    return np.random.default_rng(seed).choice(n, size=min(count, n), replace=False).astype(np.uint32)
