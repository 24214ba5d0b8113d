"""Seeded synthetic inputs for RBE retrieval tests and benchmarks.

The paper's corpus (1.2 billion keyword embeddings from a commercial search
engine, n = 64 dimensions, two or three bits per dimension, Sec. 7-8) is not
public.  These generators stand in for it: unit-norm vectors drawn from a
Gaussian mixture, so that a query has many close neighbours inside its own
cluster, in the shapes the paper uses (d = 64 or 128, ~1e6 .. 1e9 items).

This module produces *inputs only*.  It holds none of the scoring or selection
arithmetic, imports neither the GPU library nor the oracle, and serves both.

Two back-ends, each deterministic for a given (seed, chunk) pair:

* ``vectors_numpy``  -- CPU, for corpora the oracle can scan in seconds;
* ``vectors_torch``  -- any torch device, for corpora generated directly into
  HBM.  The two back-ends use different random streams and do not produce the
  same values; a test or benchmark picks one and hands the *same* arrays to the
  GPU library and to the oracle.

``pack_planes_torch`` turns device-resident vectors into packed bit-planes and
per-plane fp32 scales with plain torch ops, so that a billion-item corpus can
be produced in HBM without a round trip through the host.  It is an input
recipe (greedy sign binarisation, scale = mean absolute residual), not the
method under test; tests compare it with the oracle's encoder on a sample.
"""
from __future__ import annotations

import numpy as np

SEED_CENTRES = 18020646
SEED_ITEMS = 6466
SEED_QUERIES = 1802


# --------------------------------------------------------------------------
# numpy back-end
# --------------------------------------------------------------------------
def centres_numpy(n_clusters: int, d: int, seed: int = SEED_CENTRES) -> np.ndarray:
    rng = np.random.default_rng([seed, n_clusters, d])
    return rng.standard_normal((n_clusters, d)).astype(np.float32)


def vectors_numpy(n: int, centres: np.ndarray, sigma: float, seed: int, chunk: int = 0,
                  sort_by_cluster: bool = False) -> np.ndarray:
    """n unit vectors: centre of a uniformly drawn cluster + sigma * N(0, I)."""
    rng = np.random.default_rng([seed, chunk])
    m = rng.integers(0, centres.shape[0], size=n)
    if sort_by_cluster:
        m = np.sort(m)
    x = centres[m] + np.float32(sigma) * rng.standard_normal((n, centres.shape[1])).astype(np.float32)
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    return x.astype(np.float32)


def near_duplicates_numpy(n: int, d: int, n_distinct: int, seed: int) -> np.ndarray:
    """n unit vectors of which only n_distinct are different (exact duplicates)."""
    rng = np.random.default_rng([seed, n_distinct])
    base = rng.standard_normal((n_distinct, d)).astype(np.float32)
    base /= np.linalg.norm(base, axis=1, keepdims=True)
    return base[rng.integers(0, n_distinct, size=n)]


# --------------------------------------------------------------------------
# torch back-end (device-resident corpora)
# --------------------------------------------------------------------------
def centres_torch(n_clusters: int, d: int, device, seed: int = SEED_CENTRES):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(seed * 7919 + n_clusters * 31 + d)
    return torch.randn((n_clusters, d), generator=g, device=device, dtype=torch.float32)


def vectors_torch(n: int, centres, sigma: float, seed: int, chunk: int = 0, sort_by_cluster: bool = False):
    import torch
    dev = centres.device
    g = torch.Generator(device=dev)
    g.manual_seed((seed * 1000003 + chunk) & 0x7FFFFFFFFFFFFFFF)
    m = torch.randint(0, centres.shape[0], (n,), generator=g, device=dev)
    if sort_by_cluster:
        m = torch.sort(m).values
    x = torch.randn((n, centres.shape[1]), generator=g, device=dev, dtype=torch.float32)
    x.mul_(sigma).add_(centres[m])
    x.div_(torch.linalg.vector_norm(x, dim=1, keepdim=True))
    return x


def pack_planes_torch(x, n_planes: int):
    """x [n][d] fp32 (any device) -> planes int64 [P][n][W] (bit patterns of the
    uint64 words, dimension i = bit i%64 of word i/64, 1 = positive) and
    scales fp32 [P][n] (mean absolute residual)."""
    import torch
    n, d = x.shape
    assert d % 64 == 0
    W = d // 64
    w8 = torch.tensor([1, 2, 4, 8, 16, 32, 64, 128], dtype=torch.uint8, device=x.device)
    planes = torch.empty((n_planes, n, W), dtype=torch.int64, device=x.device)
    scales = torch.empty((n_planes, n), dtype=torch.float32, device=x.device)
    r = x.clone()
    for t in range(n_planes):
        alpha = r.abs().mean(dim=1)
        pos = r > 0
        by = (pos.view(n, d // 8, 8).to(torch.uint8) * w8).sum(dim=2, dtype=torch.uint8)
        planes[t] = by.contiguous().view(torch.int64).view(n, W)
        scales[t] = alpha
        r -= alpha[:, None] * (pos.to(torch.float32) * 2.0 - 1.0)
    return planes, scales
