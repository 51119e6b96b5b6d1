"""Seeded sample pools: arrays of ``(u, v)`` node pairs, ``uint32[P][2]``.

These pools are the *input* of the training hot path.  ``walk_pool`` gives them
the structure of the paper's workload (pairs within a window on random walks
that depart with probability proportional to degree, then shuffled) with
numpy's own generator; it is an input recipe, not the trainer's or the oracle's
augmentation code.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def walk_pool(offsets: np.ndarray, adj: np.ndarray, num_samples: int, walk_length: int = 40,
              window: int = 5, seed: int = 0, shuffle: bool = True) -> np.ndarray:
    """Pairs ``(w_i, w_j)``, ``0 < j - i <= window``, from walks of
    ``walk_length`` edges; departure node proportional to degree (owner of a
    uniformly chosen half-edge), every step to a uniformly chosen neighbour."""
    rng = _rng(seed)
    L, s = int(walk_length), int(window)
    per_walk = sum(L + 1 - delta for delta in range(1, s + 1))
    walks = -(-int(num_samples) // per_walk)
    off = offsets.astype(np.int64)
    half_edges = int(off[-1])
    path = np.empty((walks, L + 1), dtype=np.uint32)
    start = rng.integers(half_edges, size=walks)
    cur = (np.searchsorted(off, start, side="right") - 1).astype(np.int64)
    path[:, 0] = cur
    for t in range(1, L + 1):
        base = off[cur]
        deg = off[cur + 1] - base
        pick = np.minimum((rng.random(walks) * deg).astype(np.int64), deg - 1)
        cur = adj[base + pick].astype(np.int64)
        path[:, t] = cur
    parts = []
    for delta in range(1, s + 1):
        a = path[:, : L + 1 - delta].reshape(-1)
        b = path[:, delta:].reshape(-1)
        parts.append(np.stack([a, b], axis=1))
    pool = np.concatenate(parts, axis=0)
    if shuffle:
        pool = pool[rng.permutation(pool.shape[0])]
    return np.ascontiguousarray(pool[:num_samples], dtype=np.uint32)


def marginal_pool(deg: np.ndarray, num_samples: int, seed: int = 0) -> np.ndarray:
    """Both endpoints drawn independently with probability proportional to
    degree: the row-access distribution of a walk pool without the graph
    structure (stand-in when adjacency does not fit the time budget)."""
    rng = _rng(seed)
    cdf = np.cumsum(deg.astype(np.float64))
    cdf /= cdf[-1]
    n = deg.size
    u = np.minimum(np.searchsorted(cdf, rng.random(num_samples), side="right"), n - 1)
    v = np.minimum(np.searchsorted(cdf, rng.random(num_samples), side="right"), n - 1)
    return np.ascontiguousarray(np.stack([u, v], axis=1), dtype=np.uint32)
