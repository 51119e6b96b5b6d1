"""Seeded synthetic graphs with the shapes of the paper's datasets.

All graphs are undirected, simple (no self-loops, no multi-edges) and returned
as an edge list ``(src, dst)`` of ``uint32`` arrays, one entry per undirected
edge.  Randomness comes from ``numpy.random.Generator(numpy.random.PCG64(seed))``
only, so a (generator, arguments, seed) triple names one graph.
"""
from __future__ import annotations

import numpy as np


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(int(seed)))


def degrees(n: int, src: np.ndarray, dst: np.ndarray) -> np.ndarray:
    """Number of incident edges per node (uint32)."""
    deg = np.bincount(src, minlength=n) + np.bincount(dst, minlength=n)
    return deg.astype(np.uint32)


def csr_from_edges(n: int, src: np.ndarray, dst: np.ndarray):
    """Adjacency of the undirected graph with both directions stored.

    Returns ``(offsets uint64[n+1], adj uint32[2m])``.  Neighbours of a node
    appear in edge-list order (edge ``i`` contributes ``dst[i]`` to ``src[i]``
    before edge ``j > i`` does; the reverse direction likewise).
    """
    a = np.concatenate([src, dst]).astype(np.uint32)
    b = np.concatenate([dst, src]).astype(np.uint32)
    order = np.argsort(a, kind="stable")
    adj = np.ascontiguousarray(b[order])
    counts = np.bincount(a, minlength=n)
    offsets = np.zeros(n + 1, dtype=np.uint64)
    np.cumsum(counts, out=offsets[1:])
    return offsets, adj


def csr_edge_weights(src: np.ndarray, dst: np.ndarray, seed: int, values=(0.25, 1.0, 4.0, 9.0)):
    """One weight per undirected edge, drawn uniformly from ``values``, laid out like the adjacency of
    ``csr_from_edges`` (both directions of an edge carry its weight): ``float32[2m]``."""
    ew = _rng(seed).choice(np.asarray(values, dtype=np.float32), size=src.size).astype(np.float32)
    order = np.argsort(np.concatenate([src, dst]).astype(np.uint32), kind="stable")
    return np.ascontiguousarray(np.concatenate([ew, ew])[order])


def _dedupe_in_draw_order(a: np.ndarray, b: np.ndarray, n: int):
    """Drop self-loops and repeated undirected pairs, keeping first draws."""
    keep = a != b
    a, b = a[keep], b[keep]
    lo = np.minimum(a, b).astype(np.uint64)
    hi = np.maximum(a, b).astype(np.uint64)
    key = lo * np.uint64(n) + hi
    _, first = np.unique(key, return_index=True)
    first.sort()
    return a[first], b[first]


def barabasi_albert(n: int, m: int, seed: int):
    """Preferential attachment: every new node links to ``m`` distinct older
    nodes chosen with probability proportional to their current degree.
    The first ``m + 1`` nodes form a clique.  ``|E| = m(m+1)/2 + (n-m-1) m``."""
    rng = _rng(seed)
    src, dst = [], []
    ends = []  # every edge endpoint once: uniform choice here == degree-proportional
    for i in range(m + 1):
        for j in range(i + 1, m + 1):
            src.append(i)
            dst.append(j)
            ends += [i, j]
    for v in range(m + 1, n):
        chosen = set()
        while len(chosen) < m:
            chosen.add(ends[int(rng.integers(len(ends)))])
        for t in sorted(chosen):
            src.append(v)
            dst.append(t)
            ends += [v, t]
    return np.asarray(src, dtype=np.uint32), np.asarray(dst, dtype=np.uint32)


def chung_lu(n: int, num_edges: int, gamma: float, seed: int, permute: bool = True):
    """Power-law graph: both endpoints of every edge are drawn independently
    with probability proportional to ``rank^(-1/(gamma-1))``; self-loops and
    repeated pairs are dropped and drawing continues until ``num_edges``
    distinct edges exist.  Node ids are then shuffled so that hub rows are not
    neighbours in memory (real datasets carry no such order)."""
    rng = _rng(seed)
    w = np.arange(1, n + 1, dtype=np.float64) ** (-1.0 / (gamma - 1.0))
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    a = np.empty(0, dtype=np.uint32)
    b = np.empty(0, dtype=np.uint32)
    while a.size < num_edges:
        need = num_edges - a.size
        k = int(need * 1.3) + 1024
        na = np.searchsorted(cdf, rng.random(k), side="right").astype(np.uint32)
        nb = np.searchsorted(cdf, rng.random(k), side="right").astype(np.uint32)
        np.minimum(na, n - 1, out=na)
        np.minimum(nb, n - 1, out=nb)
        a, b = _dedupe_in_draw_order(np.concatenate([a, na]), np.concatenate([b, nb]), n)
    a, b = a[:num_edges], b[:num_edges]
    if permute:
        perm = rng.permutation(n).astype(np.uint32)
        a, b = perm[a], perm[b]
    return np.ascontiguousarray(a), np.ascontiguousarray(b)


def planted_partition(n: int, communities: int, num_edges: int, ratio: float, seed: int):
    """Stochastic block model with equal communities (node ``i`` belongs to
    community ``i % communities``) and ``p_in / p_out = ratio``; exactly
    ``num_edges`` distinct edges.  Returns ``(src, dst, community uint32[n])``."""
    if n % communities:
        raise ValueError("n must be a multiple of the number of communities")
    rng = _rng(seed)
    size = n // communities
    pairs_in = communities * size * (size - 1) / 2.0
    pairs_out = n * (n - 1) / 2.0 - pairs_in
    f_in = ratio * pairs_in / (ratio * pairs_in + pairs_out)
    a = np.empty(0, dtype=np.uint32)
    b = np.empty(0, dtype=np.uint32)
    while a.size < num_edges:
        need = num_edges - a.size
        k = int(need * 1.1) + 1024
        intra = rng.random(k) < f_in
        ca = rng.integers(communities, size=k)
        cb_other = (ca + 1 + rng.integers(communities - 1, size=k)) % communities if communities > 1 else ca
        cb = np.where(intra, ca, cb_other)
        na = (rng.integers(size, size=k) * communities + ca).astype(np.uint32)
        nb = (rng.integers(size, size=k) * communities + cb).astype(np.uint32)
        a, b = _dedupe_in_draw_order(np.concatenate([a, na]), np.concatenate([b, nb]), n)
    a, b = a[:num_edges], b[:num_edges]
    community = (np.arange(n, dtype=np.uint32) % np.uint32(communities)).astype(np.uint32)
    return np.ascontiguousarray(a), np.ascontiguousarray(b), community


def split_holdout(src: np.ndarray, dst: np.ndarray, fraction: float, seed: int):
    """Remove a uniformly chosen ``fraction`` of the edges for link prediction.
    Returns ``(train_src, train_dst, test_src, test_dst)``."""
    rng = _rng(seed)
    m = src.size
    k = max(1, int(round(m * fraction)))
    mask = np.zeros(m, dtype=bool)
    mask[rng.choice(m, size=k, replace=False)] = True
    return src[~mask], dst[~mask], src[mask], dst[mask]


def uniform_negative_pairs(n: int, count: int, seed: int):
    """``count`` node pairs ``(a, b)``, ``a != b``, uniform over ordered pairs."""
    rng = _rng(seed)
    a = rng.integers(n, size=count).astype(np.uint32)
    b = ((a.astype(np.int64) + 1 + rng.integers(n - 1, size=count)) % n).astype(np.uint32)
    return a, b
