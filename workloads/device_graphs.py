"""Graphs too large for the numpy recipes, generated with torch on whatever device is given.

An input recipe only: seeded draws, sorting and counting, none of the method's arithmetic.  Every
single sort, selection or count works on about 2^29 elements, whatever the size of the graph.
"""
from __future__ import annotations

import math

import numpy as np
import torch

_PIECE = 1 << 28  # elements per elementwise pass, draws per group
_BUCKET = 1 << 29  # aimed number of elements per sort


def _draw_nodes(cdf: torch.Tensor, count: int, gen: torch.Generator) -> torch.Tensor:
    """`count` node ranks, rank r with probability cdf[r] - cdf[r - 1] (int64)."""
    u = torch.rand(count, dtype=torch.float64, device=cdf.device, generator=gen)
    return torch.searchsorted(cdf, u, right=True).clamp_(max=cdf.numel() - 1)


def chung_lu_csr(n: int, num_edges: int, gamma: float, seed: int, device="cuda", piece: int = _PIECE,
                 bucket: int = _BUCKET, progress=None):
    """Power-law graph of the Chung-Lu kind as a CSR adjacency with both directions of every edge.

    Both endpoints of an edge are drawn independently with probability proportional to
    ``rank^(-1/(gamma-1))``; node ids are shuffled; self-loops and repeated pairs are dropped and drawing
    goes on until at least ``num_edges`` distinct edges exist; of those each is kept with probability
    ``num_edges / distinct`` (so the graph has ``num_edges`` edges up to a binomial deviation).
    Returns ``(offsets int64[n + 1], adj int32[2 * edges])`` on ``device``, rows sorted by neighbour id.
    ``progress``: called with a line of text after every stage (a long run should not look hung).
    """
    say = progress or (lambda text: None)
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    assert n < (1 << 31)
    w = torch.arange(1, n + 1, dtype=torch.float64, device=dev).pow_(-1.0 / (gamma - 1.0))
    cdf = torch.cumsum(w, 0)
    cdf /= cdf[-1].clone()
    del w
    perm = torch.randperm(n, device=dev, generator=gen)

    # undirected keys (smaller id << 32 | larger id), kept distinct and sorted in `lows` ranges of the
    # smaller id chosen so that every range receives about the same number of edges
    lows = max(1, math.ceil(1.3 * num_edges / bucket))
    bounds = [int(n * (1.0 - math.sqrt(1.0 - k / lows))) for k in range(lows)] + [n]
    held = [torch.empty(0, dtype=torch.int64, device=dev) for _ in range(lows)]
    distinct, wanted = 0, int(num_edges * 1.25) + 1024
    while distinct < num_edges:
        fresh = [[] for _ in range(lows)]
        for at in range(0, wanted, piece):
            k = min(piece, wanted - at)
            a = perm[_draw_nodes(cdf, k, gen)]
            b = perm[_draw_nodes(cdf, k, gen)]
            lo, hi = torch.minimum(a, b), torch.maximum(a, b)
            keys = ((lo << 32) | hi)[lo != hi]
            del a, b, lo, hi
            for r in range(lows):
                fresh[r].append(keys[(keys >= (bounds[r] << 32)) & (keys < (bounds[r + 1] << 32))])
            del keys
        for r in range(lows):
            held[r] = torch.unique(torch.cat([held[r]] + fresh[r]))  # sorted
            fresh[r] = None
        distinct = sum(h.numel() for h in held)
        say(f"chung_lu_csr: {distinct} distinct edges drawn")
        wanted = int((num_edges - distinct) * 1.5) + 1024
    del cdf, perm
    share = num_edges / distinct
    for r in range(lows):
        h = held[r]
        keep = torch.rand(h.numel(), dtype=torch.float64, device=dev, generator=gen) < share
        held[r] = h[keep]
        del h, keep
    keys = torch.cat(held)  # all edges, sorted
    del held
    m = keys.numel()

    # both directions, row by row: the entries (smaller -> larger) are already sorted by source; the
    # entries (larger -> smaller) of a range of sources are picked out and merged with them by one sort
    ranges = max(1, math.ceil(2.4 * m / bucket))
    counts = torch.zeros(n, dtype=torch.int64, device=dev)
    adj = torch.empty(2 * m, dtype=torch.int32, device=dev)
    filled = 0
    for k in range(ranges):
        first, last = n * k // ranges, n * (k + 1) // ranges  # sources first .. last - 1
        edge = torch.searchsorted(keys, torch.tensor([first << 32, last << 32], dtype=torch.int64, device=dev))
        forward = keys[int(edge[0]):int(edge[1])]
        parts = [forward]
        for at in range(0, m, piece):
            part = keys[at:at + piece]
            part = part[((part & 0xFFFFFFFF) >= first) & ((part & 0xFFFFFFFF) < last)]
            parts.append(((part & 0xFFFFFFFF) << 32) | (part >> 32))
        rows = torch.sort(torch.cat(parts)).values
        del parts, forward
        counts[first:last] = torch.bincount((rows >> 32) - first, minlength=last - first)
        adj[filled:filled + rows.numel()] = (rows & 0xFFFFFFFF).to(torch.int32)
        filled += rows.numel()
        del rows
        say(f"chung_lu_csr: rows of {k + 1}/{ranges} of the nodes sorted")
    assert filled == 2 * m
    offsets = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=offsets[1:])
    return offsets, adj


def _empty_on_huge_pages(count: int, dtype) -> np.ndarray:
    """Uninitialised host array whose pages the kernel is asked to back with huge pages (random access into
    gigabytes of adjacency otherwise misses the TLB at every step); a plain array where that is not on offer."""
    import ctypes

    out = np.empty(count, dtype=dtype)
    try:
        page = 1 << 21
        start = (out.ctypes.data + page - 1) & ~(page - 1)
        length = (out.ctypes.data + out.nbytes - start) & ~(page - 1)
        if length > 0:
            ctypes.CDLL(None, use_errno=True).madvise(ctypes.c_void_p(start), ctypes.c_size_t(length), 14)  # MADV_HUGEPAGE
    except (OSError, AttributeError):
        pass
    return out


def to_host_csr(offsets: torch.Tensor, adj: torch.Tensor):
    """numpy arrays ``(offsets uint64[n + 1], adj uint32[...])`` of a CSR built above, in host memory."""
    host_offsets = _empty_on_huge_pages(offsets.numel(), np.int64)
    host_adj = _empty_on_huge_pages(adj.numel(), np.int32)
    torch.from_numpy(host_offsets).copy_(offsets)
    torch.from_numpy(host_adj).copy_(adj)
    return host_offsets.view(np.uint64), host_adj.view(np.uint32)
