"""The input recipe that builds large graphs with torch (workloads/device_graphs.py), at a size the
CPU finishes in a second, with pieces and buckets small enough that every loop takes several turns."""
import numpy as np
import torch

from workloads import device_graphs


def build(seed=5):
    return device_graphs.chung_lu_csr(200_000, 1_000_000, 2.2, seed, device="cpu", piece=1 << 17, bucket=1 << 18)


def test_chung_lu_csr_is_a_simple_undirected_graph():
    n = 200_000
    off_t, adj_t = build()
    offsets, adj = device_graphs.to_host_csr(off_t, adj_t)
    assert offsets.dtype == np.uint64 and adj.dtype == np.uint32 and offsets.size == n + 1
    assert offsets[0] == 0 and offsets[-1] == adj.size and abs(adj.size // 2 - 1_000_000) < 5_000
    deg = np.diff(offsets.astype(np.int64))
    src = np.repeat(np.arange(n, dtype=np.int64), deg)
    assert (src != adj).all()                                   # no loops
    key = (src << 32) | adj
    assert (np.diff(key) > 0).all()                             # rows in order, neighbours in order, none repeated
    assert np.array_equal(np.sort((adj.astype(np.int64) << 32) | src), key)  # every edge in both rows


def test_chung_lu_csr_is_seeded_and_heavy_tailed():
    a = build()
    b = build()
    c = build(seed=6)
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert not torch.equal(a[0], c[0])
    deg = np.sort(np.diff(a[0].numpy()))[::-1]
    # exponent 2.2: weights fall as rank^(-1/1.2); the hub's row is cut by de-duplication, the bulk is not
    assert deg[0] > 100 * np.median(deg) and deg[0] < 200_000
    ratio = deg[1000] / deg[10000]
    assert 0.6 * 10 ** (1 / 1.2) < ratio < 1.4 * 10 ** (1 / 1.2), ratio
