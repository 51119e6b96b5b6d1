"""Pins of the oracle's weighted-graph walk (Sec. 4.3: alias tables for the departure node and for every step,
negatives from the 3/4 power of the weighted degree): a triangle by hand, exact table masses, chi-squared of
the transitions and of the departures, reductions to the unweighted routines.  No GPU."""
import numpy as np
import pytest
from scipy import stats

import oracle
import workloads as W


def weighted_csr(n, src, dst, w):
    """Both directions of every edge with its weight, rows in the order csr_from_edges uses."""
    a = np.concatenate([src, dst])
    order = np.argsort(a, kind="stable")
    offsets, adj = W.csr_from_edges(n, src, dst)
    return offsets, adj, np.ascontiguousarray(np.concatenate([w, w])[order], dtype=np.float32)


def row_mass(thresh, alias, begin, end):
    """Probability of every entry of one row under its table, from the table alone."""
    size = end - begin
    t = thresh[begin:end].astype(np.float64) + (thresh[begin:end] == 0xFFFFFFFF)
    mass = t.copy()
    np.add.at(mass, alias[begin:end], 2.0**32 - t)
    return mass / (size * 2.0**32)


def test_weighted_triangle_by_hand():
    # edges (0,1) weight 1, (0,2) weight 3, (1,2) weight 2
    offsets, adj, wts = weighted_csr(3, np.array([0, 0, 1], dtype=np.uint32), np.array([1, 2, 2], dtype=np.uint32),
                                     np.array([1.0, 3.0, 2.0], dtype=np.float32))
    assert list(adj) == [1, 2, 2, 0, 0, 1] and list(wts) == [1, 3, 2, 1, 3, 2]
    assert list(oracle.weighted_degrees(offsets, wts)) == [4.0, 3.0, 5.0]
    thresh, alias = oracle.neighbor_alias(offsets, wts)
    # row 0: weights 1, 3 -> scaled 0.5, 1.5: entry 0 keeps half and passes the rest to entry 1, which keeps all
    assert thresh[0] == 2**31 and alias[0] == 1 and thresh[1] == 0xFFFFFFFF
    for x, want in ((0, [0.25, 0.75]), (1, [2 / 3, 1 / 3]), (2, [0.6, 0.4])):
        assert np.abs(row_mass(thresh, alias, int(offsets[x]), int(offsets[x + 1])) - want).max() <= 2.0**-32
    node_thresh, node_alias = oracle.alias_build(oracle.weighted_degrees(offsets, wts))
    mass = row_mass(node_thresh, node_alias, 0, 3)
    assert np.abs(mass - np.array([4, 3, 5]) / 12).max() <= 2.0**-32
    with pytest.raises(ValueError):
        oracle.neighbor_alias(offsets, np.zeros(6, dtype=np.float32))


def test_weighted_walks_follow_the_weights(tiny_graph):
    g = tiny_graph
    n = g["n"]
    rng = np.random.default_rng(4)
    w = rng.choice([0.25, 1.0, 4.0, 9.0], size=g["src"].size).astype(np.float32)
    offsets, adj, wts = weighted_csr(n, g["src"], g["dst"], w)
    tables = oracle.walk_tables(offsets, wts)
    # every row's table reproduces its weights exactly
    for x in rng.integers(n, size=200):
        lo, hi = int(offsets[x]), int(offsets[x + 1])
        want = wts[lo:hi].astype(np.float64)
        assert np.abs(row_mass(tables[2], tables[3], lo, hi) - want / want.sum()).max() <= 2.0**-32 + 1e-15
    L, s, walks = 40, 5, 30_000
    pairs, used = oracle.augment_weighted(21, offsets, adj, tables, L, s, 190 * walks)
    assert used == walks
    per_walk = pairs.reshape(walks, 190, 2)
    # steps go along edges: the pairs at distance one are the first pair of each i-group of a walk
    starts = np.cumsum([0] + [min(s, L - i) for i in range(L)])[:-1]
    step = per_walk[:, starts, :].reshape(-1, 2)
    edge_keys = set((g["src"].astype(np.int64) * n + g["dst"]).tolist()) | set((g["dst"].astype(np.int64) * n + g["src"]).tolist())
    assert all(int(a) * n + int(b) in edge_keys for a, b in step[:5000])
    # transitions out of the heaviest node follow its edge weights
    wdeg = oracle.weighted_degrees(offsets, wts)
    hub = int(np.argmax(wdeg))
    lo, hi = int(offsets[hub]), int(offsets[hub + 1])
    to = step[step[:, 0] == hub, 1]
    assert to.size > 2000
    expected = np.zeros(n)
    np.add.at(expected, adj[lo:hi], wts[lo:hi].astype(np.float64))
    expected = expected / expected.sum() * to.size
    observed = np.bincount(to, minlength=n)
    keep = expected >= 5
    chi2 = ((observed[keep] - expected[keep]) ** 2 / expected[keep]).sum() + \
           (observed[~keep].sum() - expected[~keep].sum()) ** 2 / max(expected[~keep].sum(), 1e-9)
    assert observed[expected == 0].sum() == 0
    assert stats.chi2.sf(chi2, keep.sum()) > 1e-3
    # departures, and (stationarity) every later node of a walk, are distributed as the weighted degree
    for nodes in (per_walk[:, 0, 0], step[:, 1][::7]):
        expected = wdeg / wdeg.sum() * nodes.size
        observed = np.bincount(nodes, minlength=n)
        keep = expected >= 5
        chi2 = ((observed[keep] - expected[keep]) ** 2 / expected[keep]).sum() + \
               (observed[~keep].sum() - expected[~keep].sum()) ** 2 / max(expected[~keep].sum(), 1e-9)
        assert stats.chi2.sf(chi2, keep.sum()) > 1e-3
    # prefix and offset consistency: walks are numbered, a later call continues the stream
    again, _ = oracle.augment_weighted(21, offsets, adj, tables, L, s, 190 * 3 + 17, first_walk=5)
    assert np.array_equal(again[:190 * 3], pairs[190 * 5:190 * 8]) and np.array_equal(again[190 * 3:], pairs[190 * 8:190 * 8 + 17])


def test_unit_weights_reduce_to_the_unweighted_walk(tiny_graph):
    """With all weights one, weighted degrees are the degrees (so negatives have the same table) and every row's
    table accepts always: a step picks the entry the unweighted walk picks from the same random words."""
    g = tiny_graph
    offsets, adj = g["offsets"], g["adj"]
    wts = np.ones(adj.size, dtype=np.float32)
    wdeg = oracle.weighted_degrees(offsets, wts)
    assert np.array_equal(wdeg, g["deg"].astype(np.float64))
    assert np.array_equal(oracle.weights_pow34(wdeg), oracle.degree_weights(g["deg"]))
    q = np.array([0.0, 1.0, 16.0, 81.0, 7.5])
    assert np.allclose(oracle.weights_pow34(q), q ** 0.75, rtol=1e-15, atol=0)
    tables = oracle.walk_tables(offsets, wts)
    assert np.all(tables[2] == 0xFFFFFFFF)
    # On a regular graph the two departure rules name the same node too (owner of half-edge floor(R 2m / 2^64)
    # with m = n d / 2 is node floor(R n / 2^64), the bucket the flat node table accepts): whole walks coincide.
    n = 1000
    ring = np.arange(n, dtype=np.uint32)
    src = np.concatenate([ring, ring])
    dst = np.concatenate([(ring + 1) % n, (ring + 2) % n]).astype(np.uint32)
    offsets, adj = W.csr_from_edges(n, src, dst)
    assert np.all(np.diff(offsets.astype(np.int64)) == 4)
    tables = oracle.walk_tables(offsets, np.ones(adj.size, dtype=np.float32))
    assert np.all(tables[0] == 0xFFFFFFFF) and np.all(tables[2] == 0xFFFFFFFF)
    weighted, used_w = oracle.augment_weighted(33, offsets, adj, tables, 40, 5, 190 * 500 + 7, first_walk=2**35)
    plain, used_p = oracle.augment(33, offsets, adj, 40, 5, 190 * 500 + 7, first_walk=2**35)
    assert used_w == used_p == 501 and np.array_equal(weighted, plain)
