"""Pins of the oracle's orthogonal-block machinery (Sec. 3.2, Alg. 3; degree-guided partition, Sec. 4.3):
hand-built cases, reductions to the already pinned one-partition routines, brute force, and the
exchangeability of blocks that share no row (Def. 1).  No GPU."""
import numpy as np
import pytest
from scipy import stats

import oracle
import workloads as W


def test_zigzag_partition_by_hand():
    # degrees falling with the id: the deal is 0 1 2 | 2 1 0 | 0 1
    assert list(oracle.zigzag_partition([9, 8, 7, 6, 5, 4, 3, 2], 3)) == [0, 1, 2, 2, 1, 0, 0, 1]
    # ties go by id; the hottest node is node 3, then 0, 2 (tie 5: lower id first), 4, 1
    assert list(oracle.zigzag_partition([7, 1, 5, 9, 5], 2)) == [1, 0, 1, 0, 0]
    assert list(oracle.zigzag_partition([4, 4, 4], 1)) == [0, 0, 0]


def test_zigzag_partition_balances_nodes_and_degree(tiny_graph):
    deg = tiny_graph["deg"]
    for B in (2, 5, 8):
        part = oracle.zigzag_partition(deg, B)
        sizes = np.bincount(part, minlength=B)
        mass = np.bincount(part, weights=deg.astype(np.float64), minlength=B)
        assert sizes.max() - sizes.min() <= 1 and sizes.sum() == deg.size
        assert mass.max() / mass.min() < 1.15  # the hub sits in one partition; the rest evens out


def table_mass(members, thresh, alias, lo, hi, n):
    """Probability of every node under one partition's table, from the table alone."""
    nj = hi - lo
    mass = np.zeros(n)
    np.add.at(mass, members[lo:hi], thresh[lo:hi].astype(np.float64) + (thresh[lo:hi] == 0xFFFFFFFF))
    np.add.at(mass, alias[lo:hi], 2.0**32 - thresh[lo:hi].astype(np.float64) - (thresh[lo:hi] == 0xFFFFFFFF))
    return mass / (nj * 2.0**32)


def test_partition_alias_tables(tiny_graph):
    deg = tiny_graph["deg"].copy()
    deg[::53] = 0
    n = deg.size
    # one partition: the table of the whole graph, already pinned
    offsets, members, thresh, alias = oracle.partition_alias(deg, 1, np.zeros(n, dtype=np.uint32))
    ref_t, ref_a = oracle.alias_build(oracle.degree_weights(deg))
    assert list(offsets) == [0, n] and np.array_equal(members, np.arange(n))
    assert np.array_equal(thresh, ref_t) and np.array_equal(alias, ref_a)
    # several: members listed by id, aliases stay inside the partition, masses are degree^0.75 shares
    B = 4
    part = oracle.zigzag_partition(deg, B)
    offsets, members, thresh, alias = oracle.partition_alias(deg, B, part)
    q = deg.astype(np.float64) ** 0.75
    for j in range(B):
        lo, hi = int(offsets[j]), int(offsets[j + 1])
        assert np.array_equal(members[lo:hi], np.nonzero(part == j)[0])
        assert np.all(part[alias[lo:hi]] == j)
        mass = table_mass(members, thresh, alias, lo, hi, n)
        want = np.where(part == j, q, 0.0)
        assert np.abs(mass - want / want.sum()).max() <= 2.0**-32 + 1e-15
    with pytest.raises(ValueError):
        oracle.partition_alias(np.array([3, 0, 3, 0], dtype=np.uint32), 2, np.array([0, 1, 0, 1], dtype=np.uint32))


def test_restricted_negatives(tiny_graph):
    deg, n = tiny_graph["deg"], tiny_graph["n"]
    rng = np.random.default_rng(0)
    v = rng.integers(n, size=200_000).astype(np.uint32)
    # one partition: the unrestricted draws, bit for bit
    tables = oracle.partition_alias(deg, 1, np.zeros(n, dtype=np.uint32))
    ref = oracle.draw_negatives(77, 2**33, v.size, 2, tables[2], tables[3])
    assert np.array_equal(oracle.draw_negatives_partitioned(77, 2**33, v, 2, np.zeros(n, dtype=np.uint32), tables), ref)
    # several: every negative lies in the partition of its sample's context node, distributed as degree^0.75 there
    B = 4
    part = oracle.zigzag_partition(deg, B)
    tables = oracle.partition_alias(deg, B, part)
    negs = oracle.draw_negatives_partitioned(5, 0, v, 3, part, tables)
    assert np.all(part[negs] == part[v][:, None])
    j = 2
    mine = negs[part[v] == j].reshape(-1)
    q = np.where(part == j, deg.astype(np.float64) ** 0.75, 0.0)
    expected = q / q.sum() * mine.size
    keep = expected >= 5
    observed = np.bincount(mine, minlength=n)
    chi2 = ((observed[keep] - expected[keep]) ** 2 / expected[keep]).sum() + \
           (observed[~keep].sum() - expected[~keep].sum()) ** 2 / max(expected[~keep].sum(), 1e-9)
    assert stats.chi2.sf(chi2, keep.sum()) > 1e-3
    # a sample's negatives depend on its position and its context node only
    again = oracle.draw_negatives_partitioned(5, 1000, v[1000:1010], 3, part, tables)
    assert np.array_equal(again, negs[1000:1010])


def test_block_order_against_a_plain_sort(tiny_graph):
    g = tiny_graph
    B = 5
    part = oracle.zigzag_partition(g["deg"], B)
    pool, _ = oracle.augment(3, g["offsets"], g["adj"], 40, 5, 30_011, shuffle_seed=1)
    order, offsets = oracle.block_order(pool, B, part)
    pi, pj = part[pool[:, 0]].astype(np.int64), part[pool[:, 1]].astype(np.int64)
    key = ((pj - pi) % B) * B + pi  # sub-episode first, then the vertex partition
    assert np.array_equal(order, np.argsort(key, kind="stable"))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(key, minlength=B * B))]))
    # the blocks of one sub-episode share no partition, hence no row
    for o in range(B):
        blocks = [(i, (i + o) % B) for i in range(B)]
        assert len({i for i, _ in blocks}) == B and len({j for _, j in blocks}) == B
        for i, j in blocks:
            lo, hi = int(offsets[o * B + i]), int(offsets[o * B + i + 1])
            assert np.all(pi[order[lo:hi]] == i) and np.all(pj[order[lo:hi]] == j)
            assert np.all(np.diff(order[lo:hi].astype(np.int64)) > 0)  # pool order inside a block


def test_blocked_training_reductions_and_exchangeable_blocks(tiny_graph):
    g = tiny_graph
    n, d, K, w, seed, count = g["n"], 32, 2, 2.5, 9, 20_000
    rng = np.random.default_rng(1)
    pool, _ = oracle.augment(8, g["offsets"], g["adj"], 40, 5, count, shuffle_seed=2)
    vertex0 = ((rng.random((n, d)) - 0.5) * 0.3).astype(np.float32)
    context0 = ((rng.random((n, d)) - 0.5) * 0.3).astype(np.float32)
    kw = dict(K=K, first_g=123, T=10 * count, lr0=0.025, lr_min_ratio=0.0, w=w, seed=seed)
    # one partition: plain sequential training, bit for bit
    one = np.zeros(n, dtype=np.uint32)
    tables = oracle.partition_alias(g["deg"], 1, one)
    v1, c1 = vertex0.copy(), context0.copy()
    oracle.train_blocked(v1, c1, pool, B=1, part=one, tables=tables, **kw)
    v2, c2 = vertex0.copy(), context0.copy()
    oracle.train(v2, c2, pool, thresh=tables[2], alias=tables[3], **kw)
    assert np.array_equal(v1, v2) and np.array_equal(c1, c2)
    # several partitions: the blocks of a sub-episode may be taken in any order (Def. 1: they share no row)
    B = 4
    part = oracle.zigzag_partition(g["deg"], B)
    tables = oracle.partition_alias(g["deg"], B, part)
    negatives = oracle.draw_negatives_partitioned(seed, 123, pool[:, 1].copy(), K, part, tables)
    order, offsets = oracle.block_order(pool, B, part)
    results = []
    for flip in (False, True):
        turn = []
        for o in range(B):
            blocks = list(range(B))[::-1] if flip else list(range(B))
            turn += [order[int(offsets[o * B + i]):int(offsets[o * B + i + 1])] for i in blocks]
        v, c = vertex0.copy(), context0.copy()
        oracle.train(v, c, pool, thresh=tables[2], alias=tables[3], negatives=negatives, order=np.concatenate(turn), **kw)
        results.append((v, c))
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    v3, c3 = vertex0.copy(), context0.copy()
    oracle.train_blocked(v3, c3, pool, B=B, part=part, tables=tables, **kw)
    assert np.array_equal(v3, results[0][0]) and np.array_equal(c3, results[0][1])
    # and the order of sub-episodes does matter (rows are shared across them): the schedule is not a no-op
    turn = [order[int(offsets[b]):int(offsets[b + 1])] for b in range(B * B)][::-1]
    v4, c4 = vertex0.copy(), context0.copy()
    oracle.train(v4, c4, pool, thresh=tables[2], alias=tables[3], negatives=negatives, order=np.concatenate(turn), **kw)
    assert not np.array_equal(v4, v3)
