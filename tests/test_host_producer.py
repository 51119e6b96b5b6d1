"""Host producer of pools (parallel online augmentation + pseudo shuffle, Sec. 3.1): pins of the
oracle's pseudo shuffle, and bit-exact agreement of the library's producer with the oracle.
Needs no GPU: the producer is pure host code."""
import numpy as np
import pytest

import oracle
import workloads as W


@pytest.fixture(scope="module")
def gv():
    import os

    import paper_1903_00757_amd as gv

    if not os.path.exists(gv.LIB_PATH):
        from paper_1903_00757_amd import build

        build.build()
    gv.load()
    return gv


def test_pseudo_shuffle_is_the_round_robin_scatter():
    count, s = 23, 5
    pairs = np.stack([np.arange(count, dtype=np.uint32), np.arange(count, dtype=np.uint32) + 100], axis=1)
    out = oracle.pseudo_shuffle(pairs, s)
    # block b lists t = b, b+s, b+2s, ... in order; blocks follow each other
    expect = np.concatenate([np.arange(b, count, s) for b in range(s)])
    assert np.array_equal(out[:, 0], expect) and np.array_equal(out[:, 1], expect + 100)
    # a permutation for awkward sizes as well, and identity for s = 1
    for count, s in [(1, 5), (4, 5), (5, 5), (1000, 7), (190 * 3 + 17, 5)]:
        pairs = np.stack([np.arange(count, dtype=np.uint32)] * 2, axis=1)
        out = oracle.pseudo_shuffle(pairs, s)
        assert np.array_equal(np.sort(out[:, 0]), pairs[:, 0])
    assert np.array_equal(oracle.pseudo_shuffle(pairs, 1), pairs)


def test_pseudo_shuffle_separates_the_samples_of_a_walk(tiny_graph):
    g = tiny_graph
    count = 190 * 400
    pairs, _ = oracle.augment(3, g["offsets"], g["adj"], 40, 5, count)
    out = oracle.pseudo_shuffle(pairs, 5)
    # in generation order 4 of 5 neighbouring samples share their source node; afterwards
    # neighbours come from samples 5 apart in generation order and rarely do
    before = np.mean(pairs[1:, 0] == pairs[:-1, 0])
    after = np.mean(out[1:, 0] == out[:-1, 0])
    assert before > 0.7 and after < 0.25
    # every block is a subsequence of the generation order (sequential appends)
    block = count // 5
    first = out[:block]
    assert np.array_equal(first, pairs[0::5][:block])


@pytest.mark.parametrize("shuffle", [0, 1])
@pytest.mark.parametrize("threads", [1, 3, 8])
def test_library_producer_equals_oracle(gv, tiny_graph, shuffle, threads):
    g = tiny_graph
    for count, first_walk, L, s, seed in [(190 * 57 + 31, 0, 40, 5, 11), (5000, 123456789012, 40, 5, 2**40 + 7),
                                          (777, 5, 10, 2, 3), (1, 0, 40, 5, 1), (64, 9, 3, 7, 5)]:
        ref, walks = oracle.augment(seed, g["offsets"], g["adj"], L, s, count, first_walk=first_walk)
        if shuffle:
            ref = oracle.pseudo_shuffle(ref, s)
        got, used = gv.gv_augment(g["offsets"], g["adj"], seed=seed, walk_length=L, window=s, first_walk=first_walk,
                                  count=count, shuffle=shuffle, threads=threads)
        assert used == walks
        assert np.array_equal(got, ref), (count, first_walk, L, s)


def test_library_producer_on_hand_built_graphs(gv):
    # two nodes: strict alternation; star: centre and leaves alternate
    offsets, adj = W.csr_from_edges(2, np.array([0], dtype=np.uint32), np.array([1], dtype=np.uint32))
    got, _ = gv.gv_augment(offsets, adj, seed=1, count=190 * 10, shuffle=0, threads=2)
    ref, _ = oracle.augment(1, offsets, adj, 40, 5, 190 * 10)
    assert np.array_equal(got, ref)
    assert np.all(got[got[:, 0] != got[:, 1]].sum(axis=1) == 1)
    k = 6
    offsets, adj = W.csr_from_edges(k + 1, np.zeros(k, dtype=np.uint32), np.arange(1, k + 1, dtype=np.uint32))
    got, _ = gv.gv_augment(offsets, adj, seed=2, count=190 * 50, shuffle=1, threads=4)
    ref, _ = oracle.augment(2, offsets, adj, 40, 5, 190 * 50)
    assert np.array_equal(got, oracle.pseudo_shuffle(ref, 5))


def test_library_producer_rejects_bad_arguments(gv, tiny_graph):
    g = tiny_graph
    with pytest.raises(gv.GvError):
        gv.gv_augment(g["offsets"], g["adj"], seed=1, count=10, shuffle=7)
    with pytest.raises(gv.GvError):
        gv.gv_augment(g["offsets"], g["adj"], seed=1, count=10, walk_length=0)
    with pytest.raises(gv.GvError):
        gv.gv_augment(np.zeros(3, dtype=np.uint64), np.zeros(0, dtype=np.uint32), seed=1, count=10)  # no edges
    pairs, used = gv.gv_augment(g["offsets"], g["adj"], seed=1, count=0)
    assert pairs.shape == (0, 2) and used == 0


@pytest.mark.parametrize("threads", [1, 3, 8])
def test_library_redistribution_equals_oracle_block_order(gv, tiny_graph, threads):
    """The Redistribute step of the orthogonal-block schedule (Sec. 3.2, Alg. 3): the library's stable sort of a
    pool by block gives exactly the oracle's order and block boundaries, for any number of workers."""
    g = tiny_graph
    for B, count in ((2, 70_001), (5, 300_000), (8, 1), (3, 0)):
        part = oracle.zigzag_partition(g["deg"], B)
        pool, _ = oracle.augment(40 + B, g["offsets"], g["adj"], 40, 5, max(count, 1), shuffle_seed=3)
        pool = pool[:count]
        out, order, offsets = gv.gv_redistribute_pool(part, B, pool, threads=threads)
        ref_order, ref_offsets = oracle.block_order(pool, B, part)
        assert np.array_equal(order, ref_order) and np.array_equal(offsets, ref_offsets)
        assert np.array_equal(out, pool[ref_order])
    bad, _ = oracle.augment(1, g["offsets"], g["adj"], 40, 5, 1000)
    bad[5, 0] = g["n"]
    with pytest.raises(gv.GvError) as e:
        gv.gv_redistribute_pool(part, 3, bad, threads=threads)
    assert e.value.code == gv.GV_EINVAL


def weighted_tiny(g, seed=4):
    """The small graph with edge weights from {1/4, 1, 4, 9}: (offsets, adj, weights per adjacency entry)."""
    rng = np.random.default_rng(seed)
    w = rng.choice([0.25, 1.0, 4.0, 9.0], size=g["src"].size).astype(np.float32)
    order = np.argsort(np.concatenate([g["src"], g["dst"]]), kind="stable")
    return g["offsets"], g["adj"], np.ascontiguousarray(np.concatenate([w, w])[order])


@pytest.mark.parametrize("threads", [1, 5])
def test_library_weighted_producer_equals_oracle(gv, tiny_graph, threads):
    """Walk tables of a weighted graph (weighted degrees, node table, one table per adjacency row) and the pools
    walked with them (Sec. 4.3) are bit-identical to the oracle's, pseudo-shuffled or not, for any worker count."""
    offsets, adj, weights = weighted_tiny(tiny_graph)
    wdeg, *tables = gv.gv_build_walk_tables(offsets, weights)
    ref_tables = oracle.walk_tables(offsets, weights)
    assert np.array_equal(wdeg, oracle.weighted_degrees(offsets, weights))
    for got, ref in zip(tables, ref_tables):
        assert np.array_equal(got, ref)
    for count, first_walk, L, s, seed in [(190 * 41 + 3, 0, 40, 5, 13), (7000, 2**36 + 5, 40, 5, 2**41 + 1), (999, 7, 6, 3, 2)]:
        ref, ref_walks = oracle.augment_weighted(seed, offsets, adj, ref_tables, L, s, count, first_walk=first_walk)
        for shuffle in (0, 1):
            got, walks = gv.gv_augment_weighted(offsets, adj, tables, seed=seed, walk_length=L, window=s,
                                                first_walk=first_walk, count=count, shuffle=shuffle, threads=threads)
            assert walks == ref_walks
            assert np.array_equal(got, oracle.pseudo_shuffle(ref, s) if shuffle else ref)
    # unit weights: the steps are the unweighted producer's
    ones = np.ones(adj.size, dtype=np.float32)
    _, *unit = gv.gv_build_walk_tables(offsets, ones)
    assert np.all(unit[2] == 0xFFFFFFFF)
    for bad in (np.where(np.arange(adj.size) == 3, -1.0, 1.0), np.zeros(adj.size)):
        with pytest.raises(gv.GvError) as e:
            gv.gv_build_walk_tables(offsets, bad.astype(np.float32))
        assert e.value.code == gv.GV_EINVAL
