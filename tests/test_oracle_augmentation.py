"""Pins of the oracle's random-walk augmentation and shuffle (Sec. 3.1, Alg. 2)."""

import numpy as np
from scipy import stats

import oracle
import workloads as W

L, S = 40, 5
PER_WALK = S * (L + 1) - S * (S + 1) // 2  # sum_{delta=1..s} (L + 1 - delta)


def _graph(n, edges):
    src = np.array([e[0] for e in edges], dtype=np.uint32)
    dst = np.array([e[1] for e in edges], dtype=np.uint32)
    return W.csr_from_edges(n, src, dst)


def _paths(pairs, walk_length=L, window=S):
    """Rebuild walk paths from the emission order (i ascending, then j)."""
    per = sum(walk_length + 1 - d for d in range(1, window + 1))
    assert pairs.shape[0] % per == 0
    out = []
    for w in range(pairs.shape[0] // per):
        block = pairs[w * per:(w + 1) * per]
        path = np.zeros(walk_length + 1, dtype=np.int64)
        pos = 0
        for i in range(walk_length + 1):
            for j in range(i + 1, min(i + window, walk_length) + 1):
                if j == i + 1:
                    path[i], path[j] = block[pos, 0], block[pos, 1]
                pos += 1
        # every emitted pair is (path[i], path[j]) of that walk
        pos = 0
        for i in range(walk_length + 1):
            for j in range(i + 1, min(i + window, walk_length) + 1):
                assert block[pos, 0] == path[i] and block[pos, 1] == path[j]
                pos += 1
        out.append(path)
    return np.array(out)


def test_pairs_per_walk_is_190():
    assert PER_WALK == 190
    offsets, adj = _graph(4, [(0, 1), (0, 2), (0, 3), (1, 2), (1, 3), (2, 3)])  # K4
    pairs, walks = oracle.augment(3, offsets, adj, L, S, 190 * 7)
    assert walks == 7
    pairs, walks = oracle.augment(3, offsets, adj, L, S, 190 * 7 + 1)
    assert walks == 8  # the last walk is cut after one pair
    for length, window in [(1, 1), (3, 2), (10, 10), (4, 9)]:
        per = sum(max(0, length + 1 - d) for d in range(1, window + 1))
        _, walks = oracle.augment(3, offsets, adj, length, window, per * 5)
        assert walks == 5


def test_two_node_path_alternates():
    offsets, adj = _graph(2, [(0, 1)])
    pairs, _ = oracle.augment(11, offsets, adj, L, S, 190 * 50)
    paths = _paths(pairs)
    assert np.all(np.abs(np.diff(paths, axis=1)) == 1)  # strict alternation 0,1,0,1...
    # pair at odd distance joins different nodes, at even distance it is a self-pair
    same = pairs[:, 0] == pairs[:, 1]
    per_walk_same = same.reshape(-1, 190).sum(axis=1)
    assert np.all(per_walk_same == (L + 1 - 2) + (L + 1 - 4))
    # departure is uniform over the two nodes (equal degree)
    starts = paths[:, 0]
    assert 10 <= starts.sum() <= 40


def test_walk_steps_follow_edges_and_truncation_keeps_prefix(tiny_graph):
    g = tiny_graph
    pairs, walks = oracle.augment(5, g["offsets"], g["adj"], L, S, 190 * 300)
    paths = _paths(pairs)
    edge_keys = set((int(a) * g["n"] + int(b)) for a, b in zip(g["src"], g["dst"]))
    edge_keys |= set((int(b) * g["n"] + int(a)) for a, b in zip(g["src"], g["dst"]))
    steps = paths[:, :-1] * g["n"] + paths[:, 1:]
    assert all(int(k) in edge_keys for k in steps.reshape(-1))
    shorter, _ = oracle.augment(5, g["offsets"], g["adj"], L, S, 12345)
    assert np.array_equal(shorter, pairs[:12345])
    # walks are addressed by number: starting at walk 100 reproduces the tail
    tail, _ = oracle.augment(5, g["offsets"], g["adj"], L, S, 190 * 200, first_walk=100)
    assert np.array_equal(tail, pairs[190 * 100:])


def test_star_graph_walks_return_to_the_centre():
    k = 6
    offsets, adj = _graph(k + 1, [(0, i) for i in range(1, k + 1)])
    pairs, _ = oracle.augment(2, offsets, adj, L, S, 190 * 400)
    paths = _paths(pairs)
    centre = paths == 0
    assert np.all(centre[:, :-1] ^ centre[:, 1:])  # centre and leaf alternate
    # departure proportional to degree: centre has k of 2k half-edges
    assert abs(centre[:, 0].mean() - 0.5) < 0.1
    # leaves visited from the centre are uniform over the k leaves
    leaves = paths[~centre]
    counts = np.bincount(leaves, minlength=k + 1)[1:]
    assert stats.chisquare(counts).pvalue > 1e-3


def test_ring_displacement_is_binomial():
    n = 101
    offsets, adj = _graph(n, [(i, (i + 1) % n) for i in range(n)])
    pairs, _ = oracle.augment(8, offsets, adj, L, S, 190 * 3000)
    paths = _paths(pairs)
    steps = (np.diff(paths, axis=1) + n + 1) % n - 1  # -1 or +1
    assert set(np.unique(steps)) == {-1, 1}
    disp = steps[:, :S].sum(axis=1)  # displacement after s steps: 2*Binomial(s, 1/2) - s
    observed = np.array([(disp == 2 * k - S).sum() for k in range(S + 1)])
    expected = stats.binom.pmf(np.arange(S + 1), S, 0.5) * disp.size
    assert stats.chisquare(observed, expected).pvalue > 1e-3
    # successive steps are independent
    assert abs(np.corrcoef(steps[:, 3], steps[:, 4])[0, 1]) < 0.06


def test_source_marginal_is_proportional_to_degree(tiny_graph):
    """Departure proportional to degree is the stationary law of the walk, so every
    position of the path, hence the source of every pair, is degree-distributed."""
    g = tiny_graph
    count = 190 * 20000
    pairs, _ = oracle.augment(21, g["offsets"], g["adj"], L, S, count)
    paths = _paths(pairs[:190 * 2000])
    expected_p = g["deg"] / g["deg"].sum()
    # walks are independent of each other: test the departure node and the end node
    for position in (0, L):
        nodes = pairs.reshape(-1, 190, 2)[:, 0, 0] if position == 0 else pairs.reshape(-1, 190, 2)[:, -1, 1]
        counts = np.bincount(nodes, minlength=g["n"]).astype(np.float64)
        order = np.argsort(expected_p)
        # merge low-expectation nodes into bins of expected count >= 5
        exp_sorted = expected_p[order] * nodes.size
        cnt_sorted = counts[order]
        bins = np.floor(np.cumsum(exp_sorted) / 8.0).astype(np.int64)
        e = np.bincount(bins, weights=exp_sorted)
        o = np.bincount(bins, weights=cnt_sorted)
        keep = e >= 5
        e, o = np.append(e[keep], e[~keep].sum()), np.append(o[keep], o[~keep].sum())
        e, o = e[e > 0], o[e > 0]
        assert stats.chisquare(o, e * o.sum() / e.sum()).pvalue > 1e-3
    assert paths.shape == (2000, L + 1)


def test_shuffle_is_a_permutation_and_uniform():
    pairs = np.stack([np.arange(1000, dtype=np.uint32), np.arange(1000, dtype=np.uint32) + 5000], axis=1)
    out = oracle.shuffle(4, pairs)
    assert np.array_equal(np.sort(out[:, 0]), pairs[:, 0])
    assert np.array_equal(out[:, 1], out[:, 0] + 5000)  # pairs stay together
    assert not np.array_equal(out, pairs)
    assert np.array_equal(oracle.shuffle(4, pairs), out)
    # position of item 0 over many seeds is uniform over 4 slots
    small = np.stack([np.arange(4, dtype=np.uint32)] * 2, axis=1)
    where = [int(np.where(oracle.shuffle(s, small)[:, 0] == 0)[0][0]) for s in range(2000)]
    assert stats.chisquare(np.bincount(where, minlength=4)).pvalue > 1e-3
    # all 24 orders of 4 items occur
    orders = {tuple(oracle.shuffle(s, small)[:, 0]) for s in range(2000)}
    assert len(orders) == 24


def test_input_pools_have_the_same_structure(tiny_graph):
    """The numpy pool recipe used for benchmark inputs has the walk structure the
    oracle's augmentation has: 190 pairs per walk, steps along edges, degree marginal."""
    g = tiny_graph
    pool = W.walk_pool(g["offsets"], g["adj"], 190 * 500, L, S, seed=3, shuffle=False)
    # numpy recipe groups by distance; distance-1 pairs are edges
    first = pool[: 500 * L]
    keys = set((int(a) * g["n"] + int(b)) for a, b in zip(g["src"], g["dst"]))
    keys |= set((int(b) * g["n"] + int(a)) for a, b in zip(g["src"], g["dst"]))
    assert all(int(a) * g["n"] + int(b) in keys for a, b in first)
    big = W.walk_pool(g["offsets"], g["adj"], 2_000_000, L, S, seed=4)
    share = np.bincount(big[:, 0], minlength=g["n"]) / big.shape[0]
    hubs = np.argsort(g["deg"])[-20:]
    np.testing.assert_allclose(share[hubs], (g["deg"] / g["deg"].sum())[hubs], rtol=0.15)
