"""Pins of the oracle's random numbers, alias table and negative sampler (CPU)."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == out


def test_philox_is_a_bijection_like_mixer():
    # one flipped counter bit changes about half of the 128 output bits
    rng = np.random.default_rng(7)
    flips = []
    for _ in range(200):
        ctr = rng.integers(0, 2**32, size=4, dtype=np.uint64).astype(np.uint32)
        key = rng.integers(0, 2**32, size=2, dtype=np.uint64).astype(np.uint32)
        a = oracle.philox4x32_10(ctr, key)
        word, bit = int(rng.integers(4)), int(rng.integers(32))
        ctr2 = ctr.copy()
        ctr2[word] ^= np.uint32(1 << bit)
        b = oracle.philox4x32_10(ctr2, key)
        flips.append(sum(bin(int(x) ^ int(y)).count("1") for x, y in zip(a, b)))
    assert 58 < np.mean(flips) < 70
    # distinct counters give distinct outputs
    outs = {tuple(oracle.philox4x32_10([i, 0, 0, 0], [1, 2])) for i in range(2000)}
    assert len(outs) == 2000


def test_negative_stream_uses_counter_layout():
    # draw g of stream s with sub-index k is Philox(ctr=(g_lo, g_hi, k, s), key=(seed_lo, seed_hi)):
    # with the identity table the outcome is the bucket floor(R*n/2^64), R = (r0 << 32) | r1
    n = 1000
    thresh = np.full(n, 0xFFFFFFFF, dtype=np.uint32)
    alias = np.arange(n, dtype=np.uint32)
    seed = 0x0123456789ABCDEF
    for g in (0, 5, 2**32 + 3, 2**40 + 17):
        got = oracle.draw_negatives(seed, g, 1, 3, thresh, alias)[0]
        for k in range(3):
            r = oracle.philox4x32_10([g & 0xFFFFFFFF, g >> 32, k, 0], [seed & 0xFFFFFFFF, seed >> 32])
            R = (int(r[0]) << 32) | int(r[1])
            assert int(got[k]) == (R * n) >> 64  # identity table: bucket j always yields j


def _table_mass(thresh, alias):
    """Probability of every outcome implied by the integer table (exact in fp64 up to 2^-53)."""
    n = thresh.size
    t = thresh.astype(np.float64)
    mass = t.copy()
    np.add.at(mass, alias, 4294967296.0 - t)
    return mass / (n * 4294967296.0)


def test_alias_hand_built_tables():
    # equal weights: everything accepts itself
    thresh, alias = oracle.alias_build(np.ones(4))
    assert list(thresh) == [0xFFFFFFFF] * 4 and list(alias) == [0, 1, 2, 3]
    # weights 1:3 on two nodes: p = (0.5, 1.5); node 0 keeps 1/2 and aliases to node 1
    thresh, alias = oracle.alias_build(np.array([1.0, 3.0]))
    assert list(thresh) == [2**31, 0xFFFFFFFF] and list(alias) == [1, 1]
    # weights 0,1,1: node 0 is never drawn
    thresh, alias = oracle.alias_build(np.array([0.0, 1.0, 1.0]))
    assert thresh[0] == 0 and alias[0] in (1, 2)
    m = _table_mass(thresh, alias)
    assert m[0] == 0 and abs(m[1] - 0.5) < 1e-9 and abs(m[2] - 0.5) < 1e-9
    # 4 nodes 1,2,3,10 -> p = .25,.5,.75,2.5: smalls popped from the top (2,1,0), all alias to 3
    thresh, alias = oracle.alias_build(np.array([1.0, 2.0, 3.0, 10.0]))
    assert list(alias) == [3, 3, 3, 3]
    assert list(thresh) == [2**30, 2**31, 3 * 2**30, 0xFFFFFFFF]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_alias_table_reproduces_weights_exactly(seed):
    rng = np.random.default_rng(seed)
    n = 5000
    q = rng.pareto(1.2, size=n) + (rng.random(n) < 0.1) * 50.0
    q[rng.integers(n, size=50)] = 0.0
    thresh, alias = oracle.alias_build(q)
    mass = _table_mass(thresh, alias)
    target = q / q.sum()
    # every threshold is floored to a multiple of 2^-32 of a bucket; a node can collect the
    # remainder of many buckets, hence the n * 2^-32 / n = 2^-32 per aliasing bucket bound
    assert np.max(np.abs(mass - target)) <= (n + 2) * 2.0**-32 / n + 1e-12
    assert np.all(mass[q == 0] == 0)
    assert alias.max() < n


def test_alias_rejects_bad_weights():
    with pytest.raises(ValueError):
        oracle.alias_build(np.zeros(5))
    with pytest.raises(ValueError):
        oracle.alias_build(np.array([1.0, -1.0]))
    with pytest.raises(ValueError):
        oracle.alias_build(np.array([1.0, np.nan]))


def test_degree_weights_are_three_quarter_power():
    deg = np.array([0, 1, 2, 3, 16, 81, 10_000, 4_000_000_000], dtype=np.uint32)
    q = oracle.degree_weights(deg)
    assert q[0] == 0 and q[1] == 1 and q[4] == 8 and q[5] == 27 and q[6] == 1000
    np.testing.assert_allclose(q, deg.astype(np.float64) ** 0.75, rtol=1e-15)


def test_tiny_graph_table_mass(tiny_graph, tiny_alias):
    thresh, alias = tiny_alias
    q = tiny_graph["deg"].astype(np.float64) ** 0.75
    mass = _table_mass(thresh, alias)
    assert np.max(np.abs(mass - q / q.sum())) <= 2.0**-31


def test_negative_draws_follow_degree_power(tiny_graph, tiny_alias):
    """Chi-squared goodness of fit of 10^7 draws against deg^0.75 (Sec. 4.3)."""
    thresh, alias = tiny_alias
    n = tiny_graph["n"]
    draws = oracle.draw_negatives(1234, 0, 10_000_000, 1, thresh, alias).reshape(-1)
    assert draws.max() < n
    counts = np.bincount(draws, minlength=n).astype(np.float64)
    q = tiny_graph["deg"].astype(np.float64) ** 0.75
    expected = q / q.sum() * draws.size
    assert expected.min() > 5  # every bin is well populated at this sample size
    chi2 = ((counts - expected) ** 2 / expected).sum()
    p = stats.chi2.sf(chi2, df=n - 1)
    assert p > 1e-3, (chi2, p)
    # a table built for the wrong power is rejected by the same test
    wrong = tiny_graph["deg"].astype(np.float64)
    expected_wrong = wrong / wrong.sum() * draws.size
    chi2_wrong = ((counts - expected_wrong) ** 2 / expected_wrong).sum()
    assert stats.chi2.sf(chi2_wrong, df=n - 1) < 1e-12


def test_negative_draws_are_a_pure_function_of_position(tiny_alias):
    thresh, alias = tiny_alias
    a = oracle.draw_negatives(9, 1000, 64, 5, thresh, alias)
    b = oracle.draw_negatives(9, 1010, 10, 5, thresh, alias)
    assert np.array_equal(a[10:20], b)
    c = oracle.draw_negatives(10, 1000, 64, 5, thresh, alias)
    assert not np.array_equal(a, c)
    e = oracle.draw_negatives(9, 1000, 64, 5, thresh, alias, stream=oracle.STREAM_EVAL)
    assert not np.array_equal(a, e)
    # the K draws of one sample differ from each other (sub-index enters the counter)
    assert np.mean(a[:, 0] == a[:, 1]) < 0.1
