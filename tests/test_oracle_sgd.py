"""Pins of the oracle's SGD step, schedule, loss and evaluation (CPU)."""
import os

import numpy as np
import pytest
from scipy.special import log_expit

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _identity_table(n):
    return np.full(n, 0xFFFFFFFF, dtype=np.uint32), np.arange(n, dtype=np.uint32)


def _step(vertex, context, pairs, negatives, *, K, w, lr0=0.025, first_g=0, T=10**9, lr_min=0.0):
    v, c = vertex.copy(), context.copy()
    thresh, alias = _identity_table(v.shape[0])
    oracle.train(v, c, pairs, K=K, first_g=first_g, T=T, lr0=lr0, lr_min_ratio=lr_min, w=w, seed=0,
                 thresh=thresh, alias=alias, negatives=negatives)
    return v, c


def _loss64(vertex, context, u, v, negs, w):
    """-log sigmoid(x_u.c_v) - w sum_k log sigmoid(-x_u.c_k) through scipy's log_expit."""
    x = vertex[u]
    out = -log_expit(x @ context[v])
    for k in negs:
        out -= w * log_expit(-(x @ context[k]))
    return out


@pytest.mark.parametrize("K,w", [(1, 5.0), (1, 1.0), (5, 1.0), (5, 5.0), (3, 2.5)])
@pytest.mark.parametrize("collide", [False, True])
def test_step_is_a_gradient_step_of_the_logistic_loss(K, w, collide):
    """(new - old) / lr equals minus the central finite difference of the loss,
    for every element of every touched row, duplicates within the sample included."""
    rng = np.random.default_rng(K * 10 + int(w) + collide)
    n, d = 12, 8
    # values exactly representable in fp32 so that fp64 differences see the same point
    vertex = (rng.integers(-64, 64, size=(n, d)) / 64.0).astype(np.float32)
    context = (rng.integers(-64, 64, size=(n, d)) / 64.0).astype(np.float32)
    u, v = 3, 7
    negs = list(rng.choice([i for i in range(n) if i not in (u, v)], size=K, replace=False))
    if collide:
        negs[0] = v  # negative equals the positive context row
        if K >= 3:
            negs[2] = negs[1]  # and two negatives coincide
    lr0 = 2.0**-6
    nv, nc = _step(vertex, context, np.array([[u, v]]), np.array(negs), K=K, w=w, lr0=lr0)
    V64, C64 = vertex.astype(np.float64), context.astype(np.float64)
    h = 2.0**-20
    for mat, new, rows in ((V64, nv, [u]), (C64, nc, sorted(set([v] + negs)))):
        for r in rows:
            for j in range(d):
                old = mat[r, j]
                mat[r, j] = old + h
                up = _loss64(V64, C64, u, v, negs, w)
                mat[r, j] = old - h
                down = _loss64(V64, C64, u, v, negs, w)
                mat[r, j] = old
                grad = (up - down) / (2 * h)
                moved = (float(new[r, j]) - old) / lr0
                assert abs(moved + grad) < 3e-5 * max(1.0, abs(grad)), (r, j, moved, grad)
    # rows that the sample does not name are untouched
    others_v = [i for i in range(n) if i != u]
    others_c = [i for i in range(n) if i not in [v] + negs]
    assert np.array_equal(nv[others_v], vertex[others_v])
    assert np.array_equal(nc[others_c], context[others_c])


def test_first_step_closed_form():
    """With context = 0 every score is 0 and sigmoid is 1/2: c_v = lr/2 x_u,
    c_neg = -lr w/2 x_u, x_u unchanged."""
    rng = np.random.default_rng(0)
    n, d, lr0, w = 6, 16, 0.5, 5.0
    vertex = (rng.integers(-128, 128, size=(n, d)) / 256.0).astype(np.float32)
    context = np.zeros((n, d), dtype=np.float32)
    nv, nc = _step(vertex, context, np.array([[1, 2]]), np.array([4]), K=1, w=w, lr0=lr0)
    assert np.array_equal(nv, vertex)
    np.testing.assert_array_equal(nc[2], (0.5 * lr0) * vertex[1])
    np.testing.assert_array_equal(nc[4], (-0.5 * lr0 * w) * vertex[1])
    assert not nc[[0, 1, 3, 5]].any()
    # negative == positive row with w = 1: the two pulls cancel exactly
    nv, nc = _step(vertex, context, np.array([[1, 2]]), np.array([2]), K=1, w=1.0, lr0=lr0)
    assert np.array_equal(nv, vertex) and not nc.any()
    # same with w = 5: net coefficient lr (1/2 - 5/2) = -2 lr
    nv, nc = _step(vertex, context, np.array([[1, 2]]), np.array([2]), K=1, w=5.0, lr0=lr0)
    np.testing.assert_array_equal(nc[2], (-2.0 * lr0) * vertex[1])


def test_zero_learning_rate_is_identity():
    rng = np.random.default_rng(1)
    vertex = rng.standard_normal((20, 8)).astype(np.float32)
    context = rng.standard_normal((20, 8)).astype(np.float32)
    pairs = rng.integers(20, size=(50, 2)).astype(np.uint32)
    negs = rng.integers(20, size=(50, 2)).astype(np.uint32)
    nv, nc = _step(vertex, context, pairs, negs, K=2, w=1.0, lr0=0.0)
    assert np.array_equal(nv, vertex) and np.array_equal(nc, context)
    # last sample of a schedule that decays to zero: g = T means lr = 0
    nv, nc = _step(vertex, context, pairs[:1], negs[:1], K=2, w=1.0, lr0=0.1, first_g=1000, T=1000)
    assert np.array_equal(nv, vertex) and np.array_equal(nc, context)


def test_sequential_semantics_second_sample_sees_first():
    """Two samples through one call equal two calls (state carried in the matrices),
    and differ from applying both to the initial state."""
    rng = np.random.default_rng(2)
    vertex = rng.standard_normal((5, 4)).astype(np.float32)
    context = rng.standard_normal((5, 4)).astype(np.float32)
    pairs = np.array([[0, 1], [0, 1]], dtype=np.uint32)
    negs = np.array([[2], [2]], dtype=np.uint32)
    both_v, both_c = _step(vertex, context, pairs, negs, K=1, w=5.0, T=2, lr0=0.1)
    v1, c1 = _step(vertex, context, pairs[:1], negs[:1], K=1, w=5.0, T=2, lr0=0.1, first_g=0)
    v2, c2 = _step(v1, c1, pairs[1:], negs[1:], K=1, w=5.0, T=2, lr0=0.1, first_g=1)
    assert np.array_equal(both_v, v2) and np.array_equal(both_c, c2)


def test_gradient_exchangeable_sets_commute():
    """Def. 1 (Sec. 3.2): samples that share no vertex row and no context row may
    be applied in either order with identical result; sharing a row breaks it."""
    rng = np.random.default_rng(3)
    n, d = 40, 16
    vertex = rng.standard_normal((n, d)).astype(np.float32) * 0.3
    context = rng.standard_normal((n, d)).astype(np.float32) * 0.3
    perm_u, perm_c = rng.permutation(n), rng.permutation(n)
    m = 13
    pairs = np.stack([perm_u[:m], perm_c[:m]], axis=1).astype(np.uint32)
    negs = perm_c[m:2 * m].reshape(m, 1).astype(np.uint32)
    # note: a node may appear as a vertex row of one sample and a context row of another
    thresh, alias = _identity_table(n)

    def run(order):
        v, c = vertex.copy(), context.copy()
        for i in order:  # one call per sample so that each keeps its own position g = i
            oracle.train(v, c, pairs[i:i + 1], K=1, first_g=int(i), T=100, lr0=0.1, lr_min_ratio=0.0, w=5.0,
                         seed=0, thresh=thresh, alias=alias, negatives=negs[i:i + 1])
        return v, c

    a = run(range(m))
    b = run(rng.permutation(m))
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    pairs[5, 0] = pairs[2, 0]  # now samples 2 and 5 share a vertex row
    a = run(range(m))
    b = run(list(range(m))[::-1])
    assert not np.array_equal(a[0], b[0])


def test_learning_rate_schedule():
    """Initial rate 0.025 with linear decay (Sec. 4.3)."""
    assert oracle.learning_rate(0.025, 0.0, 0, 1000) == np.float32(0.025)
    assert oracle.learning_rate(0.025, 0.0, 500, 1000) == np.float32(np.float64(np.float32(0.025)) * 0.5)
    assert oracle.learning_rate(0.025, 0.0, 1000, 1000) == 0.0
    assert oracle.learning_rate(0.025, 0.0, 1500, 1000) == 0.0  # never negative past the planned total
    assert oracle.learning_rate(0.025, 1e-4, 999_999, 1_000_000) == np.float32(np.float64(np.float32(0.025)) * np.float64(np.float32(1e-4)))
    T = 2_000_000_000
    g = 1_234_567_891
    expect = np.float32(np.float64(np.float32(0.025)) * (1.0 - g / T))
    assert oracle.learning_rate(0.025, 0.0, g, T) == expect
    # strictly decreasing over coarse steps
    vals = [oracle.learning_rate(0.025, 0.0, g, T) for g in range(0, T, T // 50)]
    assert all(a > b for a, b in zip(vals, vals[1:]))


def test_loss_closed_forms(tiny_graph, tiny_alias):
    thresh, alias = tiny_alias
    n, d = tiny_graph["n"], 16
    pairs = np.stack([tiny_graph["src"][:2000], tiny_graph["dst"][:2000]], axis=1)
    zeros = np.zeros((n, d), dtype=np.float32)
    for K, w in [(1, 5.0), (5, 1.0), (2, 0.0)]:
        got = oracle.loss(zeros, zeros, pairs, K=K, w=w, seed=5, thresh=thresh, alias=alias)
        assert abs(got - (1 + w * K) * np.log(2.0)) < 1e-12
    rng = np.random.default_rng(4)
    vertex = rng.standard_normal((n, d)).astype(np.float32)
    context = rng.standard_normal((n, d)).astype(np.float32) * 3  # scores reach |30|: exercises both log branches
    K, w = 3, 2.0
    got = oracle.loss(vertex, context, pairs, K=K, w=w, seed=5, thresh=thresh, alias=alias)
    negs = oracle.draw_negatives(5, 0, pairs.shape[0], K, thresh, alias, stream=oracle.STREAM_EVAL)
    V, Cx = vertex.astype(np.float64), context.astype(np.float64)
    pos = np.einsum("ij,ij->i", V[pairs[:, 0]], Cx[pairs[:, 1]])
    expect = -log_expit(pos)
    for k in range(K):
        expect = expect - w * log_expit(-np.einsum("ij,ij->i", V[pairs[:, 0]], Cx[negs[:, k]]))
    assert abs(got - expect.mean()) < 1e-9 * abs(expect.mean())


def test_running_loss_is_the_loss_each_sample_sees_before_its_step():
    """The sum that training reports, against scipy's log-sigmoid on the rows saved before every step (a small
    graph, so samples share rows and the sequence matters), and in closed form for the first sample."""
    rng = np.random.default_rng(12)
    n, d, K, w, count = 12, 8, 2, 3.0, 200
    vertex = rng.standard_normal((n, d)).astype(np.float32)
    context = rng.standard_normal((n, d)).astype(np.float32)
    pairs = rng.integers(n, size=(count, 2)).astype(np.uint32)
    negs = rng.integers(n, size=(count, K)).astype(np.uint32)
    negs[3, 0] = pairs[3, 1]  # a negative that is the positive row: both terms count
    kw = dict(K=K, T=1000, lr0=0.05, lr_min_ratio=0.0, w=w, seed=1, thresh=np.zeros(n, np.uint32),
              alias=np.zeros(n, np.uint32))
    expect = 0.0
    v, c = vertex.copy(), context.copy()
    for i in range(count):
        x = v[pairs[i, 0]].astype(np.float64)
        expect += -log_expit(x @ c[pairs[i, 1]].astype(np.float64))
        for k in range(K):
            expect += -w * log_expit(-(x @ c[negs[i, k]].astype(np.float64)))
        assert oracle.train(v, c, pairs[i:i + 1], first_g=i, negatives=negs[i:i + 1], **kw) is None
    v2, c2 = vertex.copy(), context.copy()
    got = oracle.train(v2, c2, pairs, first_g=0, negatives=negs, return_loss=True, **kw)
    assert abs(got - expect) < 1e-10 * expect
    assert np.array_equal(v, v2) and np.array_equal(c, c2)  # asking for the sum changes nothing
    zeros = np.zeros((n, d), dtype=np.float32)
    first = oracle.train(vertex.copy(), zeros.copy(), pairs[:1], first_g=0, negatives=negs[:1], return_loss=True, **kw)
    assert abs(first - (1 + w * K) * np.log(2.0)) < 1e-12


def test_training_lowers_the_loss_it_descends(tiny_graph, tiny_alias):
    thresh, alias = tiny_alias
    g = tiny_graph
    d = 32
    pool, _ = oracle.augment(101, g["offsets"], g["adj"], 40, 5, 1_500_000, shuffle_seed=7)
    evalp, _ = oracle.augment(102, g["offsets"], g["adj"], 40, 5, 20_000, shuffle_seed=8)
    vertex, context = oracle.init_embeddings(1, g["n"], d)
    before = oracle.loss(vertex, context, evalp, K=1, w=5.0, seed=3, thresh=thresh, alias=alias)
    assert abs(before - 6 * np.log(2.0)) < 1e-9
    oracle.train(vertex, context, pool, K=1, first_g=0, T=pool.shape[0], lr0=0.1, lr_min_ratio=0.0, w=5.0,
                 seed=1234, thresh=thresh, alias=alias)
    after = oracle.loss(vertex, context, evalp, K=1, w=5.0, seed=3, thresh=thresh, alias=alias)
    assert after < 0.8 * before


def test_internal_negative_draws_match_explicit_ones(tiny_alias):
    thresh, alias = tiny_alias
    n, d = thresh.size, 8
    rng = np.random.default_rng(5)
    vertex = rng.standard_normal((n, d)).astype(np.float32) * 0.1
    context = rng.standard_normal((n, d)).astype(np.float32) * 0.1
    pairs = rng.integers(n, size=(500, 2)).astype(np.uint32)
    first_g = 2**33 + 11
    negs = oracle.draw_negatives(77, first_g, 500, 2, thresh, alias)
    a_v, a_c = vertex.copy(), context.copy()
    oracle.train(a_v, a_c, pairs, K=2, first_g=first_g, T=2**34, lr0=0.05, lr_min_ratio=0.0, w=1.0, seed=77,
                 thresh=thresh, alias=alias)
    b_v, b_c = vertex.copy(), context.copy()
    oracle.train(b_v, b_c, pairs, K=2, first_g=first_g, T=2**34, lr0=0.05, lr_min_ratio=0.0, w=1.0, seed=77,
                 thresh=thresh, alias=alias, negatives=negs)
    assert np.array_equal(a_v, b_v) and np.array_equal(a_c, b_c)


def test_init_embeddings():
    n, d, seed = 300, 128, 42
    vertex, context = oracle.init_embeddings(seed, n, d)
    assert not context.any()
    assert np.abs(vertex).max() < 0.5 / d and np.abs(vertex).max() > 0.49 / d
    assert abs(vertex.mean()) < 3 * (1 / d) / np.sqrt(12 * n * d)
    assert abs(vertex.std() - (1 / d) / np.sqrt(12)) < 0.02 * (1 / d)
    # element (row, col) comes from word col%4 of Philox block (row, 0, col/4, stream 1)
    for row, col in [(0, 0), (7, 5), (299, 127)]:
        r = oracle.philox4x32_10([row, 0, col // 4, 1], [seed, 0])
        expect = np.float32(((float(r[col % 4]) + 0.5) / 2.0**32 - 0.5) / d)
        assert vertex[row, col] == expect


def test_auc_rank_statistic():
    rng = np.random.default_rng(6)
    pos = np.round(rng.standard_normal(60) + 0.5, 1)  # rounding creates ties
    neg = np.round(rng.standard_normal(80), 1)
    brute = np.mean([(1.0 if p > q else 0.5 if p == q else 0.0) for p in pos for q in neg])
    assert abs(oracle.auc(pos, neg) - brute) < 1e-12
    assert oracle.auc([2.0, 3.0], [0.0, 1.0]) == 1.0
    assert oracle.auc([0.0, 1.0], [2.0, 3.0]) == 0.0
    assert oracle.auc([1.0, 1.0], [1.0, 1.0, 1.0]) == 0.5


def test_cosine():
    rng = np.random.default_rng(7)
    vertex = rng.standard_normal((30, 12)).astype(np.float32)
    vertex[5] = 0
    a = rng.integers(30, size=100).astype(np.uint32)
    b = rng.integers(30, size=100).astype(np.uint32)
    got = oracle.cosine(vertex, a, b)
    V = vertex.astype(np.float64)
    with np.errstate(invalid="ignore", divide="ignore"):
        expect = np.einsum("ij,ij->i", V[a], V[b]) / (np.linalg.norm(V[a], axis=1) * np.linalg.norm(V[b], axis=1))
    expect[(a == 5) | (b == 5)] = 0.0
    np.testing.assert_allclose(got, expect, rtol=1e-12, atol=1e-15)
    assert np.all(np.abs(got[a == b][a[a == b] != 5] - 1.0) < 1e-12)


def test_planted_partition_is_recovered():
    """Ten planted communities: rows of the same community end up closer in
    cosine than rows of different ones, and held-out edges outrank random pairs."""
    n = 1000
    src, dst, community = W.planted_partition(n, 10, 10000, 50.0, seed=9)
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, 0.05, seed=10)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    deg = W.degrees(n, tr_s, tr_d)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    pool, _ = oracle.augment(11, offsets, adj, 40, 5, 2_000_000, shuffle_seed=12)
    vertex, context = oracle.init_embeddings(13, n, 32)
    oracle.train(vertex, context, pool, K=1, first_g=0, T=pool.shape[0], lr0=0.025, lr_min_ratio=0.0, w=5.0,
                 seed=14, thresh=thresh, alias=alias)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=15)
    assert oracle.link_prediction_auc(vertex, te_s, te_d, na, nb) > 0.8
    a, b = W.uniform_negative_pairs(n, 5000, seed=16)
    cos = oracle.cosine(vertex, a, b)
    same = community[a] == community[b]
    assert cos[same].mean() > cos[~same].mean() + 0.2


def test_table1_sizes_fix_the_layout():
    """Table 1 (Sec. 2.2): 4-byte ids, 8-byte samples, 4-byte embedding elements."""
    with open(os.path.join(GOLDEN, "table1_memory.txt")) as f:
        rows = [line.split() for line in f if line.strip() and not line.startswith("#")]
    assert len(rows) == 5
    for name, count, width, printed, unit in rows:
        size = int(count) * int(width) / (2**20 if unit == "MB" else 2**30)
        digits = len(printed.split(".")[1]) if "." in printed else 0
        assert round(size, digits) == float(printed), name
    pool, _ = oracle.augment(0, *W.csr_from_edges(2, np.array([0], dtype=np.uint32), np.array([1], dtype=np.uint32)),
                             40, 5, 10)
    assert pool.dtype == np.uint32 and pool.itemsize * pool.shape[1] == 8
    v, c = oracle.init_embeddings(0, 4, 8)
    assert v.dtype == np.float32 and c.dtype == np.float32
