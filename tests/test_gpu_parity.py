"""Parity of the HIP path against the CPU oracle, through the C boundary (needs a GPU)."""
import contextlib
import os

import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu

LR0 = 0.025


@pytest.fixture(scope="module")
def gv():
    import paper_1903_00757_amd as gv

    gv.load()
    return gv


@contextlib.contextmanager
def context_for(gv, **kw):
    ctx = gv.gv_create(**kw)
    try:
        yield ctx
    finally:
        gv.gv_destroy(ctx)


def rel_errors(got, ref):
    """(Frobenius relative error, max-abs error relative to the largest entry)."""
    diff = got.astype(np.float64) - ref.astype(np.float64)
    fro = np.linalg.norm(diff) / max(np.linalg.norm(ref.astype(np.float64)), 1e-300)
    mx = np.abs(diff).max() / max(np.abs(ref).max(), 1e-300)
    return fro, mx


def random_embeddings(n, d, seed, scale=0.3):
    rng = np.random.default_rng(seed)
    vertex = ((rng.random((n, d)) - 0.5) * scale).astype(np.float32)
    context = ((rng.random((n, d)) - 0.5) * scale).astype(np.float32)
    return vertex, context


# --------------------------------------------------------------------------- tables and streams
@pytest.mark.parametrize("power", [0.75, 1.0, 0.0])
def test_alias_table_is_bit_identical(gv, tiny_graph, power):
    g = tiny_graph
    deg = g["deg"].copy()
    deg[::97] = 0  # isolated nodes
    with context_for(gv, dim=64, num_neg=1, total_samples=1, pool_capacity=1) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, power)
        thresh, alias = gv.gv_get_alias(ctx, g["n"])
    q = {0.75: oracle.degree_weights(deg), 1.0: deg.astype(np.float64), 0.0: np.ones(g["n"])}[power]
    ref_t, ref_a = oracle.alias_build(q)
    assert np.array_equal(thresh, ref_t) and np.array_equal(alias, ref_a)


def test_set_graph_counts_degrees(gv, tiny_graph, tiny_alias):
    g = tiny_graph
    with context_for(gv, dim=64, num_neg=1, total_samples=1, pool_capacity=1) as ctx:
        gv.gv_set_graph(ctx, g["n"], g["src"], g["dst"])
        gv.gv_build_alias(ctx, 0.75)
        thresh, alias = gv.gv_get_alias(ctx, g["n"])
    assert np.array_equal(thresh, tiny_alias[0]) and np.array_equal(alias, tiny_alias[1])


@pytest.mark.parametrize("d", [64, 96, 128, 512])
def test_initial_embeddings_are_bit_identical(gv, d):
    n = 3001
    with context_for(gv, dim=d, num_neg=1, total_samples=1, pool_capacity=1) as ctx:
        gv.gv_set_degrees(ctx, np.ones(n, dtype=np.uint32))
        gv.gv_init_embeddings(ctx, 0xDEADBEEF12345)
        vertex = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
        context = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
        tail = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 5, d, row0=n - 5)
    ref_v, ref_c = oracle.init_embeddings(0xDEADBEEF12345, n, d)
    assert np.array_equal(vertex, ref_v) and np.array_equal(context, ref_c)
    assert np.array_equal(tail, ref_v[-5:])


@pytest.mark.parametrize("K,first_g,count", [(1, 0, 1 << 22), (5, 0, 300_001), (1, 2**32 - 1000, 5000),
                                             (3, 2**45 + 12345, 70_000), (1, 7, 1), (2, 0, 63)])
def test_negative_draws_are_bit_identical(gv, tiny_graph, tiny_alias, K, first_g, count):
    g = tiny_graph
    seed = 0x9E3779B97F4A7C15
    with context_for(gv, dim=64, num_neg=K, total_samples=1, pool_capacity=1, seed=seed) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        got = gv.gv_draw_negatives(ctx, first_g, count, K)
    ref = oracle.draw_negatives(seed, first_g, count, K, *tiny_alias)
    assert np.array_equal(got, ref)


def test_negative_draws_large_table(gv):
    """n well above 2^16 with a skewed degree sequence (wide alias jumps)."""
    n = 3_000_017
    rng = np.random.default_rng(3)
    deg = np.minimum(rng.zipf(1.8, size=n), 10**6).astype(np.uint32)
    deg[rng.integers(n, size=1000)] = 0
    with context_for(gv, dim=64, num_neg=2, total_samples=1, pool_capacity=1, seed=5) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        thresh, alias = gv.gv_get_alias(ctx, n)
        got = gv.gv_draw_negatives(ctx, 123, 200_000, 2)
    ref_t, ref_a = oracle.alias_build(oracle.degree_weights(deg))
    assert np.array_equal(thresh, ref_t) and np.array_equal(alias, ref_a)
    assert np.array_equal(got, oracle.draw_negatives(5, 123, 200_000, 2, ref_t, ref_a))
    assert got.max() < n and np.all(deg[got.reshape(-1)] > 0)


# --------------------------------------------------------------------------- deterministic mode
def run_deterministic(gv, n, deg, d, K, w, pools, vertex, context, T, seed, lr_min=0.0, device_pool=False):
    cap = max(p.shape[0] for p in pools)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_DETERMINISTIC, total_samples=T, seed=seed,
                     pool_capacity=max(cap, 1), lr0=LR0, lr_min_ratio=lr_min) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        for p in pools:
            gv.gv_push_pool(ctx, p)
            gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        stats = gv.gv_get_stats(ctx)
        return (gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d), gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d),
                stats)


def run_oracle(deg, K, w, pools, vertex, context, T, seed, lr_min=0.0):
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    v, c = vertex.copy(), context.copy()
    g = 0
    for p in pools:
        oracle.train(v, c, p, K=K, first_g=g, T=T, lr0=LR0, lr_min_ratio=lr_min, w=w, seed=seed,
                     thresh=thresh, alias=alias)
        g += p.shape[0]
    return v, c


@pytest.mark.parametrize("d,K,w,count", [(128, 1, 5.0, 100_003), (64, 2, 2.5, 40_001), (256, 3, 1.0, 30_000),
                                         (512, 5, 1.0, 20_011), (128, 5, 1.0, 50_000), (128, 4, 1.25, 1),
                                         (96, 1, 5.0, 60_007), (32, 2, 2.5, 20_000), (160, 1, 5.0, 20_000),
                                         (480, 5, 1.0, 10_000)])
def test_deterministic_mode_matches_sequential_oracle(gv, tiny_graph, d, K, w, count):
    g = tiny_graph
    pool, _ = oracle.augment(100 + d + K, g["offsets"], g["adj"], 40, 5, count, shuffle_seed=9)
    vertex, context = random_embeddings(g["n"], d, seed=d + K)
    got_v, got_c, stats = run_deterministic(gv, g["n"], g["deg"], d, K, w, [pool], vertex, context, count, 77)
    ref_v, ref_c = run_oracle(g["deg"], K, w, [pool], vertex, context, count, 77)
    for got, ref in ((got_v, ref_v), (got_c, ref_c)):
        fro, mx = rel_errors(got, ref)
        assert fro <= 1e-5 and mx <= 1e-4, (fro, mx)
    assert stats["samples_trained"] == count and stats["batches"] >= 1
    # the run did move the embeddings
    assert rel_errors(got_v, vertex)[0] > 1e-3 or count == 1


def test_deterministic_full_tiny_configuration(gv, tiny_graph):
    """Configuration 1 end to end: 2*10^6 samples, d=128, K=1, w=5, vertex U(-.5/d,.5/d), context 0,
    in four pools (the last one ragged); error reported against sample count."""
    g = tiny_graph
    total = 2_000_000
    pool, _ = oracle.augment(101, g["offsets"], g["adj"], 40, 5, total, shuffle_seed=7)
    cuts = [0, 1 << 19, 1 << 20, 1_500_000, total]
    pools = [pool[a:b] for a, b in zip(cuts, cuts[1:])]
    vertex, context = oracle.init_embeddings(1, g["n"], 128)
    got_v, got_c, stats = run_deterministic(gv, g["n"], g["deg"], 128, 1, 5.0, pools, vertex, context, total, 1234)
    ref_v, ref_c = run_oracle(g["deg"], 1, 5.0, pools, vertex, context, total, 1234)
    for name, got, ref in (("vertex", got_v, ref_v), ("context", got_c, ref_c)):
        fro, mx = rel_errors(got, ref)
        print(f"tiny full run: {name} fro {fro:.2e} max {mx:.2e} batches {stats['batches']}")
        assert fro <= 1e-5 and mx <= 1e-4, (name, fro, mx)


@pytest.mark.parametrize("d,K,w", [(128, 1, 5.0), (96, 3, 2.0), (512, 5, 1.0)])
def test_running_loss_of_deterministic_mode_matches_oracle(gv, tiny_graph, d, K, w):
    """gv_config.track_loss: the sum of the losses the samples saw before their steps equals the sequential
    oracle's (the rows are the same up to 1e-5, so the scores are), and asking for it changes no embedding."""
    g = tiny_graph
    n, count, seed = g["n"], 60_000, 21
    pool, _ = oracle.augment(300 + d, g["offsets"], g["adj"], 40, 5, count, shuffle_seed=3)
    vertex, context = random_embeddings(n, d, seed=d, scale=1.5)  # scores of a few units: both log branches
    thresh, alias = oracle.alias_build(oracle.degree_weights(g["deg"]))
    ref_v, ref_c = vertex.copy(), context.copy()
    expect = oracle.train(ref_v, ref_c, pool[:40_000], K=K, first_g=0, T=count, lr0=LR0, lr_min_ratio=0.0, w=w, seed=seed,
                          thresh=thresh, alias=alias, return_loss=True)
    expect += oracle.train(ref_v, ref_c, pool[40_000:], K=K, first_g=40_000, T=count, lr0=LR0, lr_min_ratio=0.0, w=w,
                           seed=seed, thresh=thresh, alias=alias, return_loss=True)
    results = []
    for track in (1, 0):
        with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_DETERMINISTIC, total_samples=count,
                         seed=seed, pool_capacity=count, lr0=LR0, track_loss=track) as ctx:
            gv.gv_set_degrees(ctx, g["deg"])
            gv.gv_build_alias(ctx, 0.75)
            gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
            gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
            for part in (pool[:40_000], pool[40_000:]):
                gv.gv_push_pool(ctx, part)
                gv.gv_train_pool(ctx)
            gv.gv_sync(ctx)
            results.append((gv.gv_get_stats(ctx), gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d),
                            gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)))
    (tracked, tv, tc), (plain, pv, pc) = results
    assert tracked["train_loss_samples"] == count and plain["train_loss_samples"] == 0 and plain["train_loss_sum"] == 0.0
    assert abs(tracked["train_loss_sum"] - expect) <= 1e-5 * expect, (tracked["train_loss_sum"], expect)
    assert np.array_equal(tv, pv) and np.array_equal(tc, pc)
    assert expect / count > 1.2 * (1 + w * K) * np.log(2.0) or expect / count < 0.8 * (1 + w * K) * np.log(2.0)  # not the value at zero scores


@pytest.mark.parametrize("policy", [(0, 2), (1, 2), (1, 3)])  # (schedule, coherence): the policies that keep contended updates
def test_running_loss_of_asynchronous_mode_tracks_oracle(gv, tiny_graph, policy):
    """The same statistic from the asynchronous kernels (pool order and tiled), whole configuration 1: every
    sample sees rows that may miss a few updates, so the sum is compared at the gate of the loss (2 %)."""
    g = tiny_graph
    n, d, K, w, seed, total = g["n"], 128, 1, 5.0, 1234, 2_000_000
    pool, _ = oracle.augment(101, g["offsets"], g["adj"], 40, 5, total, shuffle_seed=7)
    thresh, alias = oracle.alias_build(oracle.degree_weights(g["deg"]))
    ref_v, ref_c = oracle.init_embeddings(1, n, d)
    expect = oracle.train(ref_v, ref_c, pool, K=K, first_g=0, T=total, lr0=LR0, lr_min_ratio=0.0, w=w, seed=seed,
                          thresh=thresh, alias=alias, return_loss=True)
    schedule, coherence = policy
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=total, seed=seed,
                     pool_capacity=1 << 19, lr0=LR0, coherence=coherence, schedule=schedule, track_loss=1) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 1)
        for lo in range(0, total, 1 << 19):
            gv.gv_push_pool(ctx, pool[lo:lo + (1 << 19)])
            gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        stats = gv.gv_get_stats(ctx)
    got = stats["train_loss_sum"]
    print(f"running loss {policy}: {got / total:.5f} vs {expect / total:.5f}")
    assert stats["train_loss_samples"] == total
    assert abs(got - expect) <= 0.02 * expect, (got, expect)


def test_duplicate_rows_inside_a_sample(gv):
    """Three nodes: the negative often equals v (and, with K = 3, other negatives)."""
    n, d = 3, 128
    deg = np.array([1, 2, 1], dtype=np.uint32)
    rng = np.random.default_rng(1)
    pool = rng.integers(n, size=(4000, 2)).astype(np.uint32)
    for K, w in ((1, 5.0), (1, 1.0), (3, 1.0)):
        vertex, context = random_embeddings(n, d, seed=K)
        got_v, got_c, _ = run_deterministic(gv, n, deg, d, K, w, [pool], vertex, context, 4000, 3)
        ref_v, ref_c = run_oracle(deg, K, w, [pool], vertex, context, 4000, 3)
        thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
        negs = oracle.draw_negatives(3, 0, 4000, K, thresh, alias)
        assert np.mean(negs[:, 0] == pool[:, 1]) > 0.2  # the case is exercised
        for got, ref in ((got_v, ref_v), (got_c, ref_c)):
            fro, mx = rel_errors(got, ref)
            assert fro <= 1e-5 and mx <= 1e-4, (K, fro, mx)


def test_learning_rate_floor_and_resume_position(gv, tiny_graph):
    g = tiny_graph
    d, K, w = 128, 1, 5.0
    pool, _ = oracle.augment(55, g["offsets"], g["adj"], 40, 5, 30_000, shuffle_seed=1)
    vertex, context = random_embeddings(g["n"], d, seed=2)
    T = 40_000
    # position set to 20000: samples 20000..49999 run past T, where only the floor keeps lr > 0
    thresh, alias = oracle.alias_build(oracle.degree_weights(g["deg"]))
    ref_v, ref_c = vertex.copy(), context.copy()
    oracle.train(ref_v, ref_c, pool, K=K, first_g=20_000, T=T, lr0=LR0, lr_min_ratio=0.1, w=w, seed=8,
                 thresh=thresh, alias=alias)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_DETERMINISTIC, total_samples=T, seed=8,
                     pool_capacity=30_000, lr0=LR0, lr_min_ratio=0.1) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        gv.gv_set_position(ctx, 20_000)
        gv.gv_push_pool(ctx, pool)
        gv.gv_train_pool(ctx)
        got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, g["n"], d)
        got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, g["n"], d)
        assert gv.gv_get_stats(ctx)["samples_trained"] == 50_000
    for got, ref in ((got_v, ref_v), (got_c, ref_c)):
        fro, mx = rel_errors(got, ref)
        assert fro <= 1e-5 and mx <= 1e-4, (fro, mx)


# --------------------------------------------------------------------------- asynchronous mode
# (schedule, coherence) pairs of the asynchronous mode
POOL_ORDER, TILED = 0, 1
PLAIN, AGENT, ATOMIC, MIXED = 0, 1, 2, 3
ALL_POLICIES = [(POOL_ORDER, PLAIN), (POOL_ORDER, AGENT), (POOL_ORDER, ATOMIC), (TILED, AGENT), (TILED, ATOMIC),
                (TILED, MIXED)]
# policies that never drop an update of a contended row: these are held to the quality gate
LOSSLESS_POLICIES = [(POOL_ORDER, ATOMIC), (TILED, ATOMIC), (TILED, MIXED)]


def hogwild_run(gv, n, deg, d, K, w, pools, vertex, context, T, seed, policy):
    cap = max(p.shape[0] for p in pools)
    schedule, coherence = policy
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=cap, lr0=LR0, coherence=coherence, schedule=schedule) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        for p in pools:
            gv.gv_push_pool(ctx, p)
            gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        return gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d), gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)


def singly_touched(pool, negs, n):
    """Samples all of whose rows are named exactly once in the whole pool."""
    cu = np.bincount(pool[:, 0], minlength=n)
    cc = np.bincount(np.concatenate([pool[:, 1], negs.reshape(-1)]), minlength=n)
    ok = (cu[pool[:, 0]] == 1) & (cc[pool[:, 1]] == 1)
    for k in range(negs.shape[1]):
        ok &= cc[negs[:, k]] == 1
    return np.nonzero(ok)[0], cu, cc


def check_single_steps(pool, negs, idx, first_g, T, K, w, seed, vertex, context, got_v, got_c, thresh, alias):
    """Each selected sample saw the initial rows only: its rows equal one oracle step from them."""
    worst = 0.0
    for i in idx:
        u, v = pool[i]
        rows_c = [v] + list(negs[i])
        sub_v = vertex[[u]].copy()
        sub_c = context[rows_c].copy()
        local_pairs = np.array([[0, 0]], dtype=np.uint32)
        local_negs = np.arange(1, K + 1, dtype=np.uint32)
        oracle.train(sub_v, sub_c, local_pairs, K=K, first_g=first_g + int(i), T=T, lr0=LR0, lr_min_ratio=0.0, w=w,
                     seed=seed, thresh=thresh[:K + 1], alias=alias[:K + 1], negatives=local_negs)
        worst = max(worst, np.abs(got_v[u] - sub_v[0]).max() / max(np.abs(sub_v[0]).max(), 1e-30))
        for r, row in enumerate(rows_c):
            worst = max(worst, np.abs(got_c[row] - sub_c[r]).max() / max(np.abs(sub_c[r]).max(), 1e-30))
    return worst


@pytest.mark.parametrize("policy", ALL_POLICIES)
@pytest.mark.parametrize("d,K", [(128, 1), (64, 1), (256, 2), (512, 5), (96, 1), (352, 3)])
def test_hogwild_rows_touched_once_equal_one_oracle_step(gv, policy, d, K):
    """A sparse pool over many nodes: most samples share no row with any other sample, so whatever
    the interleaving their rows must equal one sequential step from the initial values; rows never
    named must be bit-identical to the input.  4099 = 64 chunks and a ragged tail."""
    n, count, w, seed = 200_000, 4099, 5.0 / K, 21
    rng = np.random.default_rng(d + K)
    deg = rng.integers(1, 50, size=n).astype(np.uint32)
    pool = rng.integers(n, size=(count, 2)).astype(np.uint32)
    vertex, context = random_embeddings(n, d, seed=3)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    negs = oracle.draw_negatives(seed, 0, count, K, thresh, alias)
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, [pool], vertex, context, 10 * count, seed, policy)
    idx, cu, cc = singly_touched(pool, negs, n)
    assert idx.size > 0.3 * count
    worst = check_single_steps(pool, negs, idx[:1500], 0, 10 * count, K, w, seed, vertex, context, got_v, got_c,
                               thresh, alias)
    assert worst <= 1e-5, worst
    assert np.array_equal(got_v[cu == 0], vertex[cu == 0])
    assert np.array_equal(got_c[cc == 0], context[cc == 0])
    assert not np.array_equal(got_v[cu > 0], vertex[cu > 0])


@pytest.mark.parametrize("policy", [(TILED, MIXED), (TILED, ATOMIC)])
def test_tiled_pools_of_changing_size(gv, policy):
    """Pools of 300, 9000, 64 and 20001 samples in a row (the per-sample scratch of the tiled schedule grows
    with the largest pool seen and is reused by the smaller ones): samples whose rows nobody else names in
    any of the pools equal one oracle step at their global position."""
    n, d, K, w, seed = 200_000, 128, 2, 2.5, 23
    sizes = [300, 9000, 64, 20_001]
    count = sum(sizes)
    rng = np.random.default_rng(17)
    deg = rng.integers(1, 50, size=n).astype(np.uint32)
    pool = rng.integers(n, size=(count, 2)).astype(np.uint32)
    cuts = np.cumsum([0] + sizes)
    pools = [pool[a:b] for a, b in zip(cuts, cuts[1:])]
    vertex, context = random_embeddings(n, d, seed=5)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    negs = oracle.draw_negatives(seed, 0, count, K, thresh, alias)
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, pools, vertex, context, 10 * count, seed, policy)
    idx, cu, cc = singly_touched(pool, negs, n)
    assert idx.size > 0.15 * count
    picked = np.concatenate([idx[idx < cuts[1]], idx[(idx >= cuts[2]) & (idx < cuts[3])], idx[idx >= cuts[3]][:800],
                             idx[(idx >= cuts[1]) & (idx < cuts[2])][:800]])
    worst = check_single_steps(pool, negs, picked, 0, 10 * count, K, w, seed, vertex, context, got_v, got_c,
                               thresh, alias)
    assert worst <= 1e-5, worst
    assert np.array_equal(got_v[cu == 0], vertex[cu == 0])
    assert np.array_equal(got_c[cc == 0], context[cc == 0])


@pytest.mark.parametrize("policy", [(TILED, AGENT), (TILED, ATOMIC), (TILED, MIXED)])
def test_tiled_run_on_one_hub_row_is_sequential(gv, policy):
    """60 samples that all name one high-degree node u: the tiled schedule keeps vertex[u] in registers
    through the whole run and trades it with memory between batches.  Every context row involved is a
    multiple of its own unit vector, so the score of a sample does not depend on the other samples:
    vertex[u] must then equal the oracle's whatever the order within the run, and every context row
    must have moved by its coefficient times a value vertex[u] passed through."""
    n, d, K, count, w, seed, hub = 200_000, 128, 1, 60, 5.0, 77, 4242
    rng = np.random.default_rng(5)
    deg = rng.integers(1, 50, size=n).astype(np.uint32)
    deg[hub] = 10_000
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    negs = oracle.draw_negatives(seed, 0, count, K, thresh, alias)
    partners = np.setdiff1d(np.arange(1000, 2000, dtype=np.uint32), negs.reshape(-1))[:count]
    rows = np.concatenate([partners, negs.reshape(-1)])
    assert np.unique(rows).size == 2 * count and hub not in rows
    pool = np.stack([np.full(count, hub, dtype=np.uint32), partners], axis=1)
    vertex, context = random_embeddings(n, d, seed=9)
    vertex[hub] = rng.uniform(-1.0, 1.0, size=d).astype(np.float32)
    for j, r in enumerate(rows):
        context[r] = 0.0
        context[r, j] = rng.uniform(0.5, 2.0) * (1 if j % 2 else -1)
    T = 10 * count
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, [pool], vertex, context, T, seed, policy)
    ref_v, ref_c = run_oracle(deg, K, w, [pool], vertex, context, T, seed)
    assert np.abs(got_v[hub] - ref_v[hub]).max() <= 1e-5 * np.abs(ref_v[hub]).max()
    assert not np.allclose(ref_v[hub], vertex[hub], rtol=1e-3)
    lo, hi = np.minimum(vertex[hub], ref_v[hub]), np.maximum(vertex[hub], ref_v[hub])
    for j, r in enumerate(rows):
        moved = got_c[r].astype(np.float64) - context[r]
        coef = (ref_v[hub, j].astype(np.float64) - vertex[hub, j]) / context[r, j]  # x_j moved by coef * c_j
        seen = moved / coef  # the vertex[u] this sample multiplied its coefficient with
        tol = 1e-3 * np.abs(vertex[hub]).max()  # fp32 rounding of the row over the smallest coefficient
        assert np.all(seen >= lo - tol) and np.all(seen <= hi + tol), (j, r)
    untouched = np.ones(n, dtype=bool)
    untouched[rows] = False
    assert np.array_equal(got_c[untouched], context[untouched])


@pytest.mark.parametrize("policy", [(POOL_ORDER, ATOMIC), (TILED, AGENT), (TILED, ATOMIC), (TILED, MIXED)])
def test_single_samples_with_repeated_rows(gv, policy):
    """Three nodes, K = 3: one-sample pools at positions whose negatives repeat v, repeat each other, or equal
    the row the tiled schedule keeps in registers.  One sample alone is one sequential step whatever the
    schedule, so every pattern of repeated rows must reproduce the oracle's step."""
    n, d, K, w, seed, T = 3, 128, 3, 1.0, 3, 1000
    deg = np.array([1, 2, 1], dtype=np.uint32)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    cases = {}
    for g in range(300):
        negs = oracle.draw_negatives(seed, g, 1, K, thresh, alias)[0]
        for u in range(n):
            for v in range(n):
                rows = [v] + [int(x) for x in negs]
                pattern = (u, tuple(rows.index(r) for r in rows))  # which rows coincide, and who is u
                cases.setdefault(pattern, (g, u, v))
    assert len(cases) >= 12
    schedule, coherence = policy
    vertex, context = random_embeddings(n, d, seed=11)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=8, lr0=LR0, coherence=coherence, schedule=schedule) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        for pattern, (g, u, v) in sorted(cases.items()):
            pool = np.array([[u, v]], dtype=np.uint32)
            gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
            gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
            gv.gv_set_position(ctx, g)
            gv.gv_push_pool(ctx, pool)
            gv.gv_train_pool(ctx)
            gv.gv_sync(ctx)
            got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
            got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
            ref_v, ref_c = vertex.copy(), context.copy()
            oracle.train(ref_v, ref_c, pool, K=K, first_g=g, T=T, lr0=LR0, lr_min_ratio=0.0, w=w, seed=seed,
                         thresh=thresh, alias=alias)
            for got, ref, start in ((got_v, ref_v, vertex), (got_c, ref_c, context)):
                step = np.abs(ref - start).max()
                assert np.abs(got - ref).max() <= 1e-4 * step + 1e-7, (pattern, g, u, v)


@pytest.mark.parametrize("policy", [(TILED, AGENT), (TILED, MIXED), (TILED, ATOMIC), (POOL_ORDER, AGENT)])
@pytest.mark.parametrize("shape", ["shared context", "shared vertex", "interleaved runs"])
@pytest.mark.parametrize("d,K", [(128, 1), (128, 3), (512, 5)])  # the wave gathers 4, 2, 1 samples at once
@pytest.mark.parametrize("count", [2, 3, 4])
def test_samples_of_one_wave_sharing_a_cold_row(gv, policy, shape, d, K, count):
    """Four samples that end up next to each other in one wave and share a cold row (one that the store
    policies update with plain device-scope stores).  The wave gathers several samples at once, so a later one
    must not be gathered before the earlier ones' updates of the shared row are out: nothing that the wave
    itself wrote may be lost.  The rows that multiply the shared row have disjoint supports, so its result
    does not depend on the order of the samples: it must equal the sequential oracle's.
      shared context    (u_i, R): context[R] is fetched per sample and written back per sample
      shared vertex     (R, v_i): vertex[R] is the row the wave keeps in registers through the run
      interleaved runs  (a, .), (b, .), (a, .), (b, .) with a and b in one sort group: the register copy of
                        vertex[a] is written back when b takes over, and must be re-read when a returns
    Uniform degrees and ids beyond the ranked range: the rows of u and v are cold; the negatives are what the
    sampler draws, and where one of them has a rank, its row is the one the wave keeps and the shared row is
    fetched and written back per sample (with 2 or 3 samples the one naming the row held by the sample before it
    sits in lane 1 or 2 of the wave, where the comparison with the lanes before it has the fewest partners)."""
    if shape == "interleaved runs" and count != 4:
        pytest.skip("the interleaved shape has four samples")
    n, w, seed, T = 100_000, 5.0 / K, 41, 1000
    deg = np.ones(n, dtype=np.uint32)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    rng = np.random.default_rng(7)
    negs = oracle.draw_negatives(seed, 0, count, K, thresh, alias).reshape(-1)
    assert np.unique(negs).size == negs.size
    free = np.setdiff1d(np.arange(70_000, 90_000, dtype=np.uint32), negs)
    if shape == "shared context":
        shared = [free[0]]
        pool = np.stack([free[1:1 + count], np.full(count, shared[0], dtype=np.uint32)], axis=1)
        blocks_in, check = ("vertex", free[1:1 + count]), "context"
    elif shape == "shared vertex":
        shared = [free[0]]
        pool = np.stack([np.full(count, shared[0], dtype=np.uint32), free[1:1 + count]], axis=1)
        blocks_in, check = ("context", np.concatenate([free[1:1 + count], negs])), "vertex"
    else:
        group = ((free.astype(np.uint64) * np.uint64(0x9E3779B1)) & np.uint64(0xFFFFFFFF)) >> np.uint64(20)
        values, first, counts = np.unique(group, return_index=True, return_counts=True)
        g0 = values[counts >= 2][0]
        a, b = free[group == g0][:2]  # two nodes whose samples the tile sort puts in one group
        shared = [a, b]
        rest = np.setdiff1d(free, shared)[:count]
        pool = np.stack([np.array([a, b, a, b], dtype=np.uint32), rest], axis=1)
        blocks_in, check = ("context", np.concatenate([rest, negs])), "vertex"
    vertex, context = random_embeddings(n, d, seed=13)
    target = vertex if blocks_in[0] == "vertex" else context
    for j, r in enumerate(blocks_in[1]):  # row j of the multiplying rows lives on coordinates 8j .. 8j+7
        target[r] = 0.0
        target[r, 8 * j:8 * j + 8] = rng.uniform(0.5, 1.0, size=8)
    assert np.unique(blocks_in[1]).size == len(blocks_in[1])
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, [pool], vertex, context, T, seed, policy)
    ref_v, ref_c = run_oracle(deg, K, w, [pool], vertex, context, T, seed)
    got, ref, start = (got_v, ref_v, vertex) if check == "vertex" else (got_c, ref_c, context)
    for r in shared:
        step = np.abs(ref[r] - start[r]).max()
        assert step > 1e-3
        assert np.abs(got[r] - ref[r]).max() <= 1e-4 * step + 1e-7, (shape, policy, int(r))


@pytest.mark.parametrize("policy", [(TILED, AGENT), (TILED, MIXED), (TILED, ATOMIC), (POOL_ORDER, AGENT)])
@pytest.mark.parametrize("d,K", [(128, 1), (128, 3), (512, 5), (96, 2)])  # (96, 2): rows that do not fill their lanes
@pytest.mark.parametrize("samples,trial,filler", [(2, 0, 0), (3, 0, 0), (9, 0, 0), (64, 0, 0), (64, 1, 0), (64, 0, 300)])
@pytest.mark.parametrize("kind", ["cold vertex", "warm vertex", "cold context", "warm context"])
def test_random_sharing_of_a_few_rows_is_exact(gv, policy, d, K, trial, samples, filler, kind):
    """A few samples, or as many as a row has room for, that share a few rows at random, built so that the result
    does not depend on their order: the rows that multiply a shared row are multiples of unit vectors of their own,
    so a sample moves the shared row along its own coordinates only.  The shared rows must then come out as the
    sequential oracle leaves them, whichever rows the wave happens to keep, gather together, put off, trade with
    memory or write back in between.
      ... vertex    u drawn from the shared nodes, v different for every sample; v and the negatives are unit rows
      ... context   v drawn from the shared nodes, u different for every sample and a unit row
      cold ...      shared nodes without a rank (ids beyond the ranked range: updated with stores under the store
                    policies)
      warm ...      shared nodes among the hottest ranks (exact grouping, runs in registers, atomic updates)
    The negatives are what the sampler draws: some have a rank and become the row that is kept, some do not.
    `filler` unrelated samples (rows of their own) are mixed into the pool, so that the tile sort spreads the
    related ones over several 64-sample chunks of the wave.
    (POOL_ORDER, AGENT) runs the samples of a wave one after the other and is exact as well."""
    if filler and policy[0] == POOL_ORDER:
        pytest.skip("in pool order the chunks of a larger pool go to different waves, whose stores may race")
    n, w, T = 100_000, 5.0 / K, 1000
    count = min(samples, d // (K + 1))
    filler = min(filler, 300 // K)
    total = count + filler
    deg = np.ones(n, dtype=np.uint32)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    rng = np.random.default_rng(trial + 7 * samples)
    where = np.sort(rng.permutation(total)[:count]) if filler else np.arange(count)  # places of the related samples
    related = np.zeros(total, dtype=bool)
    related[where] = True
    for seed in range(100 + 50 * trial + 1000 * samples, 300 + 50 * trial + 1000 * samples):
        all_negs = oracle.draw_negatives(seed, 0, total, K, thresh, alias)
        negs = all_negs[related].reshape(-1)
        # the first seed with which the related samples draw different nodes and the filler draws none of them
        if np.unique(negs).size == negs.size and not np.isin(all_negs[~related], negs).any():
            break
    assert np.unique(negs).size == negs.size and not np.isin(all_negs[~related], negs).any()
    free = np.setdiff1d(np.arange(70_000, 90_000, dtype=np.uint32), all_negs)
    hot = np.setdiff1d(np.arange(100, 200, dtype=np.uint32), all_negs)
    shared = (free if kind.startswith("cold") else hot)[:5 if count > 9 else 2]
    singles = free[5:5 + count]
    drawn = rng.choice(shared, size=count).astype(np.uint32)
    vertex, context = random_embeddings(n, d, seed=trial)
    pool = np.stack([free[1000:1000 + total], free[2000:2000 + total]], axis=1)  # the filler: rows nobody else names
    if kind.endswith("vertex"):
        pool[where] = np.stack([drawn, singles], axis=1)
        for j, r in enumerate(np.concatenate([singles, negs])):
            context[r] = 0.0
            context[r, j] = rng.uniform(0.5, 2.0) * (1 if j % 2 else -1)
    else:
        pool[where] = np.stack([singles, drawn], axis=1)
        for j, r in enumerate(singles):
            vertex[r] = 0.0
            vertex[r, j] = rng.uniform(0.5, 2.0) * (1 if j % 2 else -1)
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, [pool], vertex, context, T, seed, policy)
    ref_v, ref_c = run_oracle(deg, K, w, [pool], vertex, context, T, seed)
    got, ref, start = (got_v, ref_v, vertex) if kind.endswith("vertex") else (got_c, ref_c, context)
    for r in shared:
        if not (drawn == r).any():
            continue
        step = np.abs(ref[r] - start[r]).max()
        assert step > 1e-4
        assert np.abs(got[r] - ref[r]).max() <= 1e-4 * step + 1e-7, (int(r), policy)


def test_schedule_is_chosen_from_the_graph(gv, tiny_graph):
    """GV_SCHEDULE_AUTO: a graph with rows that concurrent samples share is trained with the tiled schedule, one
    without (4*10^5 nodes of equal degree: each is named by 2 of 8192 samples in flight with probability 0.04) in
    pool order."""
    g = tiny_graph
    rng = np.random.default_rng(1)
    flat_n = 400_000
    cases = ((g["deg"], np.stack([g["src"][:5000], g["dst"][:5000]], axis=1), True),
             (np.full(flat_n, 3, dtype=np.uint32), rng.integers(flat_n, size=(5000, 2)).astype(np.uint32), False))
    for deg, pool, tiled in cases:
        with context_for(gv, dim=32, num_neg=1, total_samples=10_000, pool_capacity=5000) as ctx:
            gv.gv_set_degrees(ctx, deg)
            gv.gv_build_alias(ctx, 0.75)
            gv.gv_init_embeddings(ctx, 1)
            gv.gv_push_pool(ctx, pool)
            gv.gv_train_pool(ctx)
            gv.gv_sync(ctx)
            stats = gv.gv_get_stats(ctx)
            assert (stats["tiled_launches"] == 1) == tiled and (stats["warm_rows"] > 0) == tiled
            assert np.abs(gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, deg.size, 32)).max() > 0


def evaluation_loss(deg, vertex, context, eval_pool, K, w):
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    return oracle.loss(vertex, context, eval_pool, K=K, w=w, seed=99, thresh=thresh, alias=alias)


@pytest.mark.parametrize("policy", LOSSLESS_POLICIES)
def test_hogwild_quality_matches_oracle_on_tiny(gv, policy):
    """Configuration 1 in asynchronous mode: final evaluation loss within 2 % of the sequential
    oracle's and link-prediction AUC within 0.005 (5 % of the edges held out)."""
    n, src, dst = W.make_graph("tiny", cache=False)
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, 0.05, seed=31)
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    total, d, K, w = 2_000_000, 128, 1, 5.0
    pool, _ = oracle.augment(101, offsets, adj, 40, 5, total, shuffle_seed=7)
    eval_pool, _ = oracle.augment(202, offsets, adj, 40, 5, 1 << 18, shuffle_seed=8)
    vertex, context = oracle.init_embeddings(1, n, d)
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, [pool], vertex, context, total, 1234, policy)
    ref_v, ref_c = run_oracle(deg, K, w, [pool], vertex, context, total, 1234)
    loss_gpu = evaluation_loss(deg, got_v, got_c, eval_pool, K, w)
    loss_ref = evaluation_loss(deg, ref_v, ref_c, eval_pool, K, w)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=32)
    auc_gpu = oracle.link_prediction_auc(got_v, te_s, te_d, na, nb)
    auc_ref = oracle.link_prediction_auc(ref_v, te_s, te_d, na, nb)
    print(f"tiny hogwild policy={policy}: loss {loss_gpu:.5f} vs {loss_ref:.5f}; auc {auc_gpu:.4f} vs {auc_ref:.4f}")
    assert np.isfinite(got_v).all() and np.isfinite(got_c).all()
    assert abs(loss_gpu - loss_ref) <= 0.02 * loss_ref
    assert abs(auc_gpu - auc_ref) <= 0.005


@pytest.mark.parametrize("policy", LOSSLESS_POLICIES)
def test_hogwild_quality_with_five_negatives(gv, policy):
    """The shape of configuration 3 (K = 5, weight 1) on the small graph, d = 64: with several negatives the
    tiled schedule may keep any of the K + 2 rows of a sample in registers.  Same gates as above."""
    n, src, dst = W.make_graph("tiny", cache=False)
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, 0.05, seed=31)
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    total, d, K, w = 8_000_000, 64, 5, 1.0
    pool, _ = oracle.augment(103, offsets, adj, 40, 5, total, shuffle_seed=7)
    eval_pool, _ = oracle.augment(203, offsets, adj, 40, 5, 1 << 17, shuffle_seed=8)
    vertex, context = oracle.init_embeddings(1, n, d)
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, [pool], vertex, context, total, 1234, policy)
    ref_v, ref_c = run_oracle(deg, K, w, [pool], vertex, context, total, 1234)
    loss_gpu = evaluation_loss(deg, got_v, got_c, eval_pool, K, w)
    loss_ref = evaluation_loss(deg, ref_v, ref_c, eval_pool, K, w)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=32)
    auc_gpu = oracle.link_prediction_auc(got_v, te_s, te_d, na, nb)
    auc_ref = oracle.link_prediction_auc(ref_v, te_s, te_d, na, nb)
    print(f"tiny K=5 policy={policy}: loss {loss_gpu:.5f} vs {loss_ref:.5f}; auc {auc_gpu:.4f} vs {auc_ref:.4f}")
    assert loss_ref < 0.8 * evaluation_loss(deg, vertex, context, eval_pool, K, w)  # the run did learn
    assert abs(loss_gpu - loss_ref) <= 0.02 * loss_ref
    assert abs(auc_gpu - auc_ref) <= 0.005


@pytest.mark.parametrize("policy", LOSSLESS_POLICIES)
def test_hogwild_quality_on_planted_partition(gv, policy):
    """Scaled-down configuration 4 (5000 nodes, 10 communities, 5*10^4 edges, 5 % held out,
    8*10^6 samples in 2^20-sample pools, trained to the plateau): loss within 2 %, AUC within
    0.005 of the oracle."""
    cfg = W.CONFIGS["c4-small"]
    n = cfg["n"]
    src, dst, _ = W.planted_partition(n, cfg["communities"], cfg["edges"], cfg["ratio"], seed=4)
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, 0.05, seed=41)
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    total, d, K, w = cfg["total_samples"], 128, 1, 5.0
    pool, _ = oracle.augment(104, offsets, adj, 40, 5, total, shuffle_seed=7)
    pools = [pool[i:i + cfg["pool"]] for i in range(0, total, cfg["pool"])]
    eval_pool, _ = oracle.augment(204, offsets, adj, 40, 5, 1 << 18, shuffle_seed=8)
    vertex, context = oracle.init_embeddings(1, n, d)
    got_v, got_c = hogwild_run(gv, n, deg, d, K, w, pools, vertex, context, total, 1234, policy)
    ref_v, ref_c = run_oracle(deg, K, w, pools, vertex, context, total, 1234)
    loss_gpu = evaluation_loss(deg, got_v, got_c, eval_pool, K, w)
    loss_ref = evaluation_loss(deg, ref_v, ref_c, eval_pool, K, w)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=42)
    auc_gpu = oracle.link_prediction_auc(got_v, te_s, te_d, na, nb)
    auc_ref = oracle.link_prediction_auc(ref_v, te_s, te_d, na, nb)
    print(f"sbm hogwild policy={policy}: loss {loss_gpu:.5f} vs {loss_ref:.5f}; auc {auc_gpu:.4f} vs {auc_ref:.4f}")
    assert abs(loss_gpu - loss_ref) <= 0.02 * loss_ref
    assert abs(auc_gpu - auc_ref) <= 0.005
    assert auc_ref > 0.85


# --------------------------------------------------------------------------- full size, bench configuration
@pytest.fixture(scope="module")
def c2_workload():
    """Configuration 2 at full size: Chung-Lu graph, 10^6 nodes / 5*10^6 edges, one 2^24-sample walk pool."""
    n, src, dst = W.make_graph("c2")
    deg = W.degrees(n, src, dst)
    offsets, adj = W.csr_from_edges(n, src, dst)
    pool = W.walk_pool(offsets, adj, 1 << 24, 40, 5, seed=202)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    return dict(n=n, deg=deg, pool=pool, thresh=thresh, alias=alias, src=src, dst=dst, offsets=offsets, adj=adj)


def test_full_size_tables_and_negatives(gv, c2_workload):
    c2 = c2_workload
    with context_for(gv, dim=128, num_neg=1, total_samples=2_000_000_000, pool_capacity=1, seed=1234) as ctx:
        gv.gv_set_degrees(ctx, c2["deg"])
        gv.gv_build_alias(ctx, 0.75)
        thresh, alias = gv.gv_get_alias(ctx, c2["n"])
        assert np.array_equal(thresh, c2["thresh"]) and np.array_equal(alias, c2["alias"])
        for first_g in (0, 1_999_000_000, 2**33 + 5):
            got = gv.gv_draw_negatives(ctx, first_g, 1 << 20, 1)
            assert np.array_equal(got, oracle.draw_negatives(1234, first_g, 1 << 20, 1, c2["thresh"], c2["alias"]))


@pytest.mark.parametrize("policy", [(TILED, MIXED), (TILED, ATOMIC), (POOL_ORDER, ATOMIC)])
def test_full_size_pool_in_bench_configuration(gv, c2_workload, policy):
    """One 2^24-sample pool of configuration 2 through the launch configuration bench.py times
    (device-resident pool, d=128, K=1, w=5, T=2*10^9).  Checked on what the oracle can compute one
    by one: every sample whose three rows are named exactly once in the pool must leave exactly one
    sequential step behind, whatever happened around it; rows nobody names stay bit-identical."""
    import torch

    c2 = c2_workload
    n, d, K, w, T, seed = c2["n"], 128, 1, 5.0, 2_000_000_000, 1234
    first_g = 1_000_000_000  # mid-run: learning rate 0.0125, 64-bit positions
    # A walk pool names every node several times, so no sample is isolated by itself.  Plant some:
    # at positions whose negative is drawn nowhere else and is nobody's v, put a pair of isolated
    # (degree 0) nodes that nothing else names.  Those samples share no row with any other sample.
    pool = c2["pool"].copy()
    negs = oracle.draw_negatives(seed, first_g, pool.shape[0], K, c2["thresh"], c2["alias"])
    context_use = np.bincount(np.concatenate([pool[:, 1], negs.reshape(-1)]), minlength=n)
    where = np.nonzero(context_use[negs[:, 0]] == 1)[0]
    lonely = np.nonzero(c2["deg"] == 0)[0].astype(np.uint32)
    planted = min(where.size, lonely.size // 2, 4096)
    assert planted >= 256, (where.size, lonely.size)
    where = where[np.linspace(0, where.size - 1, planted).astype(np.int64)]
    pool[where, 0] = lonely[:planted]
    pool[where, 1] = lonely[planted:2 * planted]
    vertex, context = random_embeddings(n, d, seed=11, scale=0.2)
    dev_pool = torch.from_numpy(pool.view(np.int32)).cuda()
    torch.cuda.synchronize()
    schedule, coherence = policy
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=1, lr0=LR0, coherence=coherence, schedule=schedule) as ctx:
        gv.gv_set_degrees(ctx, c2["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        gv.gv_set_position(ctx, first_g)
        gv.gv_train_device_pool(ctx, dev_pool.data_ptr(), pool.shape[0])
        gv.gv_sync(ctx)
        got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
        got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
        assert gv.gv_get_stats(ctx)["samples_trained"] == first_g + pool.shape[0]
    idx, cu, cc = singly_touched(pool, negs, n)
    assert idx.size >= 256, idx.size
    rng = np.random.default_rng(0)
    sample = rng.choice(idx, size=min(3000, idx.size), replace=False)
    worst = check_single_steps(pool, negs, sample, first_g, T, K, w, seed, vertex, context, got_v, got_c,
                               c2["thresh"], c2["alias"])
    print(f"full size {policy}: {idx.size} isolated samples, {sample.size} checked, worst rel. error {worst:.2e}")
    assert worst <= 1e-5, worst
    assert np.array_equal(got_v[cu == 0], vertex[cu == 0])
    assert np.array_equal(got_c[cc == 0], context[cc == 0])
    assert np.isfinite(got_v).all() and np.isfinite(got_c).all()
    # the hottest rows did move, and by a bounded amount (no runaway accumulation)
    hot = np.argsort(c2["deg"])[-16:]
    moved = np.abs(got_v[hot] - vertex[hot]).max(axis=1)
    assert (moved > 0).all() and moved.max() < 4.0  # the sequential oracle moves these rows by about 1.4


# --------------------------------------------------------------------------- streaming and errors
def test_streamed_pools_equal_resident_pools(gv, tiny_graph):
    """Pinned-slot producer path (acquire, fill, push, train, double-buffered) gives the same bits
    as pushing plain host arrays and as training device-resident pools (deterministic mode)."""
    import torch

    g = tiny_graph
    d, K, w, seed = 128, 1, 5.0, 5
    counts = [40_000, 65_536, 1, 30_011, 64]
    total = sum(counts)
    pool, _ = oracle.augment(77, g["offsets"], g["adj"], 40, 5, total, shuffle_seed=3)
    cuts = np.cumsum([0] + counts)
    pools = [pool[a:b] for a, b in zip(cuts, cuts[1:])]
    vertex, context = random_embeddings(g["n"], d, seed=9)
    results = []
    for how in ("host", "slot", "device"):
        with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_DETERMINISTIC, total_samples=total,
                         seed=seed, pool_capacity=65_536, lr0=LR0) as ctx:
            gv.gv_set_degrees(ctx, g["deg"])
            gv.gv_build_alias(ctx, 0.75)
            gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
            gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
            if how == "host":
                for p in pools:
                    gv.gv_push_pool(ctx, p)
                    gv.gv_train_pool(ctx)
            elif how == "slot":
                # keep two pools in flight: fill and push pool k+1 before training pool k
                slot = gv.gv_acquire_pool_slot(ctx, 65_536)
                slot[:pools[0].shape[0]] = pools[0]
                gv.gv_push_pool(ctx, slot, pools[0].shape[0])
                for k in range(len(pools)):
                    if k + 1 < len(pools):
                        slot = gv.gv_acquire_pool_slot(ctx, 65_536)
                        slot[:pools[k + 1].shape[0]] = pools[k + 1]
                        gv.gv_push_pool(ctx, slot, pools[k + 1].shape[0])
                    gv.gv_train_pool(ctx)
            else:
                keep = [torch.from_numpy(p.copy().view(np.int32)).cuda() for p in pools]
                torch.cuda.synchronize()
                for t, p in zip(keep, pools):
                    gv.gv_train_device_pool(ctx, t.data_ptr(), p.shape[0])
            gv.gv_sync(ctx)
            stats = gv.gv_get_stats(ctx)
            assert stats["samples_trained"] == total and stats["pools_trained"] == len(pools)
            results.append((gv.gv_read_embeddings(ctx, gv.GV_VERTEX, g["n"], d),
                            gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, g["n"], d)))
    for v, c in results[1:]:
        assert np.array_equal(v, results[0][0]) and np.array_equal(c, results[0][1])
    ref_v, ref_c = run_oracle(g["deg"], K, w, pools, vertex, context, total, seed)
    assert rel_errors(results[0][0], ref_v)[0] <= 1e-5 and rel_errors(results[0][1], ref_c)[0] <= 1e-5


def test_ring_of_pinned_slots_is_cycled_without_refilling(gv, tiny_graph):
    """pool_slots = 4: four pools are written into the slots once; acquiring and pushing the slots again,
    without touching their contents, trains the same pools again.  Equal to pushing the same sequence from
    plain host arrays (deterministic mode: bit for bit)."""
    g = tiny_graph
    d, K, w, seed, R, P = 64, 1, 5.0, 5, 4, 20_000
    pools = [oracle.augment(300 + r, g["offsets"], g["adj"], 40, 5, P - 100 * r, shuffle_seed=r)[0] for r in range(R)]
    order = list(range(R)) * 3
    vertex, context = random_embeddings(g["n"], d, seed=9)
    results = []
    for how in ("host", "ring"):
        with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_DETERMINISTIC,
                         total_samples=len(order) * P, seed=seed, pool_capacity=P, lr0=LR0, pool_slots=R) as ctx:
            gv.gv_set_degrees(ctx, g["deg"])
            gv.gv_build_alias(ctx, 0.75)
            gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
            gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
            if how == "host":
                for r in order:
                    gv.gv_push_pool(ctx, pools[r])
                    gv.gv_train_pool(ctx)
            else:
                addresses = []
                for turn, r in enumerate(order):
                    slot = gv.gv_acquire_pool_slot(ctx, P)
                    if turn < R:  # first time round: fill
                        slot[:pools[r].shape[0]] = pools[r]
                        addresses.append(slot.ctypes.data)
                    else:         # afterwards the ring hands the same slots out again, contents kept
                        assert slot.ctypes.data == addresses[r]
                        assert np.array_equal(slot[:pools[r].shape[0]], pools[r])
                    gv.gv_push_pool(ctx, slot, pools[r].shape[0])
                    if turn >= 2:
                        gv.gv_train_pool(ctx)  # keep three pools in flight
                for _ in range(2):
                    gv.gv_train_pool(ctx)
            gv.gv_sync(ctx)
            assert gv.gv_get_stats(ctx)["pools_trained"] == len(order)
            results.append((gv.gv_read_embeddings(ctx, gv.GV_VERTEX, g["n"], d),
                            gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, g["n"], d)))
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    assert not np.array_equal(results[0][0], vertex)


def test_ring_limits_and_failed_pushes(gv, tiny_graph):
    g = tiny_graph
    ok = np.stack([g["src"][:500], g["dst"][:500]], axis=1)
    with context_for(gv, dim=64, num_neg=1, total_samples=100_000, pool_capacity=1000, pool_slots=3) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 3)
        for _ in range(3):
            gv.gv_push_pool(ctx, ok)
        with pytest.raises(gv.GvError) as e:
            gv.gv_push_pool(ctx, ok)
        assert e.value.code == gv.GV_ESTATE  # three pools queued in a ring of three
        with pytest.raises(gv.GvError) as e:
            gv.gv_acquire_pool_slot(ctx, 1000)
        assert e.value.code == gv.GV_ESTATE
        for _ in range(3):
            gv.gv_train_pool(ctx)
        # a push that fails hands its acquired slot back: the ring stays complete
        for _ in range(5):
            slot = gv.gv_acquire_pool_slot(ctx, 1000)
            with pytest.raises(gv.GvError) as e:
                gv.gv_push_pool(ctx, slot, 1001)
            assert e.value.code == gv.GV_EINVAL
        slots = [gv.gv_acquire_pool_slot(ctx, 1000) for _ in range(3)]
        assert len({s.ctypes.data for s in slots}) == 3
        for s_ in slots:
            s_[:500] = ok
            gv.gv_push_pool(ctx, s_, 500)
        for _ in range(3):
            gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        assert gv.gv_get_stats(ctx)["samples_trained"] == 3000


def test_link_prediction_auc_matches_oracle(gv, tiny_graph):
    """gv_link_prediction_auc against the oracle's cosine + rank statistic, with many exact ties (zero rows
    score 0 on both sides)."""
    g = tiny_graph
    n, d = g["n"], 96
    rng = np.random.default_rng(12)
    vertex = (rng.standard_normal((n, d)) * 0.3).astype(np.float32)
    vertex[rng.integers(n, size=n // 5)] = 0.0
    a, b = g["src"][:20_000], g["dst"][:20_000]
    na, nb = W.uniform_negative_pairs(n, 15_000, seed=5)
    with context_for(gv, dim=d, num_neg=1, total_samples=1, pool_capacity=1) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        got = gv.gv_link_prediction_auc(ctx, a, b, na, nb)
        with pytest.raises(gv.GvError) as e:
            gv.gv_link_prediction_auc(ctx, a, b, np.array([n], dtype=np.uint32), np.array([0], dtype=np.uint32))
        assert e.value.code == gv.GV_EINVAL
    pos, neg = oracle.cosine(vertex, a, b), oracle.cosine(vertex, na, nb)
    assert np.mean(pos == 0.0) > 0.2  # ties are exercised
    # fp32 cosines of the device decide the ranks: compare with the oracle's statistic of the same quantities
    # rounded to fp32 (ties at 0 are exact on both sides), and with its fp64 statistic within rounding noise
    assert abs(got - oracle.auc(pos, neg)) <= 1e-5


def test_errors_are_reported_not_fatal(gv, tiny_graph):
    g = tiny_graph
    n = g["n"]
    with context_for(gv, dim=128, num_neg=1, total_samples=100_000, pool_capacity=1000) as ctx:
        for call in (lambda: gv.gv_build_alias(ctx, 0.75), lambda: gv.gv_init_embeddings(ctx, 1),
                     lambda: gv.gv_push_pool(ctx, np.zeros((4, 2), dtype=np.uint32)), lambda: gv.gv_train_pool(ctx),
                     lambda: gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, 128)):
            with pytest.raises(gv.GvError) as e:
                call()
            assert e.value.code == gv.GV_ESTATE  # no graph yet
        with pytest.raises(gv.GvError) as e:
            gv.gv_set_graph(ctx, n, np.array([0, n], dtype=np.uint32), np.array([1, 2], dtype=np.uint32))
        assert e.value.code == gv.GV_EINVAL and "node id" in str(e.value)
        gv.gv_set_graph(ctx, n, g["src"], g["dst"])
        with pytest.raises(gv.GvError) as e:
            gv.gv_push_pool(ctx, np.zeros((4, 2), dtype=np.uint32))
        assert e.value.code == gv.GV_ESTATE  # no alias table yet
        with pytest.raises(gv.GvError) as e:
            gv.gv_build_alias(ctx, 0.5)
        assert e.value.code == gv.GV_EINVAL
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 3)
        with pytest.raises(gv.GvError) as e:
            gv.gv_train_pool(ctx)
        assert e.value.code == gv.GV_ESTATE  # nothing queued
        with pytest.raises(gv.GvError) as e:
            gv.gv_push_pool(ctx, np.zeros((1001, 2), dtype=np.uint32))
        assert e.value.code == gv.GV_EINVAL  # above pool_capacity
        with pytest.raises(gv.GvError) as e:
            gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 2, 128, row0=n - 1)
        assert e.value.code == gv.GV_EINVAL
        with pytest.raises(gv.GvError) as e:
            gv.gv_read_embeddings(ctx, 2, 1, 128)
        assert e.value.code == gv.GV_EINVAL
        ok = np.stack([g["src"][:500], g["dst"][:500]], axis=1)
        gv.gv_push_pool(ctx, ok)
        gv.gv_push_pool(ctx, ok)
        with pytest.raises(gv.GvError) as e:
            gv.gv_push_pool(ctx, ok)
        assert e.value.code == gv.GV_ESTATE  # two pools already queued
        gv.gv_train_pool(ctx)
        gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        before = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, 128)
        # a pool naming a node that does not exist: the sample is skipped, the next sync reports it once
        bad = ok.copy()
        bad[7, 1] = n
        bad[300, 0] = 0xFFFFFFFF
        gv.gv_push_pool(ctx, bad)
        gv.gv_train_pool(ctx)
        with pytest.raises(gv.GvError) as e:
            gv.gv_sync(ctx)
        assert e.value.code == gv.GV_EINVAL and "node id" in str(e.value)
        gv.gv_sync(ctx)  # reported once; the context stays usable
        after = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, 128)
        assert np.isfinite(after).all() and not np.array_equal(before, after)
        gv.gv_push_pool(ctx, np.zeros((0, 2), dtype=np.uint32))  # empty pool is legal
        gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        assert gv.gv_get_stats(ctx)["samples_trained"] == 1500


@pytest.fixture(scope="module")
def c2_oracle_pool(c2_workload):
    """The sequential oracle over one full 2^24-sample pool of configuration 2 (about 15 s)."""
    c2 = c2_workload
    n, d = c2["n"], 128
    vertex, context = random_embeddings(n, d, seed=11, scale=0.2)
    ref_v, ref_c = vertex.copy(), context.copy()
    oracle.train(ref_v, ref_c, c2["pool"], K=1, first_g=1_000_000_000, T=2_000_000_000, lr0=LR0, lr_min_ratio=0.0,
                 w=5.0, seed=1234, thresh=c2["thresh"], alias=c2["alias"])
    n_, src, dst = W.make_graph("c2")
    offsets, adj = W.csr_from_edges(n, src, dst)
    eval_pool = W.walk_pool(offsets, adj, 1 << 18, 40, 5, seed=303)
    return dict(vertex=vertex, context=context, ref_v=ref_v, ref_c=ref_c, eval_pool=eval_pool)


@pytest.mark.parametrize("policy", [(TILED, MIXED), (TILED, ATOMIC)])
def test_full_size_pool_tracks_the_sequential_oracle(gv, c2_workload, c2_oracle_pool, policy):
    """Same launch configuration as the benchmark (2^24 samples, 10^6 nodes, thousands of samples in
    flight): after the pool the evaluation loss is within 2 % of the sequential oracle's, and the
    hottest rows, which take part in tens of thousands of samples, moved as far as the oracle's."""
    import torch

    c2, o = c2_workload, c2_oracle_pool
    n, d, K, w, T, seed = c2["n"], 128, 1, 5.0, 2_000_000_000, 1234
    dev_pool = torch.from_numpy(c2["pool"].view(np.int32)).cuda()
    torch.cuda.synchronize()
    schedule, coherence = policy
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=1, lr0=LR0, coherence=coherence, schedule=schedule) as ctx:
        gv.gv_set_degrees(ctx, c2["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, o["vertex"])
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, o["context"])
        gv.gv_set_position(ctx, 1_000_000_000)
        gv.gv_train_device_pool(ctx, dev_pool.data_ptr(), c2["pool"].shape[0])
        got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
        got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
    kw = dict(K=K, w=w, seed=99, thresh=c2["thresh"], alias=c2["alias"])
    loss_start = oracle.loss(o["vertex"], o["context"], o["eval_pool"], **kw)
    loss_ref = oracle.loss(o["ref_v"], o["ref_c"], o["eval_pool"], **kw)
    loss_gpu = oracle.loss(got_v, got_c, o["eval_pool"], **kw)
    hot = np.argsort(c2["deg"])[-64:]
    ratios = []
    for got, ref, init in ((got_v, o["ref_v"], o["vertex"]), (got_c, o["ref_c"], o["context"])):
        moved_gpu = np.linalg.norm((got[hot] - init[hot]).astype(np.float64), axis=1)
        moved_ref = np.linalg.norm((ref[hot] - init[hot]).astype(np.float64), axis=1)
        ratios.append(moved_gpu / moved_ref)
    print(f"full size {policy}: loss {loss_start:.4f} -> gpu {loss_gpu:.4f} / oracle {loss_ref:.4f}; "
          f"hot-row movement ratio vertex {np.median(ratios[0]):.2f} context {np.median(ratios[1]):.2f}")
    assert loss_ref < 0.95 * loss_start  # the pool does train
    assert abs(loss_gpu - loss_ref) <= 0.02 * loss_ref
    assert 0.8 < np.median(ratios[0]) < 1.25 and 0.8 < np.median(ratios[1]) < 1.25


def test_rows_beyond_2_to_32_elements(gv):
    """A table of 4*10^7 rows x 128 (5.1*10^9 elements per matrix, 41 GB for both): samples that name
    rows at the far end must be read and written at the right 64-bit offsets.  With the initial
    embeddings (vertex from the counter-based generator, context zero) every isolated sample has the
    closed form of the oracle's single step."""
    n, d, K, w, seed, count, T = 40_000_000, 128, 1, 5.0, 77, 4099, 10**9
    deg = np.ones(n, dtype=np.uint32)
    rng = np.random.default_rng(5)
    far = n - 1 - rng.choice(5_000_000, size=2 * count, replace=False).astype(np.int64)  # last 5 M rows
    pool = np.stack([far[:count], far[count:]], axis=1).astype(np.uint32)
    pool[0] = (n - 1, n - 2)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=count, lr0=LR0) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 9)
        negs = gv.gv_draw_negatives(ctx, 0, count, K)
        gv.gv_push_pool(ctx, pool)
        gv.gv_train_pool(ctx)
        gv.gv_sync(ctx)
        # uniform table: the oracle's draw is the bucket itself
        thresh = np.full(1, 0xFFFFFFFF, dtype=np.uint32)
        touched_c = np.concatenate([pool[:, 1], negs[:, 0]])
        uniq, counts = np.unique(touched_c, return_counts=True)
        once = set(uniq[counts == 1].tolist())
        check = [i for i in range(count) if int(pool[i, 1]) in once and int(negs[i, 0]) in once][:400]
        assert len(check) >= 300
        worst = 0.0
        for i in check:
            u, v, z = int(pool[i, 0]), int(pool[i, 1]), int(negs[i, 0])
            x0 = oracle.init_vertex_rows(9, u, 1, d)
            sub_v, sub_c = x0.copy(), np.zeros((2, d), dtype=np.float32)
            oracle.train(sub_v, sub_c, np.array([[0, 0]], dtype=np.uint32), K=1, first_g=i, T=T, lr0=LR0,
                         lr_min_ratio=0.0, w=w, seed=seed, thresh=thresh, alias=thresh,
                         negatives=np.array([1], dtype=np.uint32))
            got_x = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, d, row0=u)[0]
            got_v = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=v)[0]
            got_z = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=z)[0]
            scale = np.abs(x0).max()
            worst = max(worst, np.abs(got_x - sub_v[0]).max() / scale, np.abs(got_v - sub_c[0]).max() / scale,
                        np.abs(got_z - sub_c[1]).max() / scale)
            assert np.abs(got_v).max() > 0 and np.abs(got_z).max() > 0
        assert worst <= 1e-5, worst
        # rows nobody names keep their initial value, at both ends of the table
        first = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 2, d, row0=0)
        assert np.array_equal(first, oracle.init_vertex_rows(9, 0, 2, d))
        last = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, d, row0=n - 3)
        if (n - 3) not in set(pool[:, 0].tolist()):
            assert np.array_equal(last, oracle.init_vertex_rows(9, n - 3, 1, d))


def test_configuration_5_size_isolated_samples(gv):
    """The node set of configuration 5 (6.6*10^7 nodes, degrees of the Chung-Lu model with exponent 2.2 for 1.8*10^9
    edges; 67.6 GB of embeddings) with a pool whose endpoints come from the degree marginal (the graph's adjacency
    is not generated): the alias table of that size equals the oracle's bit for bit, so do the negatives, and every
    sample of a 2^22-sample pool whose three rows nobody else names is exactly one oracle step from the initial
    embeddings, in the launch configuration bench.py times for this workload (device pool, default policy)."""
    import torch

    n, deg = W.expected_degrees("c5-marginal")
    d, K, w, seed, T, count = 128, 1, 5.0, 1234, 10_000_000_000, 1 << 22
    first_g = 6_000_000_000
    pool = W.marginal_pool(deg, count, seed=505)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    negs = oracle.draw_negatives(seed, first_g, count, K, thresh, alias)
    print(f"configuration 5 size: tables ready ({n} nodes)", flush=True)
    dev_pool = torch.from_numpy(pool.view(np.int32)).cuda()
    torch.cuda.synchronize()
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=8, lr0=LR0) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        got_t, got_a = gv.gv_get_alias(ctx, n)
        assert np.array_equal(got_t, thresh) and np.array_equal(got_a, alias)
        del got_t, got_a
        assert np.array_equal(gv.gv_draw_negatives(ctx, first_g, 1 << 20, K), negs[:1 << 20])
        gv.gv_init_embeddings(ctx, 9)
        gv.gv_set_position(ctx, first_g)
        gv.gv_train_device_pool(ctx, dev_pool.data_ptr(), count)
        gv.gv_sync(ctx)
        stats = gv.gv_get_stats(ctx)
        assert stats["samples_trained"] == first_g + count and stats["tiled_launches"] == 1
        idx, cu, cc = singly_touched(pool, negs, n)
        assert idx.size > 1000
        rng = np.random.default_rng(0)
        far = idx[np.argsort(pool[idx, 0])[-100:]]  # the samples with the highest vertex rows
        check = np.concatenate([rng.choice(idx, size=300, replace=False), far])
        worst = 0.0
        for i in check:
            u, v, z = int(pool[i, 0]), int(pool[i, 1]), int(negs[i, 0])
            x0 = oracle.init_vertex_rows(9, u, 1, d)
            sub_v, sub_c = x0.copy(), np.zeros((2, d), dtype=np.float32)
            oracle.train(sub_v, sub_c, np.array([[0, 0]], dtype=np.uint32), K=1, first_g=first_g + int(i), T=T, lr0=LR0,
                         lr_min_ratio=0.0, w=w, seed=seed, thresh=thresh[:2], alias=alias[:2],
                         negatives=np.array([1], dtype=np.uint32))
            got_x = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, d, row0=u)[0]
            got_v = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=v)[0]
            got_z = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=z)[0]
            scale = np.abs(x0).max()
            worst = max(worst, np.abs(got_x - sub_v[0]).max() / scale, np.abs(got_v - sub_c[0]).max() / scale,
                        np.abs(got_z - sub_c[1]).max() / scale)
            assert np.abs(got_v).max() > 0 and np.abs(got_z).max() > 0
        print(f"configuration 5 size: {idx.size} isolated samples, {check.size} checked, worst rel. error {worst:.2e}")
        assert worst <= 1e-5, worst
        # rows nobody names keep their initial value, at both ends of the matrices
        for row in (int(np.nonzero(cu == 0)[0][0]), int(np.nonzero(cu == 0)[0][-1])):
            assert np.array_equal(gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, d, row0=row)[0],
                                  oracle.init_vertex_rows(9, row, 1, d)[0])
        for row in (int(np.nonzero(cc == 0)[0][0]), int(np.nonzero(cc == 0)[0][-1])):
            assert not gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=row).any()


def test_configuration_5_as_stated_walks_and_training(gv):
    """Configuration 5 with its graph: 6.6*10^7 nodes and 1.8*10^9 edges of the Chung-Lu kind (exponent 2.2), built on
    the GPU by the input recipe and handed to the library from host memory (14.4 GB of adjacency).  The alias table
    of the real degrees, the pools of the device producer and of the host producer (walks far beyond 2^32 included)
    and the negatives are the oracle's bit for bit; every sample of a produced 2^22-sample pool whose three rows
    nobody else names is exactly one oracle step from the initial embeddings (67.6 GB of rows)."""
    import torch

    from workloads import device_graphs

    cfg = W.CONFIGS["c5"]
    n, d, K, w, seed, T, count = cfg["n"], 128, 1, 5.0, 1234, 10_000_000_000, 1 << 22
    L, s = W.configs.WALK_LENGTH, W.configs.WINDOW
    first_g = 7_000_000_000
    off_t, adj_t = device_graphs.chung_lu_csr(n, cfg["edges"], cfg["gamma"], cfg["number"],
                                              progress=lambda text: print(text, flush=True))
    # the recipe's own promises, checked where the arrays are: rows sorted, no loops, every edge in both rows
    degree_t = off_t[1:] - off_t[:-1]
    assert int(off_t[-1]) == adj_t.numel() and abs(adj_t.numel() // 2 - cfg["edges"]) < 1_000_000
    for row in (int(torch.argmax(degree_t)), 12_345_678, n - 1):
        lo, hi = int(off_t[row]), int(off_t[row + 1])
        mine = adj_t[lo:hi].to(torch.int64)
        assert bool((mine[1:] > mine[:-1]).all()) and not bool((mine == row).any())
        for other in mine[:: max(1, mine.numel() // 50)].tolist():
            theirs = adj_t[int(off_t[other]):int(off_t[other + 1])]
            assert bool((theirs == row).any())
    del degree_t
    offsets, adj = device_graphs.to_host_csr(off_t, adj_t)
    del off_t, adj_t
    torch.cuda.empty_cache()
    deg = np.diff(offsets).astype(np.uint32)
    print(f"configuration 5: graph ready, {adj.size // 2} edges, largest degree {deg.max()}, "
          f"{int((deg == 0).sum())} nodes without edge", flush=True)
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=T, seed=seed,
                     pool_capacity=8, lr0=LR0) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        got_t, got_a = gv.gv_get_alias(ctx, n)
        assert np.array_equal(got_t, thresh) and np.array_equal(got_a, alias)
        del got_t, got_a
        gv.gv_set_adjacency(ctx, offsets, adj)
        print("configuration 5: tables and adjacency on the device", flush=True)
        buf = torch.empty((count, 2), dtype=torch.int32, device="cuda")
        pool = None
        for first_walk, size in ((0, count), ((1 << 33) + 5, 190 * 2000 + 17)):
            gv.gv_augment_device(ctx, buf.data_ptr(), seed=505, first_walk=first_walk, count=size)
            gv.gv_sync(ctx)
            on_device = buf[:size].cpu().numpy().view(np.uint32)
            expect, _ = oracle.augment(505, offsets, adj, L, s, size, first_walk=first_walk)
            expect = oracle.pseudo_shuffle(expect, s)
            assert np.array_equal(on_device, expect), first_walk
            on_host, _ = gv.gv_augment(offsets, adj, seed=505, first_walk=first_walk, count=size, threads=16)
            assert np.array_equal(on_host, expect), first_walk
            if pool is None:
                pool = expect
        print("configuration 5: produced pools equal the oracle's", flush=True)
        negs = oracle.draw_negatives(seed, first_g, count, K, thresh, alias)
        assert np.array_equal(gv.gv_draw_negatives(ctx, first_g, 1 << 20, K), negs[:1 << 20])
        # no sample of a walk pool is alone on its rows (a walk names each of its nodes several times): plant
        # pairs of nodes that nothing else names at positions whose negative nothing else names
        pool = pool.copy()
        named = np.bincount(np.concatenate([pool.reshape(-1), negs.reshape(-1)]), minlength=n)
        where = np.nonzero(named[negs[:, 0]] == 1)[0]
        lonely = np.nonzero(named == 0)[0].astype(np.uint32)
        planted = 1024
        assert where.size >= planted and lonely.size >= 2 * planted
        where = where[np.linspace(0, where.size - 1, planted).astype(np.int64)]
        lonely = lonely[np.linspace(0, lonely.size - 1, 2 * planted).astype(np.int64)]  # from both ends of the matrices
        pool[where, 0], pool[where, 1] = lonely[:planted], lonely[planted:]
        del named
        buf.copy_(torch.from_numpy(pool.view(np.int32)))
        torch.cuda.synchronize()
        gv.gv_init_embeddings(ctx, 9)
        gv.gv_set_position(ctx, first_g)
        gv.gv_train_device_pool(ctx, buf.data_ptr(), count)
        gv.gv_sync(ctx)
        stats = gv.gv_get_stats(ctx)
        assert stats["samples_trained"] == first_g + count and stats["tiled_launches"] == 1
        idx, cu, cc = singly_touched(pool, negs, n)
        assert idx.size >= planted // 2, idx.size
        rng = np.random.default_rng(0)
        check = rng.choice(idx, size=300, replace=False)
        worst = 0.0
        for i in check:
            u, v, z = int(pool[i, 0]), int(pool[i, 1]), int(negs[i, 0])
            x0 = oracle.init_vertex_rows(9, u, 1, d)
            sub_v, sub_c = x0.copy(), np.zeros((2, d), dtype=np.float32)
            oracle.train(sub_v, sub_c, np.array([[0, 0]], dtype=np.uint32), K=1, first_g=first_g + int(i), T=T, lr0=LR0,
                         lr_min_ratio=0.0, w=w, seed=seed, thresh=thresh[:2], alias=alias[:2],
                         negatives=np.array([1], dtype=np.uint32))
            got_x = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, d, row0=u)[0]
            got_v = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=v)[0]
            got_z = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, 1, d, row0=z)[0]
            scale = np.abs(x0).max()
            worst = max(worst, np.abs(got_x - sub_v[0]).max() / scale, np.abs(got_v - sub_c[0]).max() / scale,
                        np.abs(got_z - sub_c[1]).max() / scale)
            assert np.abs(got_v).max() > 0 and np.abs(got_z).max() > 0
        print(f"configuration 5: {idx.size} isolated samples, {check.size} checked, worst rel. error {worst:.2e}")
        assert worst <= 1e-5, worst


# --------------------------------------------------------------------------- evaluation on the device
@pytest.mark.parametrize("d,K,w", [(128, 1, 5.0), (96, 1, 5.0), (512, 5, 1.0), (64, 3, 2.0)])
def test_device_loss_and_cosine_match_oracle(gv, tiny_graph, tiny_alias, d, K, w):
    g = tiny_graph
    n = g["n"]
    rng = np.random.default_rng(d + K)
    vertex = (rng.standard_normal((n, d)) * 0.4).astype(np.float32)
    context = (rng.standard_normal((n, d)) * 0.4).astype(np.float32)  # scores up to |20|: both log branches
    vertex[17] = 0.0
    eval_pool, _ = oracle.augment(9, g["offsets"], g["adj"], 40, 5, 70_003, shuffle_seed=2)
    a = rng.integers(n, size=5000).astype(np.uint32)
    b = rng.integers(n, size=5000).astype(np.uint32)
    a[:3], b[:3] = (17, 5, 17), (4, 17, 17)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, total_samples=1, pool_capacity=1) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        loss = gv.gv_eval_loss(ctx, eval_pool, 4242)
        cos = gv.gv_cosine(ctx, a, b)
        bad = eval_pool.copy()
        bad[5, 0] = n
        with pytest.raises(gv.GvError) as e:
            gv.gv_eval_loss(ctx, bad, 1)
        assert e.value.code == gv.GV_EINVAL
    ref = oracle.loss(vertex, context, eval_pool, K=K, w=w, seed=4242, thresh=tiny_alias[0], alias=tiny_alias[1])
    assert abs(loss - ref) <= 1e-5 * abs(ref), (loss, ref)
    ref_cos = oracle.cosine(vertex, a, b)
    assert np.abs(cos - ref_cos).max() <= 1e-5
    assert cos[0] == 0 and cos[1] == 0 and cos[2] == 0


# --------------------------------------------------------------------------- producer on the device
@pytest.mark.parametrize("L,s,count,first_walk,shuffle", [
    (40, 5, 190 * 300, 0, 0), (40, 5, 190 * 300, 0, 1), (40, 5, 57_123, 1000, 1), (40, 5, 7, 5, 1), (40, 5, 1, 0, 1),
    (40, 2, 40_000, 17, 1), (7, 7, 10_000, 3, 1), (3, 5, 9_999, 0, 1), (64, 5, 30_000, 2**33, 1), (1, 1, 500, 0, 0),
    (40, 1000, 50, 0, 1), (40, 300, 100_000, 9, 1), (64, 64, 200_000, 0, 1), (64, 64, 200_000, 0, 0), (5, 3, 128 * 12 + 5, 0, 1),
])
def test_device_producer_writes_the_oracle_pool(gv, tiny_graph, L, s, count, first_walk, shuffle):
    """gv_augment_device fills device memory with exactly the pool of the oracle's augmentation
    (and pseudo shuffle): same walks, same pairs, same order, also for ragged counts, walks far
    into the stream, and windows wider than the walk."""
    import torch

    g = tiny_graph
    with context_for(gv, dim=32, num_neg=1, neg_weight=5.0, mode=gv.GV_MODE_HOGWILD, total_samples=10, seed=1,
                     pool_capacity=8, lr0=LR0) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_set_adjacency(ctx, g["offsets"], g["adj"])
        out = torch.full((count + 3, 2), -1, dtype=torch.int32, device="cuda")
        walks = gv.gv_augment_device(ctx, out.data_ptr(), seed=91, walk_length=L, window=s, first_walk=first_walk,
                                     count=count, shuffle=shuffle)
        gv.gv_sync(ctx)
        got = out.cpu().numpy().view(np.uint32)
    ref, ref_walks = oracle.augment(91, g["offsets"], g["adj"], L, s, count, first_walk=first_walk)
    if shuffle:
        ref = oracle.pseudo_shuffle(ref, s)
    assert walks == ref_walks
    assert np.array_equal(got[:count], ref)
    assert (got[count:] == 0xFFFFFFFF).all()  # nothing written past the pool


def test_device_producer_feeds_training_like_the_host_producer(gv, tiny_graph):
    """A pool produced on the device and trained from there gives the same embeddings as the same pool
    produced by the host producer and pushed (deterministic mode: bit-identical)."""
    import torch

    g = tiny_graph
    d, K, count = 64, 2, 50_000
    vertex, context = random_embeddings(g["n"], d, seed=4)
    results = []
    for how in ("host", "device"):
        with context_for(gv, dim=d, num_neg=K, neg_weight=2.5, mode=gv.GV_MODE_DETERMINISTIC, total_samples=2 * count,
                         seed=6, pool_capacity=count, lr0=LR0) as ctx:
            gv.gv_set_degrees(ctx, g["deg"])
            gv.gv_build_alias(ctx, 0.75)
            gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
            gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
            if how == "host":
                for k in range(2):
                    pool, walks = gv.gv_augment(g["offsets"], g["adj"], seed=8, first_walk=k * 264, count=count, threads=4)
                    gv.gv_push_pool(ctx, pool)
                    gv.gv_train_pool(ctx)
            else:
                gv.gv_set_adjacency(ctx, g["offsets"], g["adj"])
                buf = torch.empty((count, 2), dtype=torch.int32, device="cuda")
                for k in range(2):  # the buffer is refilled right behind the launch that trains it
                    gv.gv_augment_device(ctx, buf.data_ptr(), seed=8, first_walk=k * 264, count=count)
                    gv.gv_train_device_pool(ctx, buf.data_ptr(), count)
            gv.gv_sync(ctx)
            results.append((gv.gv_read_embeddings(ctx, gv.GV_VERTEX, g["n"], d),
                            gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, g["n"], d)))
    assert np.array_equal(results[0][0], results[1][0]) and np.array_equal(results[0][1], results[1][1])
    assert not np.array_equal(results[0][0], vertex)


def test_device_producer_argument_errors(gv, tiny_graph):
    import torch

    g = tiny_graph
    with context_for(gv, dim=32, num_neg=1, neg_weight=5.0, mode=gv.GV_MODE_HOGWILD, total_samples=10, seed=1,
                     pool_capacity=8, lr0=LR0) as ctx:
        buf = torch.empty((100, 2), dtype=torch.int32, device="cuda")
        with pytest.raises(gv.GvError) as e:
            gv.gv_set_adjacency(ctx, g["offsets"], g["adj"])
        assert e.value.code == gv.GV_ESTATE  # no graph yet
        gv.gv_set_degrees(ctx, g["deg"])
        with pytest.raises(gv.GvError) as e:
            gv.gv_augment_device(ctx, buf.data_ptr(), seed=1, count=100)
        assert e.value.code == gv.GV_ESTATE  # no adjacency yet
        wrong = g["offsets"].copy()
        wrong[1:] += 1
        with pytest.raises(gv.GvError) as e:
            gv.gv_set_adjacency(ctx, wrong, np.concatenate([g["adj"], g["adj"][:1]]))
        assert e.value.code == gv.GV_EINVAL  # row lengths differ from the degrees
        gv.gv_set_adjacency(ctx, g["offsets"], g["adj"])
        for bad in (dict(walk_length=65), dict(walk_length=0), dict(window=0), dict(shuffle=2)):
            with pytest.raises(gv.GvError) as e:
                gv.gv_augment_device(ctx, buf.data_ptr(), seed=1, count=100, **bad)
            assert e.value.code == gv.GV_EINVAL
        with pytest.raises(gv.GvError) as e:
            gv.gv_augment_device(ctx, 0, seed=1, count=100)
        assert e.value.code == gv.GV_EINVAL
        assert gv.gv_augment_device(ctx, 0, seed=1, count=0) == 0  # nothing to do


# --------------------------------------------------------------------------- weighted graphs
def test_weighted_graph_end_to_end(gv, tiny_graph):
    """A weighted graph through the library (Sec. 4.3): the negative-sampling table follows the 3/4 power of the
    weighted degree, the device producer walks by edge weight, bit-identical to the oracle and to the host
    producer; pools produced that way train to the oracle's embeddings (deterministic mode, 1e-5)."""
    import torch

    g = tiny_graph
    n, d, K, w, seed, count = g["n"], 64, 2, 2.5, 19, 60_007
    rng = np.random.default_rng(4)
    ew = rng.choice([0.25, 1.0, 4.0, 9.0], size=g["src"].size).astype(np.float32)
    order = np.argsort(np.concatenate([g["src"], g["dst"]]), kind="stable")
    offsets, adj, weights = g["offsets"], g["adj"], np.ascontiguousarray(np.concatenate([ew, ew])[order])
    wdeg = oracle.weighted_degrees(offsets, weights)
    thresh, alias = oracle.alias_build(oracle.weights_pow34(wdeg))
    tables = oracle.walk_tables(offsets, weights)
    vertex, context = random_embeddings(n, d, seed=6)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_DETERMINISTIC, total_samples=2 * count,
                     seed=seed, pool_capacity=count, lr0=LR0) as ctx:
        gv.gv_set_weighted_graph(ctx, offsets, adj, weights)
        gv.gv_build_alias(ctx, 0.75)
        got_t, got_a = gv.gv_get_alias(ctx, n)
        assert np.array_equal(got_t, thresh) and np.array_equal(got_a, alias)
        assert not np.array_equal(got_t, oracle.alias_build(oracle.degree_weights(g["deg"]))[0])  # weights matter
        assert np.array_equal(gv.gv_draw_negatives(ctx, 2**34, 50_000, K), oracle.draw_negatives(seed, 2**34, 50_000, K, thresh, alias))
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        buf = torch.full((count + 2, 2), -1, dtype=torch.int32, device="cuda")
        ref_v, ref_c = vertex.copy(), context.copy()
        for k, (first_walk, shuffle) in enumerate([(0, 1), (2**33, 0)]):
            walks = gv.gv_augment_device(ctx, buf.data_ptr(), seed=77, first_walk=first_walk, count=count, shuffle=shuffle)
            gv.gv_sync(ctx)
            got = buf.cpu().numpy().view(np.uint32)
            ref, ref_walks = oracle.augment_weighted(77, offsets, adj, tables, 40, 5, count, first_walk=first_walk)
            if shuffle:
                ref = oracle.pseudo_shuffle(ref, 5)
            assert walks == ref_walks and np.array_equal(got[:count], ref) and (got[count:] == 0xFFFFFFFF).all()
            host, _ = gv.gv_augment_weighted(offsets, adj, tables, seed=77, first_walk=first_walk, count=count,
                                             shuffle=shuffle, threads=3)
            assert np.array_equal(host, ref)
            gv.gv_train_device_pool(ctx, buf.data_ptr(), count)
            oracle.train(ref_v, ref_c, ref, K=K, first_g=k * count, T=2 * count, lr0=LR0, lr_min_ratio=0.0, w=w,
                         seed=seed, thresh=thresh, alias=alias)
        got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
        got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
        for got, ref in ((got_v, ref_v), (got_c, ref_c)):
            fro, mx = rel_errors(got, ref)
            assert fro <= 1e-5 and mx <= 1e-4, (fro, mx)
        with pytest.raises(gv.GvError) as e:
            gv.gv_set_adjacency(ctx, offsets, adj)
        assert e.value.code == gv.GV_ESTATE  # the weighted adjacency is in place
        bad = weights.copy()
        bad[10] = -1.0
        with pytest.raises(gv.GvError) as e:
            gv.gv_set_weighted_graph(ctx, offsets, adj, bad)
        assert e.value.code == gv.GV_EINVAL


def test_weighted_graph_at_the_size_of_configuration_2(gv, c2_workload):
    """The graph of configuration 2 with edge weights from {1/4, 1, 4, 9} (10^7 adjacency entries, one alias table
    per row): negative-sampling table, negatives, and the pools of the device producer and of the host producer are
    the oracle's bit for bit, also for walk numbers beyond 2^33."""
    import torch

    c2 = c2_workload
    n, offsets, adj = c2["n"], c2["offsets"], c2["adj"]
    weights = W.csr_edge_weights(c2["src"], c2["dst"], seed=12)
    wdeg = oracle.weighted_degrees(offsets, weights)
    thresh, alias = oracle.alias_build(oracle.weights_pow34(wdeg))
    tables = oracle.walk_tables(offsets, weights)
    count = 1 << 20
    with context_for(gv, dim=128, num_neg=1, total_samples=1 << 30, seed=1234, pool_capacity=8) as ctx:
        gv.gv_set_weighted_graph(ctx, offsets, adj, weights)
        gv.gv_build_alias(ctx, 0.75)
        got_t, got_a = gv.gv_get_alias(ctx, n)
        assert np.array_equal(got_t, thresh) and np.array_equal(got_a, alias)
        assert np.array_equal(gv.gv_draw_negatives(ctx, 2**35, 1 << 18, 1), oracle.draw_negatives(1234, 2**35, 1 << 18, 1, thresh, alias))
        buf = torch.empty((count, 2), dtype=torch.int32, device="cuda")
        for first_walk, size in ((0, count), (2**33 + 11, 190 * 1000 + 3)):
            gv.gv_augment_device(ctx, buf.data_ptr(), seed=202, first_walk=first_walk, count=size)
            gv.gv_sync(ctx)
            ref, _ = oracle.augment_weighted(202, offsets, adj, tables, 40, 5, size, first_walk=first_walk)
            ref = oracle.pseudo_shuffle(ref, 5)
            assert np.array_equal(buf[:size].cpu().numpy().view(np.uint32), ref), first_walk
            host, _ = gv.gv_augment_weighted(offsets, adj, tables, seed=202, first_walk=first_walk, count=size, threads=16)
            assert np.array_equal(host, ref), first_walk
    # heavier edges are walked more often: the share of steps along weight-9 edges is far above their share of the edges
    plain, _ = oracle.augment(202, offsets, adj, 40, 5, 190 * 1000)
    assert not np.array_equal(plain, oracle.augment_weighted(202, offsets, adj, tables, 40, 5, 190 * 1000)[0])


# --------------------------------------------------------------------------- orthogonal blocks
@pytest.mark.parametrize("B", [2, 8])
def test_partitions_and_their_alias_tables_are_bit_identical(gv, tiny_graph, B):
    g = tiny_graph
    deg = g["deg"].copy()
    deg[::97] = 0
    seed = 0x1234567890ABCDEF
    with context_for(gv, dim=64, num_neg=3, total_samples=1, pool_capacity=1, partitions=B, seed=seed) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        part, offsets, members, thresh, alias = gv.gv_get_partitions(ctx, g["n"], B)
        rng = np.random.default_rng(B)
        v = rng.integers(g["n"], size=100_003).astype(np.uint32)
        got = gv.gv_draw_negatives_partitioned(ctx, 2**40 + 17, v, 3)
        whole_t, whole_a = gv.gv_get_alias(ctx, g["n"])  # the whole-graph table is still there, unchanged
        plain = gv.gv_draw_negatives(ctx, 5, 1000, 3)
    ref_part = oracle.zigzag_partition(deg, B)
    tables = oracle.partition_alias(deg, B, ref_part)
    assert np.array_equal(part, ref_part)
    for got_table, ref_table in zip((offsets, members, thresh, alias), tables):
        assert np.array_equal(got_table, ref_table)
    assert np.array_equal(got, oracle.draw_negatives_partitioned(seed, 2**40 + 17, v, 3, ref_part, tables))
    ref_t, ref_a = oracle.alias_build(oracle.degree_weights(deg))
    assert np.array_equal(whole_t, ref_t) and np.array_equal(whole_a, ref_a)
    assert np.array_equal(plain, oracle.draw_negatives(seed, 5, 1000, 3, ref_t, ref_a))


def train_blocks(gv, ctx, part, B, pool, threads=4):
    """Redistribute on the host, copy to the device, train block by block."""
    import torch

    sorted_pairs, order, offsets = gv.gv_redistribute_pool(part, B, pool, threads=threads)
    dev_pairs = torch.from_numpy(sorted_pairs.view(np.int32)).cuda()
    dev_order = torch.from_numpy(order.view(np.int32)).cuda()
    torch.cuda.synchronize()
    gv.gv_train_device_blocks(ctx, dev_pairs.data_ptr(), dev_order.data_ptr(), offsets, pool.shape[0])
    gv.gv_sync(ctx)  # the device arrays may go once the launches have ended


@pytest.mark.parametrize("policy", [(TILED, MIXED), (TILED, ATOMIC), (POOL_ORDER, ATOMIC)])
def test_block_training_single_steps(gv, policy):
    """Orthogonal-block training of a sparse pool: samples whose rows nobody else names (negatives restricted to
    the partition of v) equal one oracle step at the position they had in the pool; rows never named stay bit for
    bit.  Two pools in a row: positions continue across calls."""
    n, d, K, w, seed, B = 200_000, 128, 2, 2.5, 31, 8
    sizes = [9001, 4000]
    count = sum(sizes)
    rng = np.random.default_rng(23)
    deg = rng.integers(1, 50, size=n).astype(np.uint32)
    pool = rng.integers(n, size=(count, 2)).astype(np.uint32)
    vertex, context = random_embeddings(n, d, seed=5)
    part = oracle.zigzag_partition(deg, B)
    tables = oracle.partition_alias(deg, B, part)
    negs = oracle.draw_negatives_partitioned(seed, 0, pool[:, 1].copy(), K, part, tables)
    schedule, coherence = policy
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=10 * count, seed=seed,
                     pool_capacity=8, lr0=LR0, coherence=coherence, schedule=schedule, partitions=B) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        train_blocks(gv, ctx, part, B, pool[:sizes[0]])
        train_blocks(gv, ctx, part, B, pool[sizes[0]:])
        assert gv.gv_get_stats(ctx)["samples_trained"] == count
        got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
        got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
    idx, cu, cc = singly_touched(pool, negs, n)
    assert idx.size > 0.3 * count and (idx >= sizes[0]).sum() > 300
    picked = np.concatenate([idx[idx < sizes[0]][:700], idx[idx >= sizes[0]][:700]])
    worst = check_single_steps(pool, negs, picked, 0, 10 * count, K, w, seed, vertex, context, got_v, got_c,
                               tables[2], tables[3])
    assert worst <= 1e-5, worst
    assert np.array_equal(got_v[cu == 0], vertex[cu == 0]) and np.array_equal(got_c[cc == 0], context[cc == 0])
    assert not np.array_equal(got_v[cu > 0], vertex[cu > 0])


@pytest.mark.parametrize("policy", [(TILED, MIXED), (POOL_ORDER, ATOMIC)])
def test_block_training_quality_matches_blocked_oracle(gv, policy):
    """Configuration 1 trained in orthogonal blocks (4 partitions, pools of 2^18 samples = episodes): against the
    oracle run in the same block order with the same restricted negatives, final loss within 2 % and
    link-prediction AUC within 0.005.  The oracle's plain run is printed beside it: what the schedule itself costs."""
    n, src, dst = W.make_graph("tiny", cache=False)
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, 0.05, seed=31)
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    total, d, K, w, B, P = 2_000_000, 128, 1, 5.0, 4, 1 << 18
    pool, _ = oracle.augment(101, offsets, adj, 40, 5, total, shuffle_seed=7)
    pools = [pool[i:i + P] for i in range(0, total, P)]
    eval_pool, _ = oracle.augment(202, offsets, adj, 40, 5, 1 << 18, shuffle_seed=8)
    vertex, context = oracle.init_embeddings(1, n, d)
    part = oracle.zigzag_partition(deg, B)
    tables = oracle.partition_alias(deg, B, part)
    schedule, coherence = policy
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=total, seed=1234,
                     pool_capacity=8, lr0=LR0, coherence=coherence, schedule=schedule, partitions=B) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_set_embeddings(ctx, gv.GV_VERTEX, vertex)
        gv.gv_set_embeddings(ctx, gv.GV_CONTEXT, context)
        for p in pools:
            train_blocks(gv, ctx, part, B, p)
        got_v = gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d)
        got_c = gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d)
    ref_v, ref_c = vertex.copy(), context.copy()
    g = 0
    for p in pools:
        oracle.train_blocked(ref_v, ref_c, p, K=K, first_g=g, T=total, lr0=LR0, lr_min_ratio=0.0, w=w, seed=1234, B=B,
                             part=part, tables=tables)
        g += p.shape[0]
    plain_v, plain_c = run_oracle(deg, K, w, pools, vertex, context, total, 1234)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=32)
    loss = {name: evaluation_loss(deg, v, c, eval_pool, K, w)
            for name, v, c in (("gpu", got_v, got_c), ("blocked", ref_v, ref_c), ("plain", plain_v, plain_c))}
    auc = {name: oracle.link_prediction_auc(v, te_s, te_d, na, nb)
           for name, v in (("gpu", got_v), ("blocked", ref_v), ("plain", plain_v))}
    print(f"blocks policy={policy}: loss gpu {loss['gpu']:.5f} / blocked oracle {loss['blocked']:.5f} / plain oracle "
          f"{loss['plain']:.5f}; auc {auc['gpu']:.4f} / {auc['blocked']:.4f} / {auc['plain']:.4f}")
    assert abs(loss["gpu"] - loss["blocked"]) <= 0.02 * loss["blocked"]
    assert abs(auc["gpu"] - auc["blocked"]) <= 0.005


@pytest.fixture(scope="module")
def blocked_long_run(gv):
    """Configuration 2 under the orthogonal-block schedule as the stored oracle run has it: 8 partitions, 4
    episodes of 8 pools (2^27 samples each) redistributed into the 8 x 8 grid and trained block after block with
    restricted negatives, learning rate decaying to zero over the 32 pools.  Returns per episode
    (pools, loss, oracle loss, auc, oracle auc)."""
    s, reference = read_long_run_reference("c2-blocks")
    n, src, dst = W.make_graph(s["graph"])
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, s["holdout"], seed=s["holdout_seed"])
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    P, pools, d, B, E = s["pool"], s["pools"], s["dim"], s["partitions"], s["episode_pools"]
    walks_per_pool = -(-P // 190)
    eval_pool, _ = gv.gv_augment(offsets, adj, seed=s["eval_walk_seed"], count=s["eval_count"], threads=16)
    eval_pool = eval_pool.copy()
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=s["negative_pair_seed"])
    checkpoints = {k: rest for k, *rest in reference}
    assert pools in checkpoints and all(k % E == 0 for k in checkpoints)
    trajectory = []
    with context_for(gv, dim=d, num_neg=s["num_neg"], neg_weight=s["neg_weight"], mode=gv.GV_MODE_HOGWILD,
                     total_samples=P * pools, seed=s["train_seed"], pool_capacity=8, lr0=s["lr0"], partitions=B) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, s["init_seed"])
        part = gv.gv_get_partitions(ctx, n, B)[0]
        episode = np.empty((E * P, 2), dtype=np.uint32)
        for first in range(0, pools, E):
            for r in range(E):
                gv.gv_augment(offsets, adj, seed=s["walk_seed"], first_walk=(first + r) * walks_per_pool, count=P,
                              threads=16, out=episode[r * P:(r + 1) * P])
            train_blocks(gv, ctx, part, B, episode, threads=16)
            ref_loss, ref_auc, ref_nv, ref_nc = checkpoints[first + E]
            loss = gv.gv_eval_loss(ctx, eval_pool, s["eval_seed"])
            auc = gv.gv_link_prediction_auc(ctx, te_s, te_d, na, nb)
            print(f"blocks long run after {first + E} pools: loss {loss:.4f} vs {ref_loss:.4f}; auc {auc:.4f} vs {ref_auc:.4f}",
                  flush=True)
            trajectory.append((first + E, loss, ref_loss, auc, ref_auc))
        assert gv.gv_get_stats(ctx)["samples_trained"] == P * pools
    return trajectory


def test_block_training_long_run_converges(blocked_long_run):
    """The block schedule at full size learns: the evaluation loss falls from episode to episode and ends within
    5 % of the oracle's run in the same block order (seen: +1.2 % to +2.3 % from run to run; on the way +8 to +10 %
    after the first episode, +5 %, +3 to +4 %: inside a block a row is named 8 x as often as in the pool, so the
    same number of samples in flight lag 8 x further behind it)."""
    losses = [loss for _, loss, _, _, _ in blocked_long_run]
    assert all(later < earlier for earlier, later in zip(losses, losses[1:])), losses
    pools, loss, ref_loss, auc, ref_auc = blocked_long_run[-1]
    assert abs(loss - ref_loss) <= 0.05 * ref_loss


@pytest.mark.xfail(reason="orthogonal blocks on one GPU do not hold the gates of the default schedule at full size "
                          "(final loss +1.2 % to +2.3 % against 2 %, AUC +0.010 to +0.031 against 0.005, relative to the "
                          "blocked oracle): one of the reasons why the schedule is an option and not the default",
                   strict=False)
def test_block_training_long_run_gates(blocked_long_run):
    pools, loss, ref_loss, auc, ref_auc = blocked_long_run[-1]
    assert abs(loss - ref_loss) <= 0.02 * ref_loss
    assert abs(auc - ref_auc) <= 0.005


def test_block_training_argument_errors(gv, tiny_graph):
    import torch

    g = tiny_graph
    pool = np.stack([g["src"][:1000], g["dst"][:1000]], axis=1)
    buf = torch.zeros((1000, 2), dtype=torch.int32, device="cuda")
    order = torch.zeros(1000, dtype=torch.int32, device="cuda")
    offsets = np.zeros(17, dtype=np.uint64)
    with context_for(gv, dim=64, num_neg=1, total_samples=10_000, pool_capacity=8) as ctx:  # no partitions
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        for call in (lambda: gv.gv_get_partitions(ctx, g["n"], 4),
                     lambda: gv.gv_train_device_blocks(ctx, buf.data_ptr(), order.data_ptr(), offsets, 0),
                     lambda: gv.gv_draw_negatives_partitioned(ctx, 0, pool[:, 1].copy(), 1)):
            with pytest.raises(gv.GvError) as e:
                call()
            assert e.value.code == gv.GV_ESTATE
    with context_for(gv, dim=64, num_neg=1, total_samples=10_000, pool_capacity=8, partitions=4) as ctx:
        gv.gv_set_degrees(ctx, g["deg"])
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 1)
        gv.gv_train_device_blocks(ctx, 0, 0, offsets, 0)  # empty pool
        wrong = offsets.copy()
        wrong[-1] = 999
        with pytest.raises(gv.GvError) as e:
            gv.gv_train_device_blocks(ctx, buf.data_ptr(), order.data_ptr(), wrong, 1000)
        assert e.value.code == gv.GV_EINVAL  # offsets do not end at count
        wrong[-1], wrong[3] = 1000, 2000
        with pytest.raises(gv.GvError) as e:
            gv.gv_train_device_blocks(ctx, buf.data_ptr(), order.data_ptr(), wrong, 1000)
        assert e.value.code == gv.GV_EINVAL  # not ascending
        assert gv.gv_get_stats(ctx)["samples_trained"] == 0
    with context_for(gv, dim=64, num_neg=1, total_samples=10_000, pool_capacity=8, partitions=4) as ctx:
        gv.gv_set_degrees(ctx, np.array([3, 0, 0, 0, 0, 0, 0, 0], dtype=np.uint32))
        with pytest.raises(gv.GvError) as e:
            gv.gv_build_alias(ctx, 0.75)  # a partition without any weight
        assert e.value.code == gv.GV_EINVAL


def read_long_run_reference(name="c2"):
    """tests/golden/long_run_<name>.txt: the set-up and the oracle's checkpoints (written by the script beside it)."""
    setup, rows = {}, []
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", f"long_run_{name}.txt")) as f:
        for line in f:
            if line.startswith("#"):
                if " = " in line:
                    key, value = line[1:].strip().split(" = ")
                    setup[key] = value if key == "graph" else float(value) if "." in value else int(value)
                continue
            k, loss, auc, nv, nc = line.split()
            rows.append((int(k), float(loss), float(auc), float(nv), float(nc)))
    return setup, rows


@pytest.mark.parametrize("name,policy", [("c2", (TILED, MIXED)), ("c2", (POOL_ORDER, ATOMIC)), ("c3", (TILED, MIXED))])
def test_long_run_at_full_size_tracks_the_sequential_oracle(gv, name, policy):
    """c2: 32 pools of 2^24 samples (5.4*10^8 samples, learning rate decaying to zero) on the configuration-2
    graph with 1 % of its edges held out; c3: 4 such pools with d = 512 and 5 negatives of weight 1 (the oracle
    needs two minutes per pool there).  Pools are produced on the fly by the library's host producer into the
    pinned slots.  The evaluation loss must be within 2 % of the oracle's at every checkpoint of the stored
    oracle trajectory, and no row may have grown beyond twice the oracle's longest row (asynchronous updates
    that overshoot show up as a few very long rows well before the loss moves); at the end the
    link-prediction AUC must be within 0.005 of the oracle's (this graph has no structure beyond its degrees, so
    its AUC measures how far training has got and still falls steeply when the run ends)."""
    s, reference = read_long_run_reference(name)
    n, src, dst = W.make_graph(s["graph"])
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, s["holdout"], seed=s["holdout_seed"])
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    P, pools, d = s["pool"], s["pools"], s["dim"]
    walks_per_pool = -(-P // 190)
    eval_pool, _ = gv.gv_augment(offsets, adj, seed=s["eval_walk_seed"], count=s["eval_count"], threads=16)
    eval_pool = eval_pool.copy()
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=s["negative_pair_seed"])
    schedule, coherence = policy
    checkpoints = {k: rest for k, *rest in reference}
    assert pools in checkpoints
    with context_for(gv, dim=d, num_neg=s["num_neg"], neg_weight=s["neg_weight"], mode=gv.GV_MODE_HOGWILD,
                     total_samples=P * pools, seed=s["train_seed"], pool_capacity=P, lr0=s["lr0"],
                     coherence=coherence, schedule=schedule) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, s["init_seed"])
        for k in range(pools):
            slot = gv.gv_acquire_pool_slot(ctx, P)
            gv.gv_augment(offsets, adj, seed=s["walk_seed"], first_walk=k * walks_per_pool, count=P, threads=16,
                          out=slot)
            gv.gv_push_pool(ctx, slot, P)
            gv.gv_train_pool(ctx)
            if k + 1 in checkpoints:
                ref_loss, ref_auc, ref_nv, ref_nc = checkpoints[k + 1]
                gv.gv_sync(ctx)
                loss = gv.gv_eval_loss(ctx, eval_pool, s["eval_seed"])
                nv = np.linalg.norm(gv.gv_read_embeddings(ctx, gv.GV_VERTEX, n, d), axis=1).max()
                nc = np.linalg.norm(gv.gv_read_embeddings(ctx, gv.GV_CONTEXT, n, d), axis=1).max()
                print(f"long run {name} {policy} after {k + 1} pools: loss {loss:.4f} vs {ref_loss:.4f}; "
                      f"longest rows {nv:.2f}/{nc:.2f} vs {ref_nv:.2f}/{ref_nc:.2f}")
                assert abs(loss - ref_loss) <= 0.02 * ref_loss
                assert nv <= 2.0 * ref_nv and nc <= 2.0 * ref_nc
        auc = gv.gv_link_prediction_auc(ctx, te_s, te_d, na, nb)
        print(f"long run {name} {policy}: auc {auc:.4f} vs {checkpoints[pools][1]:.4f}")
        assert gv.gv_get_stats(ctx)["samples_trained"] == P * pools
        assert abs(auc - checkpoints[pools][1]) <= 0.005


def test_configuration_4_at_full_size_tracks_the_sequential_oracle(gv):
    """Configuration 4 at its stated size: planted partition, 4*10^6 nodes in 400 communities, 4*10^7
    edges, 1 % held out, d = 128, K = 1, 4*10^9 samples (238 pools of 2^24, learning rate decaying to zero);
    pools written in HBM by the device producer, default asynchronous policy.  The oracle's trajectory is
    stored (`tests/golden/long_run_c4.txt`, one CPU core for two hours); the evaluation loss must be within
    2 % at every checkpoint (one of them lies in the middle of the steep drop), the link-prediction AUC of the
    held-out edges within 0.005 throughout.  The graph has no warm row, so GV_SCHEDULE_AUTO trains it in pool
    order."""
    import torch

    s, reference = read_long_run_reference("c4")
    assert reference, "no checkpoint stored"
    n, src, dst = W.make_graph(s["graph"])
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, s["holdout"], seed=s["holdout_seed"])
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    print(f"configuration 4: graph ready ({n} nodes, {tr_s.size} training edges)", flush=True)
    P, pools, d = s["pool"], s["pools"], s["dim"]
    walks_per_pool = -(-P // 190)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=s["negative_pair_seed"])
    checkpoints = {k: rest for k, *rest in reference}
    last = max(checkpoints)
    with context_for(gv, dim=d, num_neg=s["num_neg"], neg_weight=s["neg_weight"], mode=gv.GV_MODE_HOGWILD,
                     total_samples=P * pools, seed=s["train_seed"], pool_capacity=8, lr0=s["lr0"]) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_set_adjacency(ctx, offsets, adj)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, s["init_seed"])
        eval_buf = torch.empty((s["eval_count"], 2), dtype=torch.int32, device="cuda")
        gv.gv_augment_device(ctx, eval_buf.data_ptr(), seed=s["eval_walk_seed"], count=s["eval_count"])
        gv.gv_sync(ctx)
        eval_pool = eval_buf.cpu().numpy().view(np.uint32)
        bufs = [torch.empty((P, 2), dtype=torch.int32, device="cuda") for _ in range(2)]
        for k in range(last):
            buf = bufs[k % 2]
            gv.gv_augment_device(ctx, buf.data_ptr(), seed=s["walk_seed"], first_walk=k * walks_per_pool, count=P)
            gv.gv_train_device_pool(ctx, buf.data_ptr(), P)
            if k + 1 in checkpoints:
                ref_loss, ref_auc, ref_nv, ref_nc = checkpoints[k + 1]
                gv.gv_sync(ctx)
                loss = gv.gv_eval_loss(ctx, eval_pool, s["eval_seed"])
                auc = gv.gv_link_prediction_auc(ctx, te_s, te_d, na, nb)
                print(f"configuration 4 after {k + 1} pools: loss {loss:.4f} vs {ref_loss:.4f}; "
                      f"auc {auc:.4f} vs {ref_auc:.4f}", flush=True)
                assert abs(loss - ref_loss) <= 0.02 * ref_loss
                assert abs(auc - ref_auc) <= 0.005
        stats = gv.gv_get_stats(ctx)
        assert stats["samples_trained"] == P * last
        assert stats["warm_rows"] == 0 and stats["tiled_launches"] == 0  # the default schedule went pool-order


def test_divergence_is_reported(gv):
    """A star (every sample names the hub) is not what asynchronous mode is for: the tiled policies drive the hub
    rows to NaN, and the next synchronising call says so instead of handing back NaN silently; deterministic mode
    trains the same pool to the oracle's embeddings."""
    n, d, K, w, seed, total = 10_001, 128, 1, 5.0, 1234, 1 << 20
    src = np.zeros(n - 1, dtype=np.uint32)
    dst = np.arange(1, n, dtype=np.uint32)
    deg = W.degrees(n, src, dst)
    offsets, adj = W.csr_from_edges(n, src, dst)
    pool, _ = oracle.augment(7, offsets, adj, 40, 5, total)
    pool = oracle.pseudo_shuffle(pool, 5)
    with context_for(gv, dim=d, num_neg=K, neg_weight=w, total_samples=total, seed=seed, pool_capacity=total, lr0=LR0,
                     schedule=TILED, coherence=ATOMIC) as ctx:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 1)
        gv.gv_push_pool(ctx, pool)
        gv.gv_train_pool(ctx)
        with pytest.raises(gv.GvError) as e:
            gv.gv_sync(ctx)
        assert e.value.code == gv.GV_ESTATE and "diverged" in str(e.value)
        gv.gv_sync(ctx)  # reported once
        assert not np.isfinite(gv.gv_read_embeddings(ctx, gv.GV_VERTEX, 1, d)).all()
    short = pool[:20_000]
    vertex, context = oracle.init_embeddings(1, n, d)
    got_v, got_c, _ = run_deterministic(gv, n, deg, d, K, w, [short], vertex, context, total, seed)
    ref_v, ref_c = run_oracle(deg, K, w, [short], vertex, context, total, seed)
    for got, ref in ((got_v, ref_v), (got_c, ref_c)):
        fro, mx = rel_errors(got, ref)
        assert fro <= 1e-5 and mx <= 1e-4, (fro, mx)
