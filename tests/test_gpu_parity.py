"""Parity of the HIP path against the CPU oracle, through the C boundary (needs a GPU)."""
import contextlib

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


@pytest.mark.parametrize("d", [64, 128, 512])
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
                                         (512, 5, 1.0, 20_011), (128, 5, 1.0, 50_000), (128, 4, 1.25, 1)])
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
POOL_ORDER, GROUPED = 0, 1
PLAIN, AGENT, ATOMIC, MIXED = 0, 1, 2, 3
ALL_POLICIES = [(POOL_ORDER, PLAIN), (POOL_ORDER, AGENT), (POOL_ORDER, ATOMIC), (GROUPED, AGENT), (GROUPED, ATOMIC),
                (GROUPED, MIXED)]
# policies that never drop an update of a contended row: these are held to the quality gate
LOSSLESS_POLICIES = [(POOL_ORDER, ATOMIC), (GROUPED, ATOMIC), (GROUPED, MIXED)]


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
@pytest.mark.parametrize("d,K", [(128, 1), (64, 1), (256, 2), (512, 5)])
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
