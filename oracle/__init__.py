"""CPU oracle of the embedding-training hot path -- TEST INFRASTRUCTURE ONLY.

Python face of ``gv_oracle.c`` (argument marshalling) plus the two evaluation
routines that are one library call each (AUC by average ranks).  Nothing in
the product package may import this; tests, the smoke check and the benchmark's
CPU-baseline leg do.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build as _build

STREAM_NEG, STREAM_INIT, STREAM_EVAL, STREAM_SHUFFLE, STREAM_WALK = 0, 1, 2, 3, 4

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build())
        u32p, u64p, f32p, f64p = (C.POINTER(C.c_uint32), C.POINTER(C.c_uint64),
                                  C.POINTER(C.c_float), C.POINTER(C.c_double))
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_philox4x32_10.restype = None
        L.orc_alias_build.argtypes = [C.c_uint64, f64p, u32p, u32p]
        L.orc_alias_build.restype = C.c_int
        L.orc_degree_weights.argtypes = [C.c_uint64, u32p, f64p]
        L.orc_degree_weights.restype = None
        L.orc_draw_negatives.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32,
                                         C.c_uint64, u32p, u32p, u32p]
        L.orc_draw_negatives.restype = None
        L.orc_augment.argtypes = [C.c_uint64, C.c_uint64, u64p, u32p, C.c_uint32, C.c_uint32,
                                  C.c_uint64, C.c_uint64, u32p]
        L.orc_augment.restype = C.c_uint64
        L.orc_weighted_degrees.argtypes = [C.c_uint64, u64p, f32p, f64p]
        L.orc_weighted_degrees.restype = None
        L.orc_weights_pow34.argtypes = [C.c_uint64, f64p, f64p]
        L.orc_weights_pow34.restype = None
        L.orc_neighbor_alias.argtypes = [C.c_uint64, u64p, f32p, u32p, u32p]
        L.orc_neighbor_alias.restype = C.c_int
        L.orc_augment_weighted.argtypes = [C.c_uint64, C.c_uint64, u64p, u32p, u32p, u32p, u32p, u32p, C.c_uint32,
                                           C.c_uint32, C.c_uint64, C.c_uint64, u32p]
        L.orc_augment_weighted.restype = C.c_uint64
        L.orc_shuffle.argtypes = [C.c_uint64, C.c_uint64, u32p]
        L.orc_shuffle.restype = None
        L.orc_pseudo_shuffle.argtypes = [C.c_uint64, C.c_uint32, u32p, u32p]
        L.orc_pseudo_shuffle.restype = None
        L.orc_init_embeddings.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, f32p, f32p]
        L.orc_init_embeddings.restype = None
        L.orc_init_vertex_rows.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_uint32, f32p]
        L.orc_init_vertex_rows.restype = None
        L.orc_learning_rate.argtypes = [C.c_float, C.c_float, C.c_uint64, C.c_uint64]
        L.orc_learning_rate.restype = C.c_float
        L.orc_train.argtypes = [f32p, f32p, C.c_uint64, C.c_uint32, C.c_uint32, u32p, C.c_uint64,
                                C.c_uint64, C.c_uint64, C.c_float, C.c_float, C.c_float, C.c_uint64,
                                u32p, u32p, u32p]
        L.orc_train.restype = None
        L.orc_train_ordered.argtypes = L.orc_train.argtypes + [u32p]
        L.orc_train_ordered.restype = None
        L.orc_train_tracked.argtypes = L.orc_train_ordered.argtypes + [f64p]
        L.orc_train_tracked.restype = None
        L.orc_zigzag_partition.argtypes = [C.c_uint64, u32p, C.c_uint32, u32p]
        L.orc_zigzag_partition.restype = None
        L.orc_partition_alias.argtypes = [C.c_uint64, u32p, C.c_uint32, u32p, u64p, u32p, u32p, u32p]
        L.orc_partition_alias.restype = C.c_int
        L.orc_draw_negatives_partitioned.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32,
                                                     u32p, u32p, u64p, u32p, u32p, u32p, u32p]
        L.orc_draw_negatives_partitioned.restype = None
        L.orc_block_order.argtypes = [C.c_uint64, u32p, C.c_uint32, u32p, u32p, u64p]
        L.orc_block_order.restype = None
        L.orc_loss.argtypes = [f32p, f32p, C.c_uint64, C.c_uint32, C.c_uint32, u32p, C.c_uint64,
                               C.c_float, C.c_uint64, C.c_uint32, u32p, u32p]
        L.orc_loss.restype = C.c_double
        L.orc_cosine.argtypes = [f32p, C.c_uint32, u32p, u32p, C.c_uint64, f64p]
        L.orc_cosine.restype = None
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _arr(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def philox4x32_10(ctr, key):
    c = _arr(ctr, np.uint32)
    k = _arr(key, np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(out, C.c_uint32))
    return out


def degree_weights(deg):
    deg = _arr(deg, np.uint32)
    q = np.empty(deg.size, dtype=np.float64)
    lib().orc_degree_weights(deg.size, _p(deg, C.c_uint32), _p(q, C.c_double))
    return q


def alias_build(q):
    q = _arr(q, np.float64)
    thresh = np.empty(q.size, dtype=np.uint32)
    alias = np.empty(q.size, dtype=np.uint32)
    rc = lib().orc_alias_build(q.size, _p(q, C.c_double), _p(thresh, C.c_uint32), _p(alias, C.c_uint32))
    if rc:
        raise ValueError(f"orc_alias_build failed ({rc})")
    return thresh, alias


def draw_negatives(seed, first_g, count, K, thresh, alias, stream=STREAM_NEG):
    out = np.empty((count, K), dtype=np.uint32)
    lib().orc_draw_negatives(seed, stream, first_g, count, K, thresh.size,
                             _p(thresh, C.c_uint32), _p(alias, C.c_uint32), _p(out, C.c_uint32))
    return out


def augment(seed, offsets, adj, walk_length, window, count, first_walk=0, shuffle_seed=None):
    """Pool of ``count`` pairs from walks ``first_walk, first_walk+1, ...``;
    shuffled with ``shuffle_seed`` unless it is None.  Returns (pairs, walks)."""
    offsets = _arr(offsets, np.uint64)
    adj = _arr(adj, np.uint32)
    pairs = np.empty((count, 2), dtype=np.uint32)
    walks = lib().orc_augment(seed, offsets.size - 1, _p(offsets, C.c_uint64), _p(adj, C.c_uint32),
                              walk_length, window, first_walk, count, _p(pairs, C.c_uint32))
    if shuffle_seed is not None:
        lib().orc_shuffle(shuffle_seed, count, _p(pairs, C.c_uint32))
    return pairs, int(walks)


def weighted_degrees(offsets, weights):
    offsets = _arr(offsets, np.uint64)
    weights = _arr(weights, np.float32)
    out = np.empty(offsets.size - 1, dtype=np.float64)
    lib().orc_weighted_degrees(out.size, _p(offsets, C.c_uint64), _p(weights, C.c_float), _p(out, C.c_double))
    return out


def weights_pow34(wdeg):
    wdeg = _arr(wdeg, np.float64)
    q = np.empty_like(wdeg)
    lib().orc_weights_pow34(wdeg.size, _p(wdeg, C.c_double), _p(q, C.c_double))
    return q


def neighbor_alias(offsets, weights):
    """Per-row alias tables over the edge weights: (thresh, alias) per adjacency entry, alias local to the row."""
    offsets = _arr(offsets, np.uint64)
    weights = _arr(weights, np.float32)
    thresh = np.zeros(weights.size, dtype=np.uint32)
    alias = np.zeros(weights.size, dtype=np.uint32)
    rc = lib().orc_neighbor_alias(offsets.size - 1, _p(offsets, C.c_uint64), _p(weights, C.c_float),
                                  _p(thresh, C.c_uint32), _p(alias, C.c_uint32))
    if rc:
        raise ValueError("an adjacency row has no weight")
    return thresh, alias


def walk_tables(offsets, weights):
    """Everything a weighted walk draws from: (node_thresh, node_alias, nbr_thresh, nbr_alias)."""
    node_thresh, node_alias = alias_build(weighted_degrees(offsets, weights))
    nbr_thresh, nbr_alias = neighbor_alias(offsets, weights)
    return node_thresh, node_alias, nbr_thresh, nbr_alias


def augment_weighted(seed, offsets, adj, tables, walk_length, window, count, first_walk=0):
    offsets = _arr(offsets, np.uint64)
    adj = _arr(adj, np.uint32)
    node_thresh, node_alias, nbr_thresh, nbr_alias = tables
    pairs = np.empty((count, 2), dtype=np.uint32)
    walks = lib().orc_augment_weighted(seed, offsets.size - 1, _p(offsets, C.c_uint64), _p(adj, C.c_uint32),
                                       _p(node_thresh, C.c_uint32), _p(node_alias, C.c_uint32),
                                       _p(nbr_thresh, C.c_uint32), _p(nbr_alias, C.c_uint32), walk_length, window,
                                       first_walk, count, _p(pairs, C.c_uint32))
    return pairs, int(walks)


def shuffle(seed, pairs):
    pairs = np.array(pairs, dtype=np.uint32, order="C")
    lib().orc_shuffle(seed, pairs.shape[0], _p(pairs, C.c_uint32))
    return pairs


def pseudo_shuffle(pairs, s):
    pairs = np.ascontiguousarray(pairs, dtype=np.uint32)
    out = np.empty_like(pairs)
    lib().orc_pseudo_shuffle(pairs.shape[0], s, _p(pairs, C.c_uint32), _p(out, C.c_uint32))
    return out


def init_embeddings(seed, n, d):
    vertex = np.empty((n, d), dtype=np.float32)
    context = np.empty((n, d), dtype=np.float32)
    lib().orc_init_embeddings(seed, n, d, _p(vertex, C.c_float), _p(context, C.c_float))
    return vertex, context


def init_vertex_rows(seed, row0, rows, d):
    """Initial vertex rows row0 .. row0+rows-1 (the initial value of a row depends on nothing else)."""
    vertex = np.empty((rows, d), dtype=np.float32)
    lib().orc_init_vertex_rows(seed, row0, rows, d, _p(vertex, C.c_float))
    return vertex


def learning_rate(lr0, lr_min_ratio, g, T):
    return float(lib().orc_learning_rate(lr0, lr_min_ratio, g, T))


def zigzag_partition(deg, B):
    """Partition number of every node (uint32[n]): degree-sorted nodes dealt back and forth."""
    deg = _arr(deg, np.uint32)
    part = np.empty(deg.size, dtype=np.uint32)
    lib().orc_zigzag_partition(deg.size, _p(deg, C.c_uint32), B, _p(part, C.c_uint32))
    return part


def partition_alias(deg, B, part):
    """One alias table per partition, concatenated: (offsets uint64[B+1], members, thresh, alias uint32[n])."""
    deg = _arr(deg, np.uint32)
    part = _arr(part, np.uint32)
    offsets = np.empty(B + 1, dtype=np.uint64)
    members = np.empty(deg.size, dtype=np.uint32)
    thresh = np.empty(deg.size, dtype=np.uint32)
    alias = np.empty(deg.size, dtype=np.uint32)
    rc = lib().orc_partition_alias(deg.size, _p(deg, C.c_uint32), B, _p(part, C.c_uint32), _p(offsets, C.c_uint64),
                                   _p(members, C.c_uint32), _p(thresh, C.c_uint32), _p(alias, C.c_uint32))
    if rc:
        raise ValueError("a partition has no weight")
    return offsets, members, thresh, alias


def draw_negatives_partitioned(seed, first_g, v, K, part, tables, stream=STREAM_NEG):
    """Negatives of positive samples first_g .. with context nodes ``v``, each from the partition of its v."""
    offsets, members, thresh, alias = tables
    v = _arr(v, np.uint32)
    part = _arr(part, np.uint32)
    out = np.empty((v.size, K), dtype=np.uint32)
    lib().orc_draw_negatives_partitioned(seed, stream, first_g, v.size, K, _p(v, C.c_uint32), _p(part, C.c_uint32),
                                         _p(offsets, C.c_uint64), _p(members, C.c_uint32), _p(thresh, C.c_uint32),
                                         _p(alias, C.c_uint32), _p(out, C.c_uint32))
    return out


def block_order(pairs, B, part):
    """(order uint32[count], block_offsets uint64[B*B+1]) of the pool under the orthogonal-block schedule."""
    pairs = _arr(pairs, np.uint32)
    part = _arr(part, np.uint32)
    order = np.empty(pairs.shape[0], dtype=np.uint32)
    block_offsets = np.empty(B * B + 1, dtype=np.uint64)
    lib().orc_block_order(pairs.shape[0], _p(pairs, C.c_uint32), B, _p(part, C.c_uint32), _p(order, C.c_uint32),
                          _p(block_offsets, C.c_uint64))
    return order, block_offsets


def train_blocked(vertex, context, pairs, *, K, first_g, T, lr0, lr_min_ratio, w, seed, B, part, tables):
    """Sequential SGD over ``pairs`` in orthogonal-block order with negatives restricted to the partition of
    each sample's context node; a sample keeps the position (negatives, learning rate) of its place in the pool."""
    pairs = _arr(pairs, np.uint32)
    negatives = draw_negatives_partitioned(seed, first_g, pairs[:, 1].copy(), K, part, tables)
    order, _ = block_order(pairs, B, part)
    train(vertex, context, pairs, K=K, first_g=first_g, T=T, lr0=lr0, lr_min_ratio=lr_min_ratio, w=w, seed=seed,
          thresh=tables[2], alias=tables[3], negatives=negatives, order=order)


def train(vertex, context, pairs, *, K, first_g, T, lr0, lr_min_ratio, w, seed, thresh, alias, negatives=None,
          order=None, return_loss=False):
    """In-place sequential SGD over ``pairs``; ``vertex``/``context`` must be
    C-contiguous float32 arrays of shape (n, d).  ``order``: the sequence in which the samples are taken
    (indices into ``pairs``), pool order when None.  ``return_loss``: return the sum over the samples of the
    loss each of them saw before its step."""
    assert vertex.dtype == np.float32 and context.dtype == np.float32
    assert vertex.flags.c_contiguous and context.flags.c_contiguous
    pairs = _arr(pairs, np.uint32)
    n, d = vertex.shape
    negp = None
    if negatives is not None:
        negatives = _arr(negatives, np.uint32)
        assert negatives.size == pairs.shape[0] * K
        negp = _p(negatives, C.c_uint32)
    orderp = None
    if order is not None:
        order = _arr(order, np.uint32)
        assert order.size == pairs.shape[0]
        orderp = _p(order, C.c_uint32)
    seen = np.zeros(1, dtype=np.float64)
    lib().orc_train_tracked(_p(vertex, C.c_float), _p(context, C.c_float), n, d, K, _p(pairs, C.c_uint32),
                            pairs.shape[0], first_g, T, lr0, lr_min_ratio, w, seed,
                            _p(thresh, C.c_uint32), _p(alias, C.c_uint32), negp, orderp,
                            _p(seen, C.c_double) if return_loss else None)
    return float(seen[0]) if return_loss else None


def loss(vertex, context, pairs, *, K, w, seed, thresh, alias, stream=STREAM_EVAL):
    pairs = _arr(pairs, np.uint32)
    vertex = _arr(vertex, np.float32)
    context = _arr(context, np.float32)
    n, d = vertex.shape
    return float(lib().orc_loss(_p(vertex, C.c_float), _p(context, C.c_float), n, d, K,
                                _p(pairs, C.c_uint32), pairs.shape[0], w, seed, stream,
                                _p(thresh, C.c_uint32), _p(alias, C.c_uint32)))


def cosine(vertex, a, b):
    vertex = _arr(vertex, np.float32)
    a = _arr(a, np.uint32)
    b = _arr(b, np.uint32)
    out = np.empty(a.size, dtype=np.float64)
    lib().orc_cosine(_p(vertex, C.c_float), vertex.shape[1], _p(a, C.c_uint32), _p(b, C.c_uint32),
                     a.size, _p(out, C.c_double))
    return out


def auc(pos_scores, neg_scores):
    """Area under the ROC curve as the rank statistic
    (sum of positive ranks - P(P+1)/2) / (P*N), ties sharing their mean rank."""
    from scipy.stats import rankdata

    pos = np.asarray(pos_scores, dtype=np.float64)
    neg = np.asarray(neg_scores, dtype=np.float64)
    ranks = rankdata(np.concatenate([pos, neg]), method="average")
    P, N = pos.size, neg.size
    return float((ranks[:P].sum() - P * (P + 1) / 2.0) / (P * N))


def link_prediction_auc(vertex, test_src, test_dst, neg_a, neg_b):
    """Sec. 4.5 protocol: held-out edges against as many uniformly drawn node
    pairs, each scored by the cosine of the two vertex rows."""
    return auc(cosine(vertex, test_src, test_dst), cosine(vertex, neg_a, neg_b))
