"""ctypes binding of libgvhot.so: the same calls as include/gvhot.h, with numpy
arrays marshalled to plain pointers.  No arithmetic of the method happens here.
The library must have been built (``python -m paper_1903_00757_amd.build``);
loading fails loudly otherwise -- there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

GV_OK, GV_EINVAL, GV_ENOMEM, GV_ESTATE, GV_EHIP = 0, -1, -2, -3, -4
GV_MODE_HOGWILD, GV_MODE_DETERMINISTIC = 0, 1
GV_VERTEX, GV_CONTEXT = 0, 1
GV_COHERENCE_PLAIN, GV_COHERENCE_AGENT, GV_COHERENCE_ATOMIC_AGENT, GV_COHERENCE_MIXED = 0, 1, 2, 3
GV_SCHEDULE_POOL_ORDER, GV_SCHEDULE_TILED, GV_SCHEDULE_AUTO = 0, 1, 2
GV_NEG_WEIGHT_DEFAULT = -1.0
GV_MAX_POOL_SLOTS = 16
GV_STATIC_SCRATCH_WORDS = 1 << 22
GV_MAX_PARTITIONS = 64
GV_SHUFFLE_NONE, GV_SHUFFLE_PSEUDO = 0, 1

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libgvhot.so")

EXPORTS = [
    "gv_create", "gv_destroy", "gv_last_error", "gv_set_graph", "gv_set_degrees", "gv_build_alias", "gv_get_alias",
    "gv_init_embeddings", "gv_set_embeddings", "gv_read_embeddings", "gv_device_embeddings",
    "gv_acquire_pool_slot", "gv_push_pool", "gv_train_pool", "gv_train_device_pool", "gv_draw_negatives",
    "gv_sync", "gv_get_stats", "gv_set_position", "gv_augment", "gv_eval_loss", "gv_cosine",
    "gv_set_adjacency", "gv_augment_device", "gv_auc", "gv_link_prediction_auc", "gv_train_device_pool_static",
    "gv_get_partitions", "gv_redistribute_pool", "gv_train_device_blocks", "gv_draw_negatives_partitioned",
    "gv_build_walk_tables", "gv_augment_weighted", "gv_set_weighted_graph",
]


class gv_config(C.Structure):
    _fields_ = [
        ("dim", C.c_uint32), ("num_neg", C.c_uint32),
        ("lr0", C.c_float), ("lr_min_ratio", C.c_float), ("neg_weight", C.c_float),
        ("mode", C.c_uint32),
        ("total_samples", C.c_uint64), ("seed", C.c_uint64), ("pool_capacity", C.c_uint64),
        ("device", C.c_int32), ("coherence", C.c_uint32), ("profile", C.c_uint32), ("schedule", C.c_uint32),
        ("pool_slots", C.c_uint32), ("partitions", C.c_uint32), ("track_loss", C.c_uint32),
    ]


class gv_stats(C.Structure):
    _fields_ = [
        ("samples_trained", C.c_uint64), ("pools_trained", C.c_uint64), ("train_launches", C.c_uint64),
        ("batches", C.c_uint64), ("train_kernel_ms", C.c_double), ("timed_launches", C.c_uint64),
        ("h2d_ms", C.c_double), ("h2d_bytes", C.c_uint64), ("tiled_launches", C.c_uint64), ("warm_rows", C.c_uint64),
        ("train_loss_sum", C.c_double), ("train_loss_samples", C.c_uint64),
    ]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class GvError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"gvhot error {code}: {text}")
        self.code = code


_lib = None


def load():
    """Load the built library (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1903_00757_amd.build`")
    # PyTorch-ROCm ships its own HIP runtime; it has to be in the process before this library
    # so that both use one runtime (two runtimes in one process do not both get the GPU).
    import torch  # noqa: F401

    L = C.CDLL(LIB_PATH)
    vp, u32p, f32p = C.c_void_p, C.POINTER(C.c_uint32), C.POINTER(C.c_float)
    L.gv_create.argtypes = [C.POINTER(gv_config), C.POINTER(vp)]
    L.gv_destroy.argtypes = [vp]
    L.gv_destroy.restype = None
    L.gv_last_error.argtypes = [vp]
    L.gv_last_error.restype = C.c_char_p
    L.gv_set_graph.argtypes = [vp, C.c_uint32, C.c_uint64, u32p, u32p]
    L.gv_set_degrees.argtypes = [vp, C.c_uint32, u32p]
    L.gv_build_alias.argtypes = [vp, C.c_double]
    L.gv_get_alias.argtypes = [vp, u32p, u32p]
    L.gv_init_embeddings.argtypes = [vp, C.c_uint64]
    L.gv_set_embeddings.argtypes = [vp, C.c_int, f32p, C.c_uint64, C.c_uint64]
    L.gv_read_embeddings.argtypes = [vp, C.c_int, f32p, C.c_uint64, C.c_uint64]
    L.gv_device_embeddings.argtypes = [vp, C.c_int, C.POINTER(vp)]
    L.gv_acquire_pool_slot.argtypes = [vp, C.POINTER(u32p)]
    L.gv_push_pool.argtypes = [vp, vp, C.c_uint64]
    L.gv_train_pool.argtypes = [vp]
    L.gv_train_device_pool.argtypes = [vp, vp, C.c_uint64]
    L.gv_train_device_pool_static.argtypes = [vp, vp, C.c_uint64]
    u64p = C.POINTER(C.c_uint64)
    L.gv_get_partitions.argtypes = [vp, u32p, u64p, u32p, u32p, u32p]
    L.gv_redistribute_pool.argtypes = [C.c_uint32, u32p, C.c_uint32, vp, C.c_uint64, C.c_uint32, vp, u32p, u64p]
    L.gv_train_device_blocks.argtypes = [vp, vp, vp, u64p, C.c_uint64]
    L.gv_draw_negatives_partitioned.argtypes = [vp, C.c_uint64, C.c_uint64, u32p, u32p]
    L.gv_build_walk_tables.argtypes = [C.c_uint32, u64p, f32p, C.POINTER(C.c_double), u32p, u32p, u32p, u32p]
    L.gv_augment_weighted.argtypes = [C.c_uint32, u64p, u32p, u32p, u32p, u32p, u32p, C.c_uint64, C.c_uint32,
                                      C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, vp, u64p]
    L.gv_set_weighted_graph.argtypes = [vp, C.c_uint32, u64p, u32p, f32p]
    L.gv_draw_negatives.argtypes = [vp, C.c_uint64, C.c_uint64, u32p]
    L.gv_sync.argtypes = [vp]
    L.gv_get_stats.argtypes = [vp, C.POINTER(gv_stats)]
    L.gv_set_position.argtypes = [vp, C.c_uint64]
    L.gv_eval_loss.argtypes = [vp, vp, C.c_uint64, C.c_uint64, C.POINTER(C.c_double)]
    L.gv_cosine.argtypes = [vp, u32p, u32p, C.c_uint64, f32p]
    L.gv_auc.argtypes = [f32p, C.c_uint64, f32p, C.c_uint64, C.POINTER(C.c_double)]
    L.gv_link_prediction_auc.argtypes = [vp, u32p, u32p, C.c_uint64, u32p, u32p, C.c_uint64, C.POINTER(C.c_double)]
    L.gv_augment.argtypes = [C.c_uint32, C.POINTER(C.c_uint64), u32p, C.c_uint64, C.c_uint32, C.c_uint32,
                             C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32, vp, C.POINTER(C.c_uint64)]
    L.gv_set_adjacency.argtypes = [vp, C.POINTER(C.c_uint64), u32p]
    L.gv_augment_device.argtypes = [vp, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32, vp,
                                    C.POINTER(C.c_uint64)]
    for name in EXPORTS:
        if name not in ("gv_destroy", "gv_last_error"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(ctx, rc):
    if rc != GV_OK:
        text = load().gv_last_error(ctx)
        raise GvError(rc, text.decode() if text else "")


def _u32(a):
    a = np.ascontiguousarray(a, dtype=np.uint32)
    return a, a.ctypes.data_as(C.POINTER(C.c_uint32))


def gv_create(*, dim, num_neg, lr0=0.025, lr_min_ratio=0.0, neg_weight=GV_NEG_WEIGHT_DEFAULT, mode=GV_MODE_HOGWILD,
              total_samples, seed=1234, pool_capacity, device=0, coherence=GV_COHERENCE_MIXED, profile=0,
              schedule=GV_SCHEDULE_AUTO, pool_slots=0, partitions=0, track_loss=0):
    cfg = gv_config(dim=dim, num_neg=num_neg, lr0=lr0, lr_min_ratio=lr_min_ratio, neg_weight=neg_weight, mode=mode,
                    total_samples=total_samples, seed=seed, pool_capacity=pool_capacity, device=device,
                    coherence=coherence, profile=profile, schedule=schedule, pool_slots=pool_slots,
                    partitions=partitions, track_loss=track_loss)
    ctx = C.c_void_p()
    rc = load().gv_create(C.byref(cfg), C.byref(ctx))
    _check(None, rc)
    return ctx


def gv_destroy(ctx):
    load().gv_destroy(ctx)


def gv_last_error(ctx=None):
    text = load().gv_last_error(ctx)
    return text.decode() if text else ""


def gv_set_graph(ctx, n, src, dst):
    src, ps = _u32(src)
    dst, pd = _u32(dst)
    if src.size != dst.size:
        raise ValueError("src and dst differ in length")
    _check(ctx, load().gv_set_graph(ctx, n, src.size, ps, pd))


def gv_set_degrees(ctx, deg):
    deg, p = _u32(deg)
    _check(ctx, load().gv_set_degrees(ctx, deg.size, p))


def gv_build_alias(ctx, power=0.75):
    _check(ctx, load().gv_build_alias(ctx, power))


def gv_get_alias(ctx, n):
    thresh = np.empty(n, dtype=np.uint32)
    alias = np.empty(n, dtype=np.uint32)
    _check(ctx, load().gv_get_alias(ctx, thresh.ctypes.data_as(C.POINTER(C.c_uint32)),
                                    alias.ctypes.data_as(C.POINTER(C.c_uint32))))
    return thresh, alias


def gv_init_embeddings(ctx, seed):
    _check(ctx, load().gv_init_embeddings(ctx, seed))


def gv_set_embeddings(ctx, which, rows, row0=0):
    rows = np.ascontiguousarray(rows, dtype=np.float32)
    _check(ctx, load().gv_set_embeddings(ctx, which, rows.ctypes.data_as(C.POINTER(C.c_float)), row0, rows.shape[0]))


def gv_read_embeddings(ctx, which, n, dim, row0=0):
    out = np.empty((n, dim), dtype=np.float32)
    _check(ctx, load().gv_read_embeddings(ctx, which, out.ctypes.data_as(C.POINTER(C.c_float)), row0, n))
    return out


def gv_device_embeddings(ctx, which):
    p = C.c_void_p()
    _check(ctx, load().gv_device_embeddings(ctx, which, C.byref(p)))
    return p.value


def gv_acquire_pool_slot(ctx, capacity):
    """Pinned slot as a writable numpy view of shape (capacity, 2)."""
    p = C.POINTER(C.c_uint32)()
    _check(ctx, load().gv_acquire_pool_slot(ctx, C.byref(p)))
    return np.ctypeslib.as_array(p, shape=(capacity, 2))


def gv_push_pool(ctx, pairs, count=None):
    if not (isinstance(pairs, np.ndarray) and pairs.dtype == np.uint32 and pairs.flags.c_contiguous):
        pairs = np.ascontiguousarray(pairs, dtype=np.uint32)
    count = pairs.shape[0] if count is None else count
    _check(ctx, load().gv_push_pool(ctx, C.c_void_p(pairs.ctypes.data), count))


def gv_train_pool(ctx):
    _check(ctx, load().gv_train_pool(ctx))


def gv_train_device_pool(ctx, dev_ptr, count):
    _check(ctx, load().gv_train_device_pool(ctx, C.c_void_p(dev_ptr), count))


def gv_train_device_pool_static(ctx, dev_ptr, count):
    _check(ctx, load().gv_train_device_pool_static(ctx, C.c_void_p(dev_ptr), count))


def gv_get_partitions(ctx, n, partitions):
    """(part uint32[n], offsets uint64[B+1], members, thresh, alias uint32[n]) of a context with partitions."""
    part = np.empty(n, dtype=np.uint32)
    offsets = np.empty(partitions + 1, dtype=np.uint64)
    members, thresh, alias = (np.empty(n, dtype=np.uint32) for _ in range(3))
    u32 = C.POINTER(C.c_uint32)
    _check(ctx, load().gv_get_partitions(ctx, part.ctypes.data_as(u32), offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                                         members.ctypes.data_as(u32), thresh.ctypes.data_as(u32),
                                         alias.ctypes.data_as(u32)))
    return part, offsets, members, thresh, alias


def gv_redistribute_pool(part, partitions, pairs, threads=1):
    """(sorted pairs uint32[count][2], order uint32[count], block_offsets uint64[B*B+1])."""
    part, pp = _u32(part)
    pairs = np.ascontiguousarray(pairs, dtype=np.uint32)
    count = pairs.shape[0]
    out = np.empty((count, 2), dtype=np.uint32)
    order = np.empty(count, dtype=np.uint32)
    offsets = np.empty(partitions * partitions + 1, dtype=np.uint64)
    rc = load().gv_redistribute_pool(part.size, pp, partitions, C.c_void_p(pairs.ctypes.data), count, threads,
                                     C.c_void_p(out.ctypes.data), order.ctypes.data_as(C.POINTER(C.c_uint32)),
                                     offsets.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc != GV_OK:
        raise GvError(rc, "gv_redistribute_pool: bad argument, node id or partition number")
    return out, order, offsets


def gv_train_device_blocks(ctx, dev_pairs_ptr, dev_order_ptr, block_offsets, count):
    block_offsets = np.ascontiguousarray(block_offsets, dtype=np.uint64)
    _check(ctx, load().gv_train_device_blocks(ctx, C.c_void_p(dev_pairs_ptr), C.c_void_p(dev_order_ptr),
                                              block_offsets.ctypes.data_as(C.POINTER(C.c_uint64)), count))


def gv_draw_negatives_partitioned(ctx, first_g, v, num_neg):
    v, pv = _u32(v)
    out = np.empty((v.size, num_neg), dtype=np.uint32)
    _check(ctx, load().gv_draw_negatives_partitioned(ctx, first_g, v.size, pv, out.ctypes.data_as(C.POINTER(C.c_uint32))))
    return out


def gv_draw_negatives(ctx, first_g, count, num_neg):
    out = np.empty((count, num_neg), dtype=np.uint32)
    _check(ctx, load().gv_draw_negatives(ctx, first_g, count, out.ctypes.data_as(C.POINTER(C.c_uint32))))
    return out


def gv_sync(ctx):
    _check(ctx, load().gv_sync(ctx))


def gv_get_stats(ctx):
    s = gv_stats()
    _check(ctx, load().gv_get_stats(ctx, C.byref(s)))
    return s.as_dict()


def gv_set_position(ctx, next_g):
    _check(ctx, load().gv_set_position(ctx, next_g))


def gv_eval_loss(ctx, pairs, eval_seed):
    pairs = np.ascontiguousarray(pairs, dtype=np.uint32)
    out = C.c_double()
    _check(ctx, load().gv_eval_loss(ctx, C.c_void_p(pairs.ctypes.data), pairs.shape[0], eval_seed, C.byref(out)))
    return out.value


def gv_cosine(ctx, first, second):
    first, pa = _u32(first)
    second, pb = _u32(second)
    if first.size != second.size:
        raise ValueError("first and second differ in length")
    out = np.empty(first.size, dtype=np.float32)
    _check(ctx, load().gv_cosine(ctx, pa, pb, first.size, out.ctypes.data_as(C.POINTER(C.c_float))))
    return out


def gv_auc(pos_scores, neg_scores):
    pos = np.ascontiguousarray(pos_scores, dtype=np.float32)
    neg = np.ascontiguousarray(neg_scores, dtype=np.float32)
    out = C.c_double()
    _check(None, load().gv_auc(pos.ctypes.data_as(C.POINTER(C.c_float)), pos.size,
                               neg.ctypes.data_as(C.POINTER(C.c_float)), neg.size, C.byref(out)))
    return out.value


def gv_link_prediction_auc(ctx, edge_first, edge_second, other_first, other_second):
    ef, pef = _u32(edge_first)
    es, pes = _u32(edge_second)
    of, pof = _u32(other_first)
    os_, pos_ = _u32(other_second)
    if ef.size != es.size or of.size != os_.size:
        raise ValueError("pair arrays differ in length")
    out = C.c_double()
    _check(ctx, load().gv_link_prediction_auc(ctx, pef, pes, ef.size, pof, pos_, of.size, C.byref(out)))
    return out.value


def gv_augment(offsets, adj, *, seed, walk_length=40, window=5, first_walk=0, count, shuffle=GV_SHUFFLE_PSEUDO,
               threads=1, out=None):
    """Fill ``out`` (uint32[count][2], allocated if None; may be a pinned slot view) with walk samples.
    Returns (pairs, walks_used)."""
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    adj = np.ascontiguousarray(adj, dtype=np.uint32)
    if out is None:
        out = np.empty((count, 2), dtype=np.uint32)
    if out.dtype != np.uint32 or not out.flags.c_contiguous or out.size < 2 * count:
        raise ValueError("out must be a C-contiguous uint32 array with room for count pairs")
    walks = C.c_uint64()
    rc = load().gv_augment(offsets.size - 1, offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                           adj.ctypes.data_as(C.POINTER(C.c_uint32)), seed, walk_length, window, first_walk, count,
                           shuffle, threads, C.c_void_p(out.ctypes.data), C.byref(walks))
    if rc != GV_OK:
        raise GvError(rc, "gv_augment: bad argument or ill-formed adjacency" if rc == GV_EINVAL
                      else "gv_augment: workers could not be set up")
    return out[:count], walks.value


def gv_build_walk_tables(offsets, weights):
    """(wdeg float64[n], node_thresh, node_alias uint32[n], nbr_thresh, nbr_alias uint32[len(weights)])."""
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    n = offsets.size - 1
    wdeg = np.empty(n, dtype=np.float64)
    node_thresh, node_alias = np.empty(n, dtype=np.uint32), np.empty(n, dtype=np.uint32)
    nbr_thresh, nbr_alias = np.zeros(weights.size, dtype=np.uint32), np.zeros(weights.size, dtype=np.uint32)
    u32 = C.POINTER(C.c_uint32)
    rc = load().gv_build_walk_tables(n, offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                                     weights.ctypes.data_as(C.POINTER(C.c_float)),
                                     wdeg.ctypes.data_as(C.POINTER(C.c_double)), node_thresh.ctypes.data_as(u32),
                                     node_alias.ctypes.data_as(u32), nbr_thresh.ctypes.data_as(u32),
                                     nbr_alias.ctypes.data_as(u32))
    if rc != GV_OK:
        raise GvError(rc, "gv_build_walk_tables: bad argument or a row without weight")
    return wdeg, node_thresh, node_alias, nbr_thresh, nbr_alias


def gv_augment_weighted(offsets, adj, tables, *, seed, walk_length=40, window=5, first_walk=0, count,
                        shuffle=GV_SHUFFLE_PSEUDO, threads=1, out=None):
    """gv_augment on a weighted graph; ``tables`` = (node_thresh, node_alias, nbr_thresh, nbr_alias)."""
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    adj = np.ascontiguousarray(adj, dtype=np.uint32)
    if out is None:
        out = np.empty((count, 2), dtype=np.uint32)
    if out.dtype != np.uint32 or not out.flags.c_contiguous or out.size < 2 * count:
        raise ValueError("out must be a C-contiguous uint32 array with room for count pairs")
    t = [np.ascontiguousarray(x, dtype=np.uint32) for x in tables]
    u32 = C.POINTER(C.c_uint32)
    walks = C.c_uint64()
    rc = load().gv_augment_weighted(offsets.size - 1, offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                                    adj.ctypes.data_as(u32), t[0].ctypes.data_as(u32), t[1].ctypes.data_as(u32),
                                    t[2].ctypes.data_as(u32), t[3].ctypes.data_as(u32), seed, walk_length, window,
                                    first_walk, count, shuffle, threads, C.c_void_p(out.ctypes.data), C.byref(walks))
    if rc != GV_OK:
        raise GvError(rc, "gv_augment_weighted: bad argument or ill-formed adjacency / tables")
    return out[:count], walks.value


def gv_set_weighted_graph(ctx, offsets, adj, weights):
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    adj = np.ascontiguousarray(adj, dtype=np.uint32)
    weights = np.ascontiguousarray(weights, dtype=np.float32)
    if adj.size != weights.size:
        raise ValueError("adj and weights differ in length")
    _check(ctx, load().gv_set_weighted_graph(ctx, offsets.size - 1, offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                                             adj.ctypes.data_as(C.POINTER(C.c_uint32)),
                                             weights.ctypes.data_as(C.POINTER(C.c_float))))


def gv_set_adjacency(ctx, offsets, adj):
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    adj = np.ascontiguousarray(adj, dtype=np.uint32)
    _check(ctx, load().gv_set_adjacency(ctx, offsets.ctypes.data_as(C.POINTER(C.c_uint64)),
                                        adj.ctypes.data_as(C.POINTER(C.c_uint32))))


def gv_augment_device(ctx, device_ptr, *, seed, walk_length=40, window=5, first_walk=0, count,
                      shuffle=GV_SHUFFLE_PSEUDO):
    """Fill device memory at ``device_ptr`` (room for count x 2 uint32) with walk samples; returns walks used."""
    walks = C.c_uint64()
    _check(ctx, load().gv_augment_device(ctx, seed, walk_length, window, first_walk, count, shuffle,
                                         C.c_void_p(device_ptr), C.byref(walks)))
    return walks.value
