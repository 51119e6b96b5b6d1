#!/usr/bin/env python3
"""Benchmark of the training hot path on one MI355X.

A step = one pool of 2^24 positive samples of configuration 2 (Chung-Lu graph,
10^6 nodes / 5*10^6 edges, d = 128, K = 1) through the whole path: pool copy
host -> device from a pinned slot, sample read, negative draw, row gathers, dot
products, sigmoid-gradient, in-place updates.  Eight pools are produced once
(the library's own producer: walks of length 40, pairs within distance 5,
pseudo shuffle) into the context's ring of pinned slots and then cycled with no
host work in the loop; the copy of a pool overlaps the training of the pools
before it.  The same steps are also timed with the pools already resident in
HBM.  Every leg is timed three times (median and min are printed).
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import threading
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0
REPETITIONS = 3
RING = 8
# HBM bytes per launch measured with rocprofv3 counters in separate runs: the figures and the commands that
# produced them are kept in this file (workload, schedule, coherence, bytes per launch, source summary)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")
SCHEDULES = ["pool-order", "tiled", "auto"]
COHERENCES = ["plain", "agent", "atomic-agent", "mixed"]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes_per_sample(dim: int, num_neg: int) -> int:
    """Each of the 2+K rows is read once and written once (4d bytes each way), plus the
    8-byte sample and one 8-byte alias entry per negative."""
    return 2 * (2 + num_neg) * 4 * dim + 8 + 8 * num_neg


def profiled_traffic(workload: str, schedule: str, coherence: str):
    """(bytes per launch, name of the profile summary) from the tracked table, or (None, None)."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                cols = line.split()
                if len(cols) >= 5 and not line.startswith("#") and cols[:3] == [workload, schedule, coherence]:
                    return float(cols[3]), cols[4]
    except OSError:
        pass
    return None, None


def cpu_baseline(offsets, adj, deg, cfg, seed, samples_one_core, samples_per_thread):
    """The sequential oracle, as it stands, on a bounded slice of the same workload: once on one core, and
    once as the same plain loop run lock-free on all host cores (every thread trains its own slice of the pool
    on the shared matrices, as asynchronous SGD on a CPU does)."""
    import oracle

    import workloads as W

    n, dim, K, w, total = deg.size, cfg["dim"], cfg["num_neg"], cfg["neg_weight"], cfg["total_samples"]
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    vertex, context = oracle.init_embeddings(1, n, dim)
    cores = max(1, min(os.cpu_count() or 1, 16))
    need = max(samples_one_core, samples_per_thread * cores)
    if adj is not None:
        pool, _ = oracle.augment(100 * cfg["number"], offsets, adj, W.configs.WALK_LENGTH, W.configs.WINDOW, need)
        pool = oracle.pseudo_shuffle(pool, W.configs.WINDOW)
        what = "walk pool of the same graph (the oracle's own augmentation and pseudo shuffle)"
    else:
        pool = W.marginal_pool(deg, need, seed=100 * cfg["number"])
        what = "pool with endpoints from the degree marginal"
    kw = dict(K=K, T=total, lr0=0.025, lr_min_ratio=0.0, w=w, seed=seed, thresh=thresh, alias=alias)
    part = pool[:samples_one_core]
    t0 = time.perf_counter()
    oracle.train(vertex, context, part, first_g=0, **kw)
    dt = time.perf_counter() - t0
    out = {"value": part.shape[0] / dt, "unit": "positive samples/s", "cores": 1, "kind": "oracle",
           "sample": f"first {part.shape[0]} samples of a {what}, sequential C oracle (fp64 arithmetic), {dt:.1f} s"}

    def work(t):
        lo = t * samples_per_thread
        oracle.train(vertex, context, pool[lo:lo + samples_per_thread], first_g=lo, **kw)

    threads = [threading.Thread(target=work, args=(t,)) for t in range(cores)]
    t0 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    dt = time.perf_counter() - t0
    out["all_cores"] = {"value": cores * samples_per_thread / dt, "unit": "positive samples/s", "cores": cores,
                        "kind": "oracle", "sample": f"{cores} threads x {samples_per_thread} samples of the same pool, the "
                        f"same loop run lock-free on shared matrices, {dt:.1f} s"}
    # configuration 1 whole (2*10^6 samples on 10^4 nodes: matrices that fit the host caches)
    tiny = W.CONFIGS["tiny"]
    tn, tsrc, tdst = W.make_graph("tiny")
    tdeg = W.degrees(tn, tsrc, tdst)
    toff, tadj = W.csr_from_edges(tn, tsrc, tdst)
    tpool, _ = oracle.augment(100 * tiny["number"], toff, tadj, W.configs.WALK_LENGTH, W.configs.WINDOW, tiny["pool"])
    tpool = oracle.pseudo_shuffle(tpool, W.configs.WINDOW)
    tt, ta = oracle.alias_build(oracle.degree_weights(tdeg))
    tv, tc = oracle.init_embeddings(1, tn, tiny["dim"])
    t0 = time.perf_counter()
    oracle.train(tv, tc, tpool, first_g=0, K=tiny["num_neg"], T=tiny["total_samples"], lr0=0.025, lr_min_ratio=0.0,
                 w=tiny["neg_weight"], seed=seed, thresh=tt, alias=ta)
    dt = time.perf_counter() - t0
    out["configuration_1"] = {"value": tpool.shape[0] / dt, "unit": "positive samples/s", "cores": 1, "kind": "oracle",
                              "sample": f"all {tpool.shape[0]} samples of configuration 1, {dt:.1f} s"}
    return out


def timed_legs(gv, ctx, run_steps, steps):
    """REPETITIONS x `steps` steps, each repetition bracketed by a full synchronisation; per repetition the wall
    time and the event-timed mean duration of its training launches."""
    import torch

    reps = []
    for _ in range(REPETITIONS):
        gv.gv_sync(ctx)
        torch.cuda.synchronize()
        before = gv.gv_get_stats(ctx)
        t0 = time.perf_counter()
        run_steps(steps)
        gv.gv_sync(ctx)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        after = gv.gv_get_stats(ctx)
        launches = max(after["timed_launches"] - before["timed_launches"], 1)
        reps.append({"wall_s": wall, "kernel_ms": (after["train_kernel_ms"] - before["train_kernel_ms"]) / launches,
                     "h2d_ms": after["h2d_ms"] - before["h2d_ms"], "h2d_bytes": after["h2d_bytes"] - before["h2d_bytes"]})
    return reps


def summarise(reps, steps, P):
    walls = sorted(r["wall_s"] for r in reps)
    median = next(r for r in reps if r["wall_s"] == walls[len(walls) // 2])
    return median, {"samples_per_s_median": steps * P / median["wall_s"], "samples_per_s_best": steps * P / walls[0],
                    "ms_per_step": [r["wall_s"] / steps * 1e3 for r in reps],
                    "kernel_ms": [r["kernel_ms"] for r in reps]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "tiny", "c5-marginal", "c5"])
    ap.add_argument("--coherence", type=int, default=3, help="GV_COHERENCE_* of the asynchronous launches")
    ap.add_argument("--schedule", type=int, default=2, help="GV_SCHEDULE_* of the asynchronous launches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-online", action="store_true", help="skip the legs with pools produced on the fly")
    ap.add_argument("--cpu-samples", type=int, default=1 << 24)
    ap.add_argument("--blocked-partitions", type=int, default=0,
                    help="also time the orthogonal-block schedule (Sec. 3.2) with this many partitions")
    ap.add_argument("--episode-pools", type=int, default=8, help="pools per episode of the orthogonal-block leg")
    ap.add_argument("--weighted", action="store_true",
                    help="put edge weights from {1/4, 1, 4, 9} on the graph (Sec. 4.3): weighted walks, negatives from "
                         "the weighted degree")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference point for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1")

    import torch

    import paper_1903_00757_amd as gv
    import workloads as W

    gv.load()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cfg = W.CONFIGS[args.workload]
    dim, K, w = cfg["dim"], cfg["num_neg"], cfg["neg_weight"]
    P = cfg["pool"]
    total = cfg["total_samples"]
    L, s = W.configs.WALK_LENGTH, W.configs.WINDOW
    walks_per_pool = -(-P // sum(L + 1 - delta for delta in range(1, s + 1)))
    threads = min(16, os.cpu_count() or 1)

    t0 = time.perf_counter()
    if cfg["graph"] == "expected_degrees":
        # too large to walk inside a benchmark run: degrees from the model, endpoints from their marginal
        n, deg = W.expected_degrees(args.workload)
        offsets = adj = None
        edges = cfg["edges"]
        args.no_online = True
        log(f"degrees {args.workload}: n={n} ({time.perf_counter() - t0:.1f} s)")
    elif cfg["graph"] == "chung_lu_on_device":
        # the graph is built on the GPU with torch (sorting 3.6*10^9 adjacency entries on the host would take
        # longer than everything else together) and handed to the library from host memory like any other
        from workloads import device_graphs

        off_t, adj_t = device_graphs.chung_lu_csr(cfg["n"], cfg["edges"], cfg["gamma"], cfg["number"], progress=log)
        offsets, adj = device_graphs.to_host_csr(off_t, adj_t)
        del off_t, adj_t
        torch.cuda.empty_cache()
        n, edges = cfg["n"], adj.size // 2
        deg = np.diff(offsets).astype(np.uint32)
        args.no_cpu_baseline = True  # the oracle's matrices of this size take minutes to initialise on the host
        log(f"graph {args.workload}: n={n} edges={edges} max degree {deg.max()} ({time.perf_counter() - t0:.1f} s)")
    else:
        n, src, dst = W.make_graph(args.workload)
        deg = W.degrees(n, src, dst)
        offsets, adj = W.csr_from_edges(n, src, dst)
        edges = src.size
        log(f"graph {args.workload}: n={n} edges={edges} ({time.perf_counter() - t0:.1f} s)")
    weights = tables = None
    if args.weighted:
        if adj is None or cfg["graph"] == "chung_lu_on_device":
            sys.exit("bench.py: --weighted needs a graph whose edge list is in host memory (c2, c3, c4, tiny)")
        weights = W.csr_edge_weights(src, dst, seed=12)
        tables = gv.gv_build_walk_tables(offsets, weights)[1:]
        args.no_cpu_baseline = True  # the CPU leg is the one of the unweighted graph

    ctx = gv.gv_create(dim=dim, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=total,
                       seed=W.configs.TRAIN_SEED, pool_capacity=P, coherence=args.coherence, schedule=args.schedule,
                       profile=1, pool_slots=RING)
    online = {}
    try:
        if weights is not None:
            gv.gv_set_weighted_graph(ctx, offsets, adj, weights)  # also uploads adjacency and walk tables
        else:
            gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 1)

        def produce(out, seed, first_walk):  # one pool from the host producer of this graph
            if tables is not None:
                gv.gv_augment_weighted(offsets, adj, tables, seed=seed, first_walk=first_walk, count=P, threads=threads, out=out)
            else:
                gv.gv_augment(offsets, adj, seed=seed, first_walk=first_walk, count=P, threads=threads, out=out)

        # Fill the ring once: RING distinct pools, written by the producer straight into the pinned slots.
        t0 = time.perf_counter()
        dev_pools = []
        for r in range(RING):
            slot = gv.gv_acquire_pool_slot(ctx, P)
            if adj is None:
                np.copyto(slot, W.marginal_pool(deg, P, seed=100 * cfg["number"] + r))
            else:
                produce(slot, 100 * cfg["number"], r * walks_per_pool)
            dev_pools.append(torch.from_numpy(slot.view(np.int32)).cuda())
            gv.gv_push_pool(ctx, slot, P)
            gv.gv_train_pool(ctx)  # the first RING steps double as warm-up of the streamed path
            log(f"pool {r + 1}/{RING} ({time.perf_counter() - t0:.1f} s)")
        gv.gv_sync(ctx)
        torch.cuda.synchronize()

        def streamed_steps(count):
            for _ in range(count):
                slot = gv.gv_acquire_pool_slot(ctx, P)  # next slot of the ring, still holding its pool
                gv.gv_push_pool(ctx, slot, P)           # copy host -> device on the copy stream
                gv.gv_train_pool(ctx)                   # launch; waits on the device for that copy only

        position = [0]

        def resident_steps(count):
            for _ in range(count):
                gv.gv_train_device_pool(ctx, dev_pools[position[0] % RING].data_ptr(), P)
                position[0] += 1

        streamed_steps(args.warmup)
        streamed_reps = timed_legs(gv, ctx, streamed_steps, args.steps)
        resident_steps(args.warmup)
        resident_reps = timed_legs(gv, ctx, resident_steps, args.steps)
        s_med, s_sum = summarise(streamed_reps, args.steps, P)
        r_med, r_sum = summarise(resident_reps, args.steps, P)
        h2d_GBps = s_med["h2d_bytes"] / max(s_med["h2d_ms"], 1e-9) / 1e6
        s_sum.update({"h2d_GBps": h2d_GBps, "ring": RING, "exposed_copy_ms_per_step":
                      s_med["wall_s"] / args.steps * 1e3 - s_med["kernel_ms"]})
        stats = gv.gv_get_stats(ctx)
        tiled = stats["tiled_launches"] > 0
        gap = 1.0 - s_sum["samples_per_s_median"] / r_sum["samples_per_s_median"]
        streamed_is_headline = gap <= 0.02
        head, head_sum = (s_med, s_sum) if streamed_is_headline else (r_med, r_sum)
        log(f"streamed: {s_sum['samples_per_s_median']:.4g} samples/s (kernel {s_med['kernel_ms']:.3f} ms/launch, "
            f"H2D {h2d_GBps:.1f} GB/s); resident: {r_sum['samples_per_s_median']:.4g} samples/s "
            f"(kernel {r_med['kernel_ms']:.3f} ms/launch); gap {gap * 100:.2f} %")

        if not args.no_online:
            # Online pipeline (Sec. 3.3): the host producer (parallel online augmentation with pseudo shuffle,
            # Sec. 3.1) fills one pinned slot while the GPU trains the others.
            steps = max(8, args.steps // 2)
            first = RING * walks_per_pool
            gv.gv_sync(ctx)
            t0 = time.perf_counter()
            slot = gv.gv_acquire_pool_slot(ctx, P)
            produce(slot, 900, first)
            produce_s = time.perf_counter() - t0
            gv.gv_push_pool(ctx, slot, P)
            t0 = time.perf_counter()
            for i in range(steps):
                gv.gv_train_pool(ctx)
                if i + 1 < steps:
                    slot = gv.gv_acquire_pool_slot(ctx, P)
                    produce(slot, 900, first + (i + 1) * walks_per_pool)
                    gv.gv_push_pool(ctx, slot, P)
            gv.gv_sync(ctx)
            wall_o = time.perf_counter() - t0
            online["host_producer"] = {"value": steps * P / wall_o, "unit": "positive samples/s", "steps": steps,
                                       "host_threads": threads, "producer_alone": P / produce_s,
                                       "note": "pools generated on the fly by gv_augment into the pinned slots while the GPU trains the others"}
            log(f"online, host producer: {online['host_producer']['value']:.4g} samples/s end to end, producer alone "
                f"{P / produce_s:.4g} samples/s on {threads} threads")
            # The same pipeline with the producer on the device (gv_augment_device): pool k+1 is written
            # into the buffer that pool k-1 was trained from; producer and trainer share one stream.
            if weights is None:
                gv.gv_set_adjacency(ctx, offsets, adj)
            bufs = dev_pools[:2]
            t0 = time.perf_counter()
            for i in range(8):
                gv.gv_augment_device(ctx, bufs[i % 2].data_ptr(), seed=901, first_walk=i * walks_per_pool, count=P)
            gv.gv_sync(ctx)
            produce_d = (time.perf_counter() - t0) / 8
            steps = args.steps
            t0 = time.perf_counter()
            for i in range(steps):
                gv.gv_augment_device(ctx, bufs[i % 2].data_ptr(), seed=902, first_walk=i * walks_per_pool, count=P)
                gv.gv_train_device_pool(ctx, bufs[i % 2].data_ptr(), P)
            gv.gv_sync(ctx)
            wall_d = time.perf_counter() - t0
            online["device_producer"] = {"value": steps * P / wall_d, "unit": "positive samples/s", "steps": steps,
                                         "producer_alone": P / produce_d,
                                         "note": "pools generated on the GPU by gv_augment_device, then trained; "
                                                 "nothing crosses PCIe"}
            log(f"online, device producer: {online['device_producer']['value']:.4g} samples/s end to end, producer "
                f"alone {P / produce_d:.4g} samples/s")
    finally:
        gv.gv_destroy(ctx)

    blocked = None
    if args.blocked_partitions and adj is not None:
        # Orthogonal blocks (Sec. 3.2, Alg. 3) on one GPU: an episode of several pools is redistributed into the
        # B x B grid on the host (not timed, like pool production), then trained block after block; a launch
        # touches one vertex partition and one context partition only.
        B, E = args.blocked_partitions, args.episode_pools
        ctx = gv.gv_create(dim=dim, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=total,
                           seed=W.configs.TRAIN_SEED, pool_capacity=8, coherence=args.coherence, schedule=args.schedule,
                           profile=1, partitions=B)
        try:
            gv.gv_set_degrees(ctx, deg)
            gv.gv_build_alias(ctx, 0.75)
            gv.gv_init_embeddings(ctx, 1)
            part = gv.gv_get_partitions(ctx, n, B)[0]
            t0 = time.perf_counter()
            episode = np.empty((E * P, 2), dtype=np.uint32)
            for r in range(E):
                gv.gv_augment(offsets, adj, seed=100 * cfg["number"], first_walk=r * walks_per_pool, count=P,
                              threads=threads, out=episode[r * P:(r + 1) * P])
            sorted_pairs, order, block_offsets = gv.gv_redistribute_pool(part, B, episode, threads=threads)
            log(f"episode of {E} pools produced and redistributed into {B}x{B} blocks ({time.perf_counter() - t0:.1f} s)")
            del episode
            dev_pairs = torch.from_numpy(sorted_pairs.view(np.int32)).cuda()
            dev_order = torch.from_numpy(order.view(np.int32)).cuda()
            torch.cuda.synchronize()

            def episode_steps(count):
                for _ in range(count):
                    gv.gv_train_device_blocks(ctx, dev_pairs.data_ptr(), dev_order.data_ptr(), block_offsets, E * P)

            episode_steps(1)
            reps = timed_legs(gv, ctx, episode_steps, max(1, args.steps // E))
            episodes = max(1, args.steps // E)
            walls = sorted(r["wall_s"] for r in reps)
            sizes = np.diff(block_offsets.astype(np.int64))
            blocked = {"partitions": B, "episode_samples": E * P, "launches_per_episode": int((sizes > 0).sum()),
                       "samples_per_s_median": episodes * E * P / walls[len(walls) // 2],
                       "samples_per_s_best": episodes * E * P / walls[0],
                       "kernel_ms_per_launch": [r["kernel_ms"] for r in reps],
                       "block_samples_min_max": [int(sizes.min()), int(sizes.max())],
                       "warm_rows": gv.gv_get_stats(ctx)["warm_rows"],
                       "note": "negatives restricted to the context partition of the block; redistribution on the host, "
                               "outside the timed region"}
            log(f"orthogonal blocks {B}x{B}, episode {E} pools: {blocked['samples_per_s_median']:.4g} samples/s")
            del dev_pairs, dev_order
        finally:
            gv.gv_destroy(ctx)

    if args.calibrate_copy:
        src_t = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst_t = torch.empty_like(src_t)
        for _ in range(3):
            dst_t.copy_(src_t)
        torch.cuda.synchronize()
        log("calibration: 3 device copies of 1 GiB done")
        del src_t, dst_t

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(offsets, adj, deg, cfg, W.configs.TRAIN_SEED, args.cpu_samples, args.cpu_samples // 4)
        log(f"cpu oracle: {cpu['value']:.4g} samples/s on one core, {cpu['all_cores']['value']:.4g} on "
            f"{cpu['all_cores']['cores']} cores")

    bytes_per_sample = algorithmic_bytes_per_sample(dim, K)
    achieved = bytes_per_sample * P / (head["kernel_ms"] * 1e-3) / 1e9
    traffic, traffic_source = profiled_traffic(args.workload, SCHEDULES[args.schedule], COHERENCES[args.coherence])
    pools_text = "endpoints from the degree marginal" if adj is None else \
        f"walks L={L}, s={s}, pseudo-shuffled, written by the library's producer"
    out = {
        "metric": "positive edge samples/sec (d=128,K=1) + achieved HBM GB/s fraction, 1 MI355X"
                  if args.workload == "c2" else f"positive edge samples/sec (d={dim},K={K}), 1 MI355X",
        "value": head_sum["samples_per_s_median"], "unit": "positive samples/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": head["wall_s"] / args.steps * 1e3, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg['graph']} n={n} edges={edges}, d={dim}, K={K}, "
                               f"neg_weight={w}, " + ("edge weights from {1/4, 1, 4, 9}, " if args.weighted else "")
                               + f"pools of 2^{int(np.log2(P))} samples "
                               + (f"streamed from {RING} pinned pools (host -> device copy overlapped with training)"
                                  if streamed_is_headline else
                                  f"resident in HBM ({RING} distinct pools cycled; the streamed rate is {gap * 100:.1f} % lower, "
                                  "see `streamed`)")
                               + f", {pools_text}, asynchronous mode",
                   "coherence": COHERENCES[args.coherence], "schedule": SCHEDULES[args.schedule],
                   "kernel": "k_train_tiled" if tiled else "k_train_hogwild", "warm_rows": stats["warm_rows"],
                   "samples_per_step": P, "repetitions": REPETITIONS, "value_is": "median of the repetitions"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "k_train_tiled" if tiled else "k_train_hogwild", "kernel_ms": head["kernel_ms"],
                     "bytes_per_sample": bytes_per_sample},
        "cpu_baseline": cpu,
        "streamed": s_sum,
        "resident": r_sum,
        "online": online or None,
        "blocked": blocked,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
