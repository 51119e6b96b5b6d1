#!/usr/bin/env python3
"""Benchmark of the training hot path on one MI355X.

A step = one pool of 2^24 positive samples of configuration 2 (Chung-Lu graph,
10^6 nodes / 5*10^6 edges, d = 128, K = 1) through the whole path: sample read,
negative draw, row gathers, dot products, sigmoid-gradient, in-place updates.
Pools are resident in HBM before the timed region; the streamed (PCIe-inclusive)
rate is measured separately and reported beside it.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch from rocprofv3 FETCH_SIZE / WRITE_SIZE counters, scaled by what the same counters
# read for a 1 GiB device copy (profiles/k_train_tiled_*.md); only for the profiled setups.
PROFILED_TRAFFIC_BYTES = {("c2", 1, 3): 50.45e9, ("c3", 1, 3): 463.4e9, ("c4", 1, 3): 56.11e9}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes_per_sample(dim: int, num_neg: int) -> int:
    """Each of the 2+K rows is read once and written once (4d bytes each way), plus the
    8-byte sample and one 8-byte alias entry per negative."""
    return 2 * (2 + num_neg) * 4 * dim + 8 + 8 * num_neg


def cpu_baseline(n, deg, pool, dim, num_neg, w, total, seed, budget_samples):
    """The sequential oracle, as it stands, on a bounded slice of the same workload."""
    import oracle

    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    vertex, context = oracle.init_embeddings(1, n, dim)
    part = pool[:budget_samples]
    t0 = time.perf_counter()
    oracle.train(vertex, context, part, K=num_neg, first_g=0, T=total, lr0=0.025, lr_min_ratio=0.0, w=w,
                 seed=seed, thresh=thresh, alias=alias)
    dt = time.perf_counter() - t0
    return {"value": part.shape[0] / dt, "unit": "positive samples/s", "cores": 1, "kind": "oracle",
            "sample": f"first {part.shape[0]} samples of one {pool.shape[0]}-sample pool of the same workload, "
                      f"sequential C oracle (fp64 arithmetic), {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=4)
    ap.add_argument("--workload", default="c2", choices=["c2", "c3", "c4", "tiny", "c5-marginal"])
    ap.add_argument("--pools", type=int, default=8, help="distinct pre-generated pools cycled through")
    ap.add_argument("--coherence", type=int, default=int(os.environ.get("GV_BENCH_COHERENCE", "3")))
    ap.add_argument("--schedule", type=int, default=int(os.environ.get("GV_BENCH_SCHEDULE", "1")))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-streamed", action="store_true")
    ap.add_argument("--cpu-samples", type=int, default=1 << 24)
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

    t0 = time.perf_counter()
    if cfg["graph"] == "expected_degrees":
        # too large to walk inside a benchmark run: degrees from the model, endpoints from their marginal
        n, deg = W.expected_degrees(args.workload)
        offsets = adj = None
        edges = cfg["edges"]
        args.no_streamed = True
        log(f"degrees {args.workload}: n={n} ({time.perf_counter() - t0:.1f} s)")
        t0 = time.perf_counter()
        pools = []
        for r in range(args.pools):  # one progress line per pool: these take a while at 6.6*10^7 nodes
            pools.append(W.marginal_pool(deg, P, seed=100 * cfg["number"] + r))
            log(f"pool {r + 1}/{args.pools} ({time.perf_counter() - t0:.1f} s)")
    else:
        n, src, dst = W.make_graph(args.workload)
        deg = W.degrees(n, src, dst)
        offsets, adj = W.csr_from_edges(n, src, dst)
        edges = src.size
        log(f"graph {args.workload}: n={n} edges={edges} ({time.perf_counter() - t0:.1f} s)")
        t0 = time.perf_counter()
        pools = [W.walk_pool(offsets, adj, P, W.configs.WALK_LENGTH, W.configs.WINDOW, seed=100 * cfg["number"] + r)
                 for r in range(args.pools)]
    log(f"{args.pools} pools of {P} samples ({time.perf_counter() - t0:.1f} s)")
    dev_pools = [torch.from_numpy(p.view(np.int32)).cuda() for p in pools]
    torch.cuda.synchronize()

    ctx = gv.gv_create(dim=dim, num_neg=K, neg_weight=w, mode=gv.GV_MODE_HOGWILD, total_samples=total,
                       seed=W.configs.TRAIN_SEED, pool_capacity=P, coherence=args.coherence, schedule=args.schedule,
                       profile=1)
    try:
        gv.gv_set_degrees(ctx, deg)
        gv.gv_build_alias(ctx, 0.75)
        gv.gv_init_embeddings(ctx, 1)

        def step(i):
            t = dev_pools[i % len(dev_pools)]
            gv.gv_train_device_pool(ctx, t.data_ptr(), P)

        for i in range(args.warmup):
            step(i)
        gv.gv_sync(ctx)
        before = gv.gv_get_stats(ctx)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        gv.gv_sync(ctx)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        after = gv.gv_get_stats(ctx)
        launches = after["timed_launches"] - before["timed_launches"]
        kernel_ms = (after["train_kernel_ms"] - before["train_kernel_ms"]) / max(launches, 1)
        value = args.steps * P / wall
        bytes_per_sample = algorithmic_bytes_per_sample(dim, K)
        achieved = bytes_per_sample * P / (kernel_ms * 1e-3) / 1e9
        log(f"resident: {value:.4g} samples/s, train kernel {kernel_ms:.3f} ms/launch, {achieved:.0f} GB/s algorithmic")

        streamed = None
        if not args.no_streamed:
            # PCIe-inclusive path: the producer fills the library's pinned slot in place,
            # the copy of pool k+1 overlaps training of pool k.
            steps = max(4, args.steps // 2)
            slot = gv.gv_acquire_pool_slot(ctx, P)
            np.copyto(slot, pools[0])
            gv.gv_push_pool(ctx, slot, P)
            gv.gv_sync(ctx)
            s0 = gv.gv_get_stats(ctx)
            t0 = time.perf_counter()
            for i in range(steps):
                gv.gv_train_pool(ctx)
                if i + 1 < steps:
                    slot = gv.gv_acquire_pool_slot(ctx, P)
                    np.copyto(slot, pools[(i + 1) % len(pools)])
                    gv.gv_push_pool(ctx, slot, P)
            gv.gv_sync(ctx)
            wall_s = time.perf_counter() - t0
            s1 = gv.gv_get_stats(ctx)
            streamed = {"value": steps * P / wall_s, "unit": "positive samples/s", "steps": steps,
                        "h2d_GBps": (s1["h2d_bytes"] - s0["h2d_bytes"]) / max(s1["h2d_ms"] - s0["h2d_ms"], 1e-9) / 1e6,
                        "note": "pools filled into the pinned slot by one host thread (numpy copy) and copied "
                                "host-to-device while the previous pool trains"}
            log(f"streamed: {streamed['value']:.4g} samples/s")
            # Online pipeline (Sec. 3.3): the host producer (parallel online augmentation with
            # pseudo shuffle, Sec. 3.1) fills one pinned slot while the GPU trains the other.
            threads = min(16, os.cpu_count() or 1)
            walks_per_pool = -(-P // 190)
            slot = gv.gv_acquire_pool_slot(ctx, P)
            t0 = time.perf_counter()
            gv.gv_augment(offsets, adj, seed=900, first_walk=0, count=P, threads=threads, out=slot)
            produce_s = time.perf_counter() - t0
            gv.gv_push_pool(ctx, slot, P)
            gv.gv_sync(ctx)
            steps = max(3, args.steps // 8)
            t0 = time.perf_counter()
            for i in range(steps):
                gv.gv_train_pool(ctx)
                if i + 1 < steps:
                    slot = gv.gv_acquire_pool_slot(ctx, P)
                    gv.gv_augment(offsets, adj, seed=900, first_walk=(i + 1) * walks_per_pool, count=P,
                                  threads=threads, out=slot)
                    gv.gv_push_pool(ctx, slot, P)
            gv.gv_sync(ctx)
            wall_o = time.perf_counter() - t0
            streamed["online"] = {"value": steps * P / wall_o, "unit": "positive samples/s", "steps": steps,
                                  "host_threads": threads, "producer_alone": P / produce_s,
                                  "note": "pools generated on the fly by gv_augment into the pinned slots; "
                                          "host-bound"}
            log(f"online: {streamed['online']['value']:.4g} samples/s end to end, producer alone "
                f"{P / produce_s:.4g} samples/s on {threads} threads")
            # The same pipeline with the producer on the device (gv_augment_device): pool k+1 is written
            # into the buffer that pool k-1 was trained from; producer and trainer share one stream.
            gv.gv_set_adjacency(ctx, offsets, adj)
            bufs = [torch.empty((P, 2), dtype=torch.int32, device="cuda") for _ in range(2)]
            for i in range(2):
                gv.gv_augment_device(ctx, bufs[i].data_ptr(), seed=901, first_walk=i * walks_per_pool, count=P)
            gv.gv_sync(ctx)
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
            streamed["online_device"] = {"value": steps * P / wall_d, "unit": "positive samples/s", "steps": steps,
                                         "producer_alone": P / produce_d,
                                         "note": "pools generated on the GPU by gv_augment_device, then trained; "
                                                 "nothing crosses PCIe"}
            log(f"online on the device: {streamed['online_device']['value']:.4g} samples/s end to end, producer "
                f"alone {P / produce_d:.4g} samples/s")
            del bufs
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
        cpu = cpu_baseline(n, deg, pools[0], dim, K, w, total, W.configs.TRAIN_SEED, args.cpu_samples)
        log(f"cpu oracle: {cpu['value']:.4g} samples/s")

    out = {
        "metric": "positive edge samples/sec (d=128,K=1) + achieved HBM GB/s fraction, 1 MI355X"
                  if args.workload == "c2" else f"positive edge samples/sec (d={dim},K={K}), 1 MI355X",
        "value": value, "unit": "positive samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {cfg['graph']} n={n} edges={edges}, d={dim}, K={K}, "
                               f"neg_weight={w}, pool=2^{int(np.log2(P))} samples resident in HBM, "
                               f"{args.pools} distinct pools cycled ("
                               + ("endpoints from the degree marginal" if adj is None else "walks L=40, s=5")
                               + "), asynchronous mode",
                   "coherence": ["plain", "agent", "atomic-agent", "mixed"][args.coherence],
                   "schedule": ["pool-order", "tiled"][args.schedule], "samples_per_step": P},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": PROFILED_TRAFFIC_BYTES.get((args.workload, args.schedule, args.coherence)),
                     "kernel": "k_train_tiled" if args.schedule else "k_train_hogwild", "kernel_ms": kernel_ms,
                     "bytes_per_sample": bytes_per_sample},
        "cpu_baseline": cpu,
        "streamed": streamed,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
