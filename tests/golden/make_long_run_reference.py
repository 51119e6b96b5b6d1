"""Writes tests/golden/long_run_<name>.txt: the sequential CPU oracle's trajectory over a long
training run (Sec. 4.3 hyper-parameters: d = 128, one negative of weight 5, walks of length 40
augmented with window 5, learning rate decaying linearly to zero), against which the GPU tests
compare the library's asynchronous training.

Everything here is computed by ``oracle/`` from seeded synthetic inputs; the library under test
is not involved.  One core; about 20 minutes for c2 (32 pools on the 10^6-node power-law graph), 10 minutes for
c3 (4 pools of the same graph with d = 512 and 5 negatives of weight 1),
about an hour and a half for c4 (the full 4*10^9 samples of the planted-partition configuration;
checkpoints are written as they are reached, and the test uses those that exist):

    python tests/golden/make_long_run_reference.py c2
    python tests/golden/make_long_run_reference.py c3
    python tests/golden/make_long_run_reference.py c4
    python tests/golden/make_long_run_reference.py c2-blocks     (c2 under the orthogonal-block schedule, 25 minutes)

A second argument replaces the training seed (the key of the negative-sampling stream) and writes
long_run_<name>_seed<seed>.txt: the same run with other negatives.  How far two such runs of the
oracle lie apart is the scale against which the asynchronous trainer's distance is read:

    python tests/golden/make_long_run_reference.py c2 4321
    python tests/golden/make_long_run_reference.py c3 4321
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
import workloads as W  # noqa: E402

# the tests read these from the files, so the two cannot drift apart
SETUPS = {
    "c2": dict(graph="c2", holdout=0.01, holdout_seed=51, pool=1 << 24, pools=32, dim=128, num_neg=1,
               neg_weight=5.0, lr0=0.025, train_seed=1234, init_seed=1, walk_seed=500, eval_walk_seed=777,
               eval_count=1 << 18, eval_seed=99, negative_pair_seed=52, walk_length=40, window=5),
    "c3": dict(graph="c3", holdout=0.01, holdout_seed=51, pool=1 << 24, pools=4, dim=512, num_neg=5,
               neg_weight=1.0, lr0=0.025, train_seed=1234, init_seed=1, walk_seed=500, eval_walk_seed=777,
               eval_count=1 << 18, eval_seed=99, negative_pair_seed=52, walk_length=40, window=5),
    "c4": dict(graph="c4", holdout=0.01, holdout_seed=61, pool=1 << 24, pools=238, dim=128, num_neg=1,
               neg_weight=5.0, lr0=0.025, train_seed=1234, init_seed=1, walk_seed=600, eval_walk_seed=778,
               eval_count=1 << 18, eval_seed=99, negative_pair_seed=62, walk_length=40, window=5),
}
# c2 under the orthogonal-block schedule of Sec. 3.2: 8 partitions, episodes of 8 pools (2^27 samples) that are
# redistributed into the 8 x 8 grid and trained block after block with negatives restricted to the block's
# context partition; same graph, pools, seeds and learning-rate schedule as c2, so the two files differ by the
# schedule alone
SETUPS["c2-blocks"] = dict(SETUPS["c2"], partitions=8, episode_pools=8)
CHECKPOINTS = {"c2": (1, 2, 4, 8, 16, 24, 32), "c3": (1, 2, 3, 4), "c4": (4, 16, 32, 64, 96, 128, 160, 192, 238),
               "c2-blocks": (8, 16, 24, 32)}


def pool_of(offsets, adj, seed, first_walk, count, s):
    pairs, _ = oracle.augment(seed, offsets, adj, s["walk_length"], s["window"], count, first_walk=first_walk)
    return oracle.pseudo_shuffle(pairs, s["window"])


def main():
    name = sys.argv[1] if len(sys.argv) > 1 else "c2"
    s = dict(SETUPS[name])
    out_path = os.path.join(HERE, f"long_run_{name}.txt")
    if len(sys.argv) > 2:
        s["train_seed"] = int(sys.argv[2])
        out_path = os.path.join(HERE, f"long_run_{name}_seed{s['train_seed']}.txt")
    n, src, dst = W.make_graph(s["graph"])
    tr_s, tr_d, te_s, te_d = W.split_holdout(src, dst, s["holdout"], seed=s["holdout_seed"])
    deg = W.degrees(n, tr_s, tr_d)
    offsets, adj = W.csr_from_edges(n, tr_s, tr_d)
    P, pools = s["pool"], s["pools"]
    per_walk = sum(min(s["window"], s["walk_length"] - i) for i in range(s["walk_length"]))
    walks_per_pool = -(-P // per_walk)
    eval_pool = pool_of(offsets, adj, s["eval_walk_seed"], 0, s["eval_count"], s)
    na, nb = W.uniform_negative_pairs(n, te_s.size, seed=s["negative_pair_seed"])
    thresh, alias = oracle.alias_build(oracle.degree_weights(deg))
    B, E = s.get("partitions", 0), s.get("episode_pools", 1)
    if B:
        part = oracle.zigzag_partition(deg, B)
        tables = oracle.partition_alias(deg, B, part)
    vertex, context = oracle.init_embeddings(s["init_seed"], n, s["dim"])
    lines = [f"# written by tests/golden/make_long_run_reference.py {name} (CPU oracle only)"]
    lines += [f"# {k} = {v}" for k, v in s.items()]
    lines.append("# pools_trained eval_loss link_prediction_auc max_vertex_norm max_context_norm")
    with open(out_path, "w") as f:
        f.write("\n".join(lines) + "\n")
    for k in range(E - 1, pools, E):  # k = last pool of the step: one pool, or one episode of E pools
        t0 = time.time()
        first = k + 1 - E
        pool = np.concatenate([pool_of(offsets, adj, s["walk_seed"], r * walks_per_pool, P, s) for r in range(first, k + 1)])
        kw = dict(K=s["num_neg"], first_g=first * P, T=P * pools, lr0=s["lr0"], lr_min_ratio=0.0, w=s["neg_weight"],
                  seed=s["train_seed"])
        if B:
            oracle.train_blocked(vertex, context, pool, B=B, part=part, tables=tables, **kw)
        else:
            oracle.train(vertex, context, pool, thresh=thresh, alias=alias, **kw)
        print(f"pool {k + 1}/{pools}: {time.time() - t0:.0f} s", flush=True)
        if k + 1 in CHECKPOINTS[name]:
            loss = oracle.loss(vertex, context, eval_pool, K=s["num_neg"], w=s["neg_weight"], seed=s["eval_seed"],
                               thresh=thresh, alias=alias)
            auc = oracle.link_prediction_auc(vertex, te_s, te_d, na, nb)
            lines.append(f"{k + 1} {loss:.6f} {auc:.6f} {np.linalg.norm(vertex, axis=1).max():.3f} "
                         f"{np.linalg.norm(context, axis=1).max():.3f}")
            print(lines[-1], f"({time.time() - t0:.0f} s for this pool)", flush=True)
            with open(out_path, "a") as f:
                f.write(lines[-1] + "\n")


if __name__ == "__main__":
    main()
