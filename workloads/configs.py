"""The benchmark configurations as data, and one call that builds their graph."""
from __future__ import annotations

import os
import tempfile

import numpy as np

from . import graphs

# seeds: graph seed = config number, walk seed = 100 + config number, training seed 1234
CONFIGS = {
    "tiny": dict(number=1, graph="barabasi_albert", n=10_000, m_attach=5, dim=128, num_neg=1,
                 neg_weight=5.0, total_samples=2_000_000, pool=2_000_000),
    "c2": dict(number=2, graph="chung_lu", n=1_000_000, edges=5_000_000, gamma=2.1, dim=128, num_neg=1,
               neg_weight=5.0, total_samples=2_000_000_000, pool=1 << 24),
    "c3": dict(number=3, graph="chung_lu", n=1_000_000, edges=5_000_000, gamma=2.1, dim=512, num_neg=5,
               neg_weight=1.0, total_samples=1_000_000_000, pool=1 << 24, graph_seed=2),
    "c4": dict(number=4, graph="planted_partition", n=4_000_000, communities=400, edges=40_000_000,
               ratio=50.0, dim=128, num_neg=1, neg_weight=5.0, total_samples=4_000_000_000, pool=1 << 24),
    # scaled-down stand-in for c4 that the sequential oracle finishes in seconds and that is
    # trained to its plateau (1600 samples per node), so that quality comparisons are stable
    "c4-small": dict(number=4, graph="planted_partition", n=5_000, communities=10, edges=50_000,
                     ratio=50.0, dim=128, num_neg=1, neg_weight=5.0, total_samples=8_000_000, pool=1 << 20),
    # generated on the GPU (device_graphs.chung_lu_csr): far too large for the numpy recipe
    "c5": dict(number=5, graph="chung_lu_on_device", n=66_000_000, edges=1_800_000_000, gamma=2.2, dim=128, num_neg=1,
               neg_weight=5.0, total_samples=10_000_000_000, pool=1 << 24),
}
# configuration 5 without its adjacency: Chung-Lu expected degrees for 6.6*10^7 nodes / 1.8*10^9 edges and pools
# whose endpoints are drawn independently from the degree-proportional marginal (same row-access distribution)
CONFIGS["c5-marginal"] = dict(CONFIGS["c5"], graph="expected_degrees")
WALK_LENGTH = 40
WINDOW = 5
LR0 = 0.025
TRAIN_SEED = 1234


def make_graph(name: str, cache: bool = True):
    """Edge list ``(n, src, dst)`` of a named configuration (cached as .npz in
    the temp directory because the million-node graphs take a while)."""
    cfg = CONFIGS[name]
    if cfg["graph"] in ("chung_lu_on_device", "expected_degrees"):
        raise ValueError(f"{name}: no edge list in host memory; see device_graphs.chung_lu_csr / expected_degrees")
    seed = cfg.get("graph_seed", cfg["number"])
    path = os.path.join(tempfile.gettempdir(), f"gv_workload_{cfg['graph']}_{cfg['n']}_{seed}.npz")
    if cache and os.path.exists(path):
        z = np.load(path)
        return int(cfg["n"]), z["src"], z["dst"]
    if cfg["graph"] == "barabasi_albert":
        src, dst = graphs.barabasi_albert(cfg["n"], cfg["m_attach"], seed)
    elif cfg["graph"] == "chung_lu":
        src, dst = graphs.chung_lu(cfg["n"], cfg["edges"], cfg["gamma"], seed)
    elif cfg["graph"] == "planted_partition":
        src, dst, _ = graphs.planted_partition(cfg["n"], cfg["communities"], cfg["edges"], cfg["ratio"], seed)
    else:
        raise KeyError(cfg["graph"])
    if cache:
        tmp = path + f".{os.getpid()}.tmp.npz"
        np.savez(tmp, src=src, dst=dst)
        os.replace(tmp, path)
    return int(cfg["n"]), src, dst


def expected_degrees(name: str):
    """Degrees of a Chung-Lu configuration without generating its edges: round(2 m w_i / sum w), permuted."""
    cfg = CONFIGS[name]
    n, m, gamma = cfg["n"], cfg["edges"], cfg["gamma"]
    rng = np.random.Generator(np.random.PCG64(cfg["number"]))
    w = np.arange(1, n + 1, dtype=np.float64) ** (-1.0 / (gamma - 1.0))
    deg = np.minimum(np.rint(2.0 * m * w / w.sum()), n - 1).astype(np.uint32)
    return n, deg[rng.permutation(n)]
