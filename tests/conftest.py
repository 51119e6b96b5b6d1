import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def tiny_graph():
    """Configuration 1: Barabasi-Albert, 10^4 nodes, m=5."""
    import workloads as W

    n, src, dst = W.make_graph("tiny", cache=False)
    deg = W.degrees(n, src, dst)
    offsets, adj = W.csr_from_edges(n, src, dst)
    return dict(n=n, src=src, dst=dst, deg=deg, offsets=offsets, adj=adj)


@pytest.fixture(scope="session")
def tiny_alias(tiny_graph):
    import oracle

    return oracle.alias_build(oracle.degree_weights(tiny_graph["deg"]))
