import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


_config = None


def pytest_configure(config):
    global _config
    _config = config
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_runtest_logfinish(nodeid, location):
    """The progress mark of every finished test leaves the process at once, also when the output is a pipe or a
    file (a long run then shows that it is alive)."""
    reporter = _config.pluginmanager.get_plugin("terminalreporter") if _config else None
    writer = getattr(reporter, "_tw", None)
    for stream in (getattr(writer, "_file", None), sys.stdout, sys.stderr):
        try:
            if stream is not None:
                stream.flush()
        except (OSError, ValueError):
            pass


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
