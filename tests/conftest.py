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
def tiny():
    """The Tiny workload's host inputs (numpy)."""
    import synth
    w = synth.WORKLOADS["tiny"]
    d = synth.make_inputs(w)
    d["w"] = w
    return d


@pytest.fixture(scope="session")
def small_graphs():
    """A few very small graphs for brute-force checks, as (indptr, indices) pairs."""
    import synth
    out = []
    for n, e, seed in [(40, 300, 11), (97, 1500, 12), (256, 1200, 13)]:
        out.append(synth.rmat_csr(n, e, (0.57, 0.19, 0.19), seed))
    # a hand-made graph with an isolated node, a self loop and a duplicated edge
    indptr = np.array([0, 0, 3, 4, 9, 9], dtype=np.int64)
    indices = np.array([1, 3, 3, 2, 0, 1, 2, 3, 4], dtype=np.int64)
    out.append((indptr, indices))
    return out
