import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def random_symmetric_csr(n, avg_deg, rng, hub_boost=0):
    """Small random undirected graph as int64 indptr / int32 indices (rows
    ascending, no self loops, no duplicates).  Optional hubs for skew."""
    m = n * avg_deg // 2
    a = rng.integers(0, n, size=m)
    b = rng.integers(0, n, size=m)
    if hub_boost:
        hubs = rng.integers(0, n, size=max(1, n // 50))
        a[: m // 3] = hubs[rng.integers(0, len(hubs), size=m // 3)]
    keep = a != b
    a, b = a[keep], b[keep]
    key = np.unique(np.minimum(a, b) * n + np.maximum(a, b))
    a, b = key // n, key % n
    row = np.concatenate([a, b])
    col = np.concatenate([b, a])
    order = np.lexsort((col, row))
    row, col = row[order], col[order]
    indptr = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(np.bincount(row, minlength=n), out=indptr[1:])
    return indptr, col.astype(np.int32)


@pytest.fixture(scope="session")
def small_graph():
    rng = np.random.default_rng(7)
    return random_symmetric_csr(400, 12, rng, hub_boost=1)
