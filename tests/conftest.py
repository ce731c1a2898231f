import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


def random_csr(n, avg_deg, rng, symmetric=True, allow_loops=False):
    """Small seeded random {0,1} adjacency in CSR (int64 rowptr, int32 col, rows sorted, unique)."""
    m = int(n * avg_deg / (2 if symmetric else 1))
    src = rng.integers(0, n, size=m)
    # skewed destinations so that some rows are long and some empty
    dst = np.minimum((rng.random(m) ** 2.5 * n).astype(np.int64), n - 1)
    if symmetric:
        src, dst = np.concatenate([src, dst]), np.concatenate([dst, src])
    if not allow_loops:
        keep = src != dst
        src, dst = src[keep], dst[keep]
    key = np.unique(src * n + dst)
    src, dst = key // n, key % n
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, src + 1, 1)
    rowptr = np.cumsum(rowptr)
    return rowptr, dst.astype(np.int32)


def skewed_csr(n, m, rng):
    """Directed graph whose edge endpoints follow a power law (hubs on both sides), rows sorted and unique."""
    src = (n * rng.random(m) ** 3).astype(np.int64)
    dst = (n * rng.random(m) ** 2).astype(np.int64)
    perm = rng.permutation(n)
    key = np.unique(perm[src] * n + perm[dst])
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, key // n + 1, 1)
    return np.cumsum(rowptr), (key % n).astype(np.int32)


def random_batches(n, k, b, rng, candidates=None):
    """k x b int32, distinct inside each minibatch."""
    pool = np.arange(n) if candidates is None else np.asarray(candidates)
    return np.stack([rng.choice(pool, size=b, replace=False) for _ in range(k)]).astype(np.int32)


@pytest.fixture
def rng():
    return np.random.default_rng(12345)
