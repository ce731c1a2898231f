"""Pins of the oracle's forward aggregation (Sec. 6.2: SpMM of a minibatch's sampled adjacency and its feature rows)."""
import numpy as np
import pytest

from conftest import random_batches, random_csr
from oracle import bms_oracle as O


def _sample(seed=1, k=3, b=12, fanouts=(4, 3)):
    rng = np.random.default_rng(seed)
    rowptr, col = random_csr(400, 7.0, rng)
    batches = random_batches(400, k, b, rng)
    return rng, O.sample_nodewise(rowptr, col, batches, fanouts, 11)


def _dense_blocks(hop):
    """Per minibatch the dense 0/1 matrix A_i (rows of the minibatch x its own columns)."""
    for i in range(len(hop.mb_rowoff) - 1):
        r0, r1 = hop.mb_rowoff[i], hop.mb_rowoff[i + 1]
        c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
        A = np.zeros((r1 - r0, c1 - c0))
        for r in range(r0, r1):
            A[r - r0, hop.col[hop.rowptr[r]:hop.rowptr[r + 1]]] = 1.0
        yield (r0, r1, c0, c1, A)


@pytest.mark.parametrize("mean", [True, False])
def test_equals_the_dense_product_per_minibatch(mean):
    rng, hops = _sample()
    for hop in hops:
        X = rng.standard_normal((hop.ncols, 6)).astype(np.float32)
        out = O.aggregate(hop, X, mean=mean)
        for r0, r1, c0, c1, A in _dense_blocks(hop):
            ref = A @ X[c0:c1].astype(np.float64)
            if mean:
                ref = ref / np.maximum(A.sum(axis=1, keepdims=True), 1.0)
            assert np.allclose(out[r0:r1], ref, rtol=0, atol=1e-6 * np.abs(X).max() * A.sum(axis=1).max())
            assert np.array_equal(out[r0:r1], ref.astype(np.float32))  # one rounding, of the double result


def test_closed_forms():
    rng, hops = _sample(seed=2)
    hop = hops[0]
    lens = np.diff(hop.rowptr)
    ones = np.ones((hop.ncols, 3), dtype=np.float32)
    assert np.array_equal(O.aggregate(hop, ones, mean=False), np.repeat(lens[:, None], 3, axis=1).astype(np.float32))
    assert np.array_equal(O.aggregate(hop, ones, mean=True), np.repeat((lens > 0)[:, None], 3, axis=1).astype(np.float32))
    # X = identity-like block: column j of minibatch i is a one-hot -> the output row is the row's pattern
    i = 1
    c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
    X = np.zeros((hop.ncols, c1 - c0), dtype=np.float32)
    X[np.arange(c0, c1), np.arange(c1 - c0)] = 1.0
    out = O.aggregate(hop, X, mean=False)
    for r in range(hop.mb_rowoff[i], hop.mb_rowoff[i + 1]):
        pattern = np.zeros(c1 - c0, dtype=np.float32)
        pattern[hop.col[hop.rowptr[r]:hop.rowptr[r + 1]]] = 1.0
        assert np.array_equal(out[r], pattern)
    # rows of other minibatches never see this block
    other = np.ones(hop.rows, dtype=bool)
    other[hop.mb_rowoff[i]:hop.mb_rowoff[i + 1]] = False
    assert not out[other].any()


def test_rows_without_neighbours_and_linearity():
    rowptr = np.array([0, 0, 2, 2, 3], dtype=np.int64)  # vertices 0 and 2 have no out-edges
    col = np.array([0, 3, 1], dtype=np.int32)
    hop = O.sample_nodewise(rowptr, col, np.array([[0, 1, 2, 3]], dtype=np.int32), (5,), 1)[0]
    X = np.array([[1.0, 2.0], [10.0, 20.0], [100.0, 200.0]], dtype=np.float32)  # columns {0, 1, 3}
    assert hop.col_vertex.tolist() == [0, 1, 3]
    assert O.aggregate(hop, X, mean=True).tolist() == [[0, 0], [50.5, 101.0], [0, 0], [10.0, 20.0]]
    assert O.aggregate(hop, X, mean=False).tolist() == [[0, 0], [101.0, 202.0], [0, 0], [10.0, 20.0]]
    rng, hops = _sample(seed=3)
    h = hops[1]
    Xa = rng.integers(-50, 50, size=(h.ncols, 4)).astype(np.float32)
    Xb = rng.integers(-50, 50, size=(h.ncols, 4)).astype(np.float32)
    assert np.array_equal(O.aggregate(h, Xa + Xb, mean=False), O.aggregate(h, Xa, mean=False) + O.aggregate(h, Xb, mean=False))
