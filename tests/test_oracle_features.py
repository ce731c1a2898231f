"""Pins of the oracle's feature fetching (Sec. 6.2: H_i = the rows of H of a minibatch's last frontier)."""
import numpy as np
import pytest

from oracle import bms_oracle as O


def test_rows_are_the_listed_rows_of_h_in_list_order():
    rng = np.random.default_rng(3)
    H = rng.standard_normal((500, 37)).astype(np.float32)
    ids = rng.integers(0, 500, size=2000).astype(np.int32)  # repeats allowed: a vertex can serve several minibatches
    out = O.fetch_features(H, ids)
    assert out.dtype == np.float32 and out.shape == (2000, 37)
    # library routine for the same definition: fancy indexing; bit patterns must agree (a fetch is a copy)
    assert np.array_equal(out.view(np.uint32), H[ids].view(np.uint32))


def test_selection_matrix_product_gives_the_same_rows():
    # H_i = Q H with Q the 0/1 selection matrix that has one nonzero per row (the paper's matrix view)
    rng = np.random.default_rng(4)
    H = rng.integers(-8, 8, size=(40, 5)).astype(np.float32)  # small integers: the product is exact in fp32
    ids = rng.permutation(40)[:17].astype(np.int32)
    Q = np.zeros((17, 40), dtype=np.float32)
    Q[np.arange(17), ids] = 1.0
    assert np.array_equal(O.fetch_features(H, ids), Q @ H)


def test_special_values_and_edges():
    H = np.array([[0.0, -0.0, np.inf], [np.nan, 1e-45, -np.inf]], dtype=np.float32)
    out = O.fetch_features(H, np.array([1, 0, 1], dtype=np.int32))
    assert np.array_equal(out.view(np.uint32), H[[1, 0, 1]].view(np.uint32))  # NaN payload, signed zero, denormal kept
    assert O.fetch_features(H, np.zeros(0, dtype=np.int32)).shape == (0, 3)
    one = O.fetch_features(np.arange(7, dtype=np.float32).reshape(7, 1), np.array([6, 0], dtype=np.int32))
    assert one.ravel().tolist() == [6.0, 0.0]
    for bad in ([2], [-1], [0, 5]):
        with pytest.raises(ValueError):
            O.fetch_features(H, np.array(bad, dtype=np.int32))


def test_frontier_of_a_sample_is_a_valid_id_list():
    # the ids fed to the fetch are a hop's stacked col_vertex: distinct and ascending inside every minibatch
    from conftest import random_batches, random_csr
    rng = np.random.default_rng(5)
    rowptr, col = random_csr(300, 6.0, rng)
    batches = random_batches(300, 3, 10, rng)
    hop = O.sample_nodewise(rowptr, col, batches, (4, 3), 7)[-1]
    H = rng.standard_normal((300, 8)).astype(np.float32)
    out = O.fetch_features(H, hop.col_vertex)
    for i in range(3):
        c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
        assert np.all(np.diff(hop.col_vertex[c0:c1]) > 0)
        assert np.array_equal(out[c0:c1], H[hop.col_vertex[c0:c1]])
