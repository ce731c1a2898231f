"""Pins for the oracle's GraphSAGE path (Sec. 4.1, Alg. 1, Eq. 1) -- no GPU."""
import numpy as np
import pytest

import brute
from conftest import random_batches, random_csr
from oracle import bms_oracle as O


def _check_against_brute(rowptr, col, batches, fanouts, seed, mb_base=0):
    A = brute.dense_adjacency(rowptr, col)
    ref = brute.nodewise(A, batches, fanouts, seed, mb_base)
    hops = O.sample_nodewise(rowptr, col, batches, fanouts, seed, mb_base)
    assert len(hops) == len(fanouts)
    for h, hop in enumerate(hops):
        for i in range(len(batches)):
            F, Adense, kept = ref[i][h]
            r0, r1 = hop.mb_rowoff[i], hop.mb_rowoff[i + 1]
            c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
            assert hop.row_vertex[r0:r1].tolist() == F
            assert hop.col_vertex[c0:c1].tolist() == kept.tolist()
            assert (brute.hop_block_dense(hop, i) == Adense).all()
        assert hop.rows == hop.mb_rowoff[-1] == len(hop.row_vertex) == len(hop.rowptr) - 1
        assert hop.nnz == hop.rowptr[-1] == len(hop.col)
        assert hop.ncols == hop.mb_coloff[-1] == len(hop.col_vertex)
        if h + 1 < len(hops):   # the kept columns are the next hop's rows
            assert (hops[h + 1].row_vertex == hop.col_vertex).all()
            assert (hops[h + 1].mb_rowoff == hop.mb_coloff).all()


@pytest.mark.parametrize("n,avg,k,b,fanouts,seed", [
    (24, 5.0, 3, 4, (2, 2), 1),
    (40, 8.0, 4, 6, (3, 2, 2), 2),
    (64, 12.0, 2, 8, (5, 3), 3),
    (33, 6.0, 5, 1, (1, 1, 1), 4),
    (48, 10.0, 2, 5, (4, 1, 6), 5),
])
def test_matches_dense_brute_force(n, avg, k, b, fanouts, seed):
    rng = np.random.default_rng(seed)
    rowptr, col = random_csr(n, avg, rng)
    batches = random_batches(n, k, b, rng)
    _check_against_brute(rowptr, col, batches, fanouts, 1000 + seed, mb_base=seed)


def test_directed_graph_with_loops_matches_brute_force():
    rng = np.random.default_rng(77)
    rowptr, col = random_csr(36, 7.0, rng, symmetric=False, allow_loops=True)
    batches = random_batches(36, 3, 5, rng)
    _check_against_brute(rowptr, col, batches, (3, 2), 5)


def test_fanout_at_least_max_degree_reproduces_exact_QA():
    # no randomness left: rows are the exact rows of A, frontiers are the BFS-style level sets
    rng = np.random.default_rng(8)
    n = 60
    rowptr, col = random_csr(n, 6.0, rng)
    A = brute.dense_adjacency(rowptr, col)
    maxdeg = int(np.diff(rowptr).max())
    batches = random_batches(n, 3, 4, rng)
    for fan in ((maxdeg, maxdeg, maxdeg), (maxdeg + 5, 2**31 - 1, maxdeg)):
        for seed in (1, 2):   # result must not depend on the seed
            hops = O.sample_nodewise(rowptr, col, batches, fan, seed)
            for i in range(3):
                F = batches[i].tolist()
                for hop in hops:
                    nxt = np.nonzero(A[F].sum(axis=0) > 0)[0]
                    c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
                    assert hop.col_vertex[c0:c1].tolist() == nxt.tolist()
                    assert (brute.hop_block_dense(hop, i) == A[F][:, nxt]).all()
                    F = nxt.tolist()


def test_row_invariants_on_a_skewed_graph():
    # each sampled row has exactly min(deg, s) distinct true neighbours, ascending
    rng = np.random.default_rng(9)
    n = 3000
    rowptr, col = random_csr(n, 30.0, rng)
    deg = np.diff(rowptr)
    batches = random_batches(n, 6, 50, rng)
    fan = (7, 4, 3)
    hops = O.sample_nodewise(rowptr, col, batches, fan, 99)
    for h, hop in enumerate(hops):
        s = fan[h]
        for i in range(6):
            r0, r1 = hop.mb_rowoff[i], hop.mb_rowoff[i + 1]
            cv = hop.col_vertex[hop.mb_coloff[i]:hop.mb_coloff[i + 1]]
            assert (np.diff(cv) > 0).all()
            used = np.zeros(len(cv), dtype=bool)
            for r in range(r0, r1):
                v = hop.row_vertex[r]
                loc = hop.col[hop.rowptr[r]:hop.rowptr[r + 1]]
                assert len(loc) == min(deg[v], s)
                assert (np.diff(loc) > 0).all()
                nb = cv[loc]
                assert np.isin(nb, col[rowptr[v]:rowptr[v + 1]]).all()
                used[loc] = True
            assert used.all()        # no empty column survives
        assert hop.rows <= 6 * 50 * int(np.prod(fan[:h]))   # dimension bound of Sec. 4.1.4


def test_bulk_equals_stack_of_single_minibatch_calls():
    rng = np.random.default_rng(10)
    n = 500
    rowptr, col = random_csr(n, 12.0, rng)
    batches = random_batches(n, 5, 16, rng)
    fan = (4, 3)
    bulk = O.sample_nodewise(rowptr, col, batches, fan, 31, mb_base=10)
    for h in range(2):
        rv, cl, cvx, rows_nnz = [], [], [], []
        for i in range(5):
            one = O.sample_nodewise(rowptr, col, batches[i:i + 1], fan, 31, mb_base=10 + i)[h]
            rv.append(one.row_vertex); cl.append(one.col); cvx.append(one.col_vertex)
            rows_nnz.append(np.diff(one.rowptr))
        assert (np.concatenate(rv) == bulk[h].row_vertex).all()
        assert (np.concatenate(cl) == bulk[h].col).all()
        assert (np.concatenate(cvx) == bulk[h].col_vertex).all()
        assert (np.concatenate(rows_nnz) == np.diff(bulk[h].rowptr)).all()
    # a different minibatch index gives a different sample for the same seeds
    other = O.sample_nodewise(rowptr, col, batches, fan, 31, mb_base=11)
    assert not np.array_equal(other[0].col_vertex, bulk[0].col_vertex)


def test_same_vertex_in_two_minibatches_and_two_hops_draws_independently():
    # star-ish graph: vertex 0 has 40 neighbours; the same seed vertex in two minibatches
    n = 41
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = 40
    rowptr[2:] = 40 + np.arange(1, n)
    col = np.concatenate([np.arange(1, n), np.zeros(n - 1, dtype=np.int64)]).astype(np.int32)
    batches = np.array([[0], [0], [0]], dtype=np.int32)
    hops = O.sample_nodewise(rowptr, col, batches, (5,), 4)
    picks = [tuple(hops[0].col_vertex[hops[0].mb_coloff[i]:hops[0].mb_coloff[i + 1]]) for i in range(3)]
    assert len(set(picks)) == 3


def test_degenerate_inputs():
    rowptr = np.array([0, 0, 1, 1], dtype=np.int64)      # 0: isolated, 1 -> 2, 2: isolated
    col = np.array([2], dtype=np.int32)
    hops = O.sample_nodewise(rowptr, col, np.array([[0, 1], [2, 0]], dtype=np.int32), (3, 3), 1)
    assert hops[0].rows == 4 and hops[0].nnz == 1 and hops[0].col_vertex.tolist() == [2]
    assert hops[0].mb_coloff.tolist() == [0, 1, 1]
    assert hops[1].rows == 1 and hops[1].nnz == 0 and hops[1].ncols == 0
    assert hops[1].rowptr.tolist() == [0, 0]
    with pytest.raises(ValueError):
        O.sample_nodewise(rowptr, col, np.array([[0, 0]], dtype=np.int32), (1,), 1)   # repeated seed
    with pytest.raises(ValueError):
        O.sample_nodewise(rowptr, col, np.array([[0, 3]], dtype=np.int32), (1,), 1)   # out of range
    with pytest.raises(ValueError):
        O.sample_nodewise(rowptr, col, np.array([[0, 1]], dtype=np.int32), (0,), 1)   # fanout < 1
