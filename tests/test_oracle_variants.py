"""Pins for the two GraphSAGE variants of the oracle -- no GPU.

union_dst: the frontier's own vertices stay columns of the sampled adjacency (next frontier = frontier + sampled
vertices).  replace: the s draws of a row are independent (the repeat-until-distinct step of Sec. 4.1.2 left out)
and the row keeps the distinct picks."""
import itertools

import numpy as np
import pytest

import brute
from conftest import random_batches, random_csr
from oracle import bms_oracle as O

VARIANTS = [dict(union_dst=True), dict(replace=True), dict(union_dst=True, replace=True)]


@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: "+".join(sorted(v)))
@pytest.mark.parametrize("n,avg,k,b,fanouts,seed", [
    (24, 5.0, 3, 4, (2, 2), 1),
    (40, 8.0, 4, 6, (3, 2, 2), 2),
    (64, 12.0, 2, 8, (5, 3), 3),
    (33, 6.0, 5, 1, (1, 1, 1), 4),
    (48, 10.0, 2, 5, (4, 1, 6), 5),
])
def test_variants_match_dense_brute_force(n, avg, k, b, fanouts, seed, variant):
    rng = np.random.default_rng(seed)
    rowptr, col = random_csr(n, avg, rng, symmetric=seed % 2 == 1, allow_loops=seed % 2 == 0)
    batches = random_batches(n, k, b, rng)
    A = brute.dense_adjacency(rowptr, col)
    ref = brute.nodewise(A, batches, fanouts, 50 + seed, mb_base=seed, **variant)
    hops = O.sample_nodewise(rowptr, col, batches, fanouts, 50 + seed, seed, **variant)
    for h, hop in enumerate(hops):
        for i in range(k):
            F, Adense, kept = ref[i][h]
            r0, r1 = hop.mb_rowoff[i], hop.mb_rowoff[i + 1]
            c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
            assert hop.row_vertex[r0:r1].tolist() == F
            assert hop.col_vertex[c0:c1].tolist() == kept.tolist()
            assert (brute.hop_block_dense(hop, i) == Adense).all()
            if variant.get("union_dst"):
                # the row's own column: position of its vertex among the kept columns
                assert hop.row_self[r0:r1].tolist() == [kept.tolist().index(v) for v in F]
        assert (hop.row_self is not None) == bool(variant.get("union_dst"))
        assert hop.nnz == hop.rowptr[-1] == len(hop.col) and hop.ncols == len(hop.col_vertex)
        if h + 1 < len(hops):
            assert (hops[h + 1].row_vertex == hop.col_vertex).all()
            assert (hops[h + 1].mb_rowoff == hop.mb_coloff).all()


def test_union_with_full_fanout_gives_closed_balls():
    # no randomness left: the frontier after h hops is every vertex within distance h of the batch
    rng = np.random.default_rng(11)
    n = 70
    rowptr, col = random_csr(n, 4.0, rng)
    A = brute.dense_adjacency(rowptr, col)
    maxdeg = int(np.diff(rowptr).max())
    batches = random_batches(n, 3, 3, rng)
    hops = O.sample_nodewise(rowptr, col, batches, (maxdeg,) * 4, 1, union_dst=True)
    reach = A + np.eye(n, dtype=np.int64)
    for i in range(3):
        ball = np.zeros(n, dtype=np.int64)
        ball[batches[i]] = 1
        for hop in hops:
            rows = hop.row_vertex[hop.mb_rowoff[i]:hop.mb_rowoff[i + 1]]
            assert sorted(rows.tolist()) == np.nonzero(ball)[0].tolist()
            ball = (ball @ reach > 0).astype(np.int64)
            cols = hop.col_vertex[hop.mb_coloff[i]:hop.mb_coloff[i + 1]]
            assert cols.tolist() == np.nonzero(ball)[0].tolist()
            # and the rows are the exact rows of A restricted to the ball
            assert (brute.hop_block_dense(hop, i) == A[rows][:, cols]).all()


def test_union_keeps_frontier_and_samples_like_the_plain_method():
    rng = np.random.default_rng(12)
    n = 2000
    rowptr, col = random_csr(n, 20.0, rng)
    batches = random_batches(n, 5, 40, rng)
    fan = (6, 4, 3)
    plain = O.sample_nodewise(rowptr, col, batches, fan, 9, mb_base=2)
    union = O.sample_nodewise(rowptr, col, batches, fan, 9, mb_base=2, union_dst=True)

    def rows_by_vertex(hop, i):
        out = {}
        c0 = hop.mb_coloff[i]
        for r in range(hop.mb_rowoff[i], hop.mb_rowoff[i + 1]):
            out[int(hop.row_vertex[r])] = hop.col_vertex[c0 + hop.col[hop.rowptr[r]:hop.rowptr[r + 1]]].tolist()
        return out

    shared = 0
    for h in range(3):
        for i in range(5):
            pu, pp = rows_by_vertex(union[h], i), rows_by_vertex(plain[h], i)
            cols = set(union[h].col_vertex[union[h].mb_coloff[i]:union[h].mb_coloff[i + 1]].tolist())
            assert set(pu) <= cols                                  # frontier kept
            assert cols == set(pu) | {g for row in pu.values() for g in row}   # and nothing else added
            # the random stream of a row depends on (seed, hop, minibatch, vertex) only, so a vertex that is in
            # both frontiers gets the same neighbours; at hop 0 that is every row
            for v in set(pu) & set(pp):
                assert pu[v] == pp[v]
                shared += 1
            if h == 0:
                assert list(pu) == list(pp) == batches[i].tolist()
            r0, r1 = union[h].mb_rowoff[i], union[h].mb_rowoff[i + 1]
            own = union[h].col_vertex[union[h].mb_coloff[i] + union[h].row_self[r0:r1]]
            assert (own == union[h].row_vertex[r0:r1]).all()
    assert shared > 500


def test_replace_positions_exhaustively_against_the_set_of_draws():
    for deg, s, seed in itertools.product(range(1, 13), range(1, 9), range(5)):
        key = O.rowkey(seed, 1, 2, 100 + deg)
        want = sorted({O.bounded32(O.draw32(key, j), deg) for j in range(s)})
        assert O.its_replace(key, deg, s) == want
    # one draw: with and without replacement are the same pick
    for deg in (2, 3, 17, 1000, 2**31 - 1):
        key = O.rowkey(4, 0, 0, deg)
        assert O.its_replace(key, deg, 1) == O.its_distinct(key, deg, 1)


def test_replace_row_invariants_and_expected_row_length():
    rng = np.random.default_rng(13)
    n = 3000
    rowptr, col = random_csr(n, 30.0, rng)
    deg = np.diff(rowptr)
    batches = random_batches(n, 6, 50, rng)
    fan = (7, 4, 3)
    hops = O.sample_nodewise(rowptr, col, batches, fan, 21, replace=True)
    got = expect = 0.0
    for h, hop in enumerate(hops):
        lens = np.diff(hop.rowptr)
        d = deg[hop.row_vertex]
        assert (lens <= np.minimum(d, fan[h])).all() and (lens[d > 0] >= 1).all() and (lens[d == 0] == 0).all()
        for i in range(6):
            c0 = hop.mb_coloff[i]
            for r in range(hop.mb_rowoff[i], hop.mb_rowoff[i + 1]):
                g = hop.col_vertex[c0 + hop.col[hop.rowptr[r]:hop.rowptr[r + 1]]]
                v = hop.row_vertex[r]
                assert (np.diff(g) > 0).all() and np.isin(g, col[rowptr[v]:rowptr[v + 1]]).all()
        dd = d[d > 0].astype(np.float64)
        got += lens.sum()
        expect += (dd * (1.0 - (1.0 - 1.0 / dd) ** fan[h])).sum()   # E[#distinct] of s draws over deg cells
    assert abs(got - expect) < 0.02 * expect


def test_replace_distribution_chi_square():
    # a vertex of degree 3 sampled with s = 2 independent draws: the row is {a} with probability 1/9 each and
    # {a, b} with probability 2/9 each; over many seeds the six outcomes must fit (chi-square, 5 degrees of freedom)
    rowptr = np.array([0, 3, 4, 5, 6], dtype=np.int64)
    col = np.array([1, 2, 3, 0, 0, 0], dtype=np.int32)
    batches = np.array([[0]], dtype=np.int32)
    counts = {}
    N = 9000
    for seed in range(N):
        hop = O.sample_nodewise(rowptr, col, batches, (2,), seed, replace=True)[0]
        key = tuple(hop.col_vertex[hop.col].tolist())
        counts[key] = counts.get(key, 0) + 1
    prob = {(1,): 1 / 9, (2,): 1 / 9, (3,): 1 / 9, (1, 2): 2 / 9, (1, 3): 2 / 9, (2, 3): 2 / 9}
    assert set(counts) == set(prob)
    chi2 = sum((counts[o] - N * p) ** 2 / (N * p) for o, p in prob.items())
    assert chi2 < 20.5   # 99.9 % quantile of chi-square with 5 degrees of freedom


@pytest.mark.parametrize("variant", VARIANTS, ids=lambda v: "+".join(sorted(v)))
def test_variants_bulk_equals_stacked_single_calls(variant):
    rng = np.random.default_rng(14)
    n = 500
    rowptr, col = random_csr(n, 9.0, rng)
    batches = random_batches(n, 4, 10, rng)
    fan = (4, 3)
    bulk = O.sample_nodewise(rowptr, col, batches, fan, 3, mb_base=10, **variant)
    for i in range(4):
        one = O.sample_nodewise(rowptr, col, batches[i:i + 1], fan, 3, mb_base=10 + i, **variant)
        for h in range(2):
            hb, ho = bulk[h], one[h]
            r0, r1 = hb.mb_rowoff[i], hb.mb_rowoff[i + 1]
            assert (hb.row_vertex[r0:r1] == ho.row_vertex).all()
            assert (hb.rowptr[r0:r1 + 1] - hb.rowptr[r0] == ho.rowptr).all()
            assert (hb.col[hb.rowptr[r0]:hb.rowptr[r1]] == ho.col).all()
            assert (hb.col_vertex[hb.mb_coloff[i]:hb.mb_coloff[i + 1]] == ho.col_vertex).all()
            if variant.get("union_dst"):
                assert (hb.row_self[r0:r1] == ho.row_self).all()


def test_unknown_variant_bit_is_rejected():
    import ctypes as C
    rowptr = np.array([0, 1, 2], dtype=np.int64)
    col = np.array([1, 0], dtype=np.int32)
    batches = np.array([[0]], dtype=np.int32)
    fan = np.array([1], dtype=np.int32)
    out = C.c_void_p()
    rc = O.lib().orc_sample_nodewise_variant(rowptr.ctypes.data, col.ctypes.data, 2, batches.ctypes.data, 1, 1,
                                             fan.ctypes.data, 1, 1, 0, 4, C.byref(out))
    assert rc == -1 and not out.value
