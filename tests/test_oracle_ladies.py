"""Pins for the oracle's LADIES path (Sec. 2.2 definition, Sec. 4.2) -- no GPU."""
import os

import numpy as np
import pytest
from scipy import stats

import brute
from conftest import random_batches, random_csr
from oracle import bms_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "ladies_worked_example.txt")


def _check_against_brute(rowptr, col, batches, s_per_layer, seed, mb_base=0, squared=False):
    A = brute.dense_adjacency(rowptr, col)
    ref = brute.ladies(A, batches, s_per_layer, seed, mb_base, squared)
    hops = O.sample_ladies(rowptr, col, batches, s_per_layer, seed, mb_base, squared)
    for h, hop in enumerate(hops):
        for i in range(len(batches)):
            F, P, S, AS = ref[i][h]
            r0, r1 = hop.mb_rowoff[i], hop.mb_rowoff[i + 1]
            c0, c1 = hop.mb_coloff[i], hop.mb_coloff[i + 1]
            p0, p1 = hop.p_off[i], hop.p_off[i + 1]
            assert hop.row_vertex[r0:r1].tolist() == F
            # column weights of Q A == brute-force adjacency counts, entry for entry
            dense_p = np.zeros(len(P), dtype=np.int64)
            dense_p[hop.p_col[p0:p1]] = hop.p_cnt[p0:p1]
            assert (dense_p == P).all()
            assert (hop.p_cnt[p0:p1] > 0).all() and (np.diff(hop.p_col[p0:p1]) > 0).all()
            assert hop.col_vertex[c0:c1].tolist() == S
            assert len(S) <= s_per_layer[h]
            assert (brute.hop_block_dense(hop, i) == AS).all()
        if h + 1 < len(hops):
            assert (hops[h + 1].row_vertex == hop.col_vertex).all()


@pytest.mark.parametrize("n,avg,k,b,s,seed,squared", [
    (24, 5.0, 3, 4, (3, 3), 1, False),
    (40, 8.0, 4, 6, (5, 4, 3), 2, False),
    (64, 12.0, 2, 8, (10, 20), 3, False),
    (30, 6.0, 3, 2, (1, 1, 1), 4, False),
    (40, 8.0, 3, 6, (5, 4), 5, True),
    (64, 14.0, 2, 7, (8, 8, 8), 6, True),
])
def test_matches_dense_brute_force(n, avg, k, b, s, seed, squared):
    rng = np.random.default_rng(seed)
    rowptr, col = random_csr(n, avg, rng)
    batches = random_batches(n, k, b, rng)
    _check_against_brute(rowptr, col, batches, s, 500 + seed, mb_base=seed, squared=squared)


def test_directed_graph_matches_brute_force():
    rng = np.random.default_rng(21)
    rowptr, col = random_csr(36, 7.0, rng, symmetric=False, allow_loops=True)
    _check_against_brute(rowptr, col, random_batches(36, 3, 5, rng), (4, 4), 9)


def _read_golden():
    vals = {}
    for line in open(GOLDEN):
        if line.startswith("#") or ":" not in line:
            continue
        key, rest = line.split(":")
        vals[key.strip()] = [int(x) for x in rest.split()]
    return vals


def _stand_in_graph():
    # 4 is adjacent to both batch vertices; 0, 2, 3 to exactly one; 1 and 5 are not adjacent
    edges = [(0, 1), (2, 1), (3, 5), (4, 1), (4, 5)]
    n = 6
    A = np.zeros((n, n), dtype=np.int64)
    for u, v in edges:
        A[u, v] = A[v, u] = 1
    rowptr = np.concatenate([[0], np.cumsum(A.sum(axis=1))]).astype(np.int64)
    col = np.concatenate([np.nonzero(A[v])[0] for v in range(n)]).astype(np.int32)
    return A, rowptr, col


def test_paper_worked_example_probabilities_and_extraction():
    g = _read_golden()
    A, rowptr, col = _stand_in_graph()
    batch = np.array([g["batch"]], dtype=np.int32)
    s = g["s"][0]
    numer, denom = np.array(g["prob_numerators"]), g["prob_denominator"][0]
    found = None
    for seed in range(200):
        hop = O.sample_ladies(rowptr, col, batch, (s,), seed, squared=True)[0]
        e = np.zeros(6, dtype=np.int64)
        e[hop.p_col] = hop.p_cnt
        assert (e * e == numer).all() and (e * e).sum() == denom       # the printed array
        if hop.col_vertex.tolist() == g["sampled"]:
            found = hop
            break
    assert found is not None, "no seed reproduced the paper's sampled set"
    # every edge between the batch {1,5} and the sampled {0,4}
    assert (brute.hop_block_dense(found, 0) == A[g["batch"]][:, g["sampled"]]).all()
    assert found.nnz == 3
    # unsquared reading (Sec. 4.2.1): same counts, denominator 5
    hop = O.sample_ladies(rowptr, col, batch, (s,), 0, squared=False)[0]
    assert hop.p_cnt.sum() == 5


def _twenty_vertex_graph():
    rng = np.random.default_rng(2020)
    return random_csr(20, 6.0, rng)


@pytest.mark.parametrize("squared", [False, True])
def test_single_draw_distribution_chi_square(squared):
    rowptr, col = _twenty_vertex_graph()
    A = brute.dense_adjacency(rowptr, col)
    batch = np.array([[2, 7, 11, 15]], dtype=np.int32)
    e = A[batch[0]].sum(axis=0)
    w = e * e if squared else e
    support = np.nonzero(w)[0]
    counts = np.zeros(20)
    trials = 20000
    for seed in range(trials):
        hop = O.sample_ladies(rowptr, col, batch, (1,), seed, squared=squared)[0]
        assert hop.ncols == 1
        counts[hop.col_vertex[0]] += 1
    assert counts[w == 0].sum() == 0              # only the aggregated neighbourhood is sampled
    expected = w[support] / w.sum() * trials
    assert stats.chisquare(counts[support], expected).pvalue > 1e-3


def test_inclusion_frequency_matches_closed_form():
    rowptr, col = _twenty_vertex_graph()
    A = brute.dense_adjacency(rowptr, col)
    batch = np.array([[0, 5, 9]], dtype=np.int32)
    e = A[batch[0]].sum(axis=0).astype(float)
    s, trials = 4, 20000
    inc = np.zeros(20)
    for t in range(trials):
        hop = O.sample_ladies(rowptr, col, batch, (s,), 7, mb_base=t)[0]
        inc[hop.col_vertex] += 1
    p = 1.0 - (1.0 - e / e.sum()) ** s
    sup = e > 0
    z = (inc[sup] / trials - p[sup]) / np.sqrt(p[sup] * (1 - p[sup]) / trials)
    assert np.abs(z).max() < 4.0, z
    assert inc[~sup].sum() == 0


def test_bulk_equals_stack_and_degenerate_inputs():
    rng = np.random.default_rng(14)
    rowptr, col = random_csr(300, 10.0, rng)
    batches = random_batches(300, 4, 12, rng)
    bulk = O.sample_ladies(rowptr, col, batches, (9, 9), 3, mb_base=2)
    for h in range(2):
        parts = [O.sample_ladies(rowptr, col, batches[i:i + 1], (9, 9), 3, mb_base=2 + i)[h] for i in range(4)]
        for name in ("row_vertex", "col", "col_vertex", "p_col", "p_cnt"):
            assert (np.concatenate([getattr(p, name) for p in parts]) == getattr(bulk[h], name)).all()
    # a batch of isolated vertices: empty P, nothing sampled, empty next frontier
    rowptr2 = np.array([0, 0, 0, 1, 2], dtype=np.int64)
    col2 = np.array([3, 2], dtype=np.int32)
    hops = O.sample_ladies(rowptr2, col2, np.array([[0, 1], [2, 0]], dtype=np.int32), (2, 2), 1)
    assert hops[0].p_off.tolist() == [0, 0, 1] and hops[0].mb_coloff.tolist() == [0, 0, 1]
    assert hops[0].rowptr.tolist() == [0, 0, 0, 1, 1]
    assert hops[1].rows == 1 and hops[1].col_vertex.tolist() == [2]
    with pytest.raises(ValueError):
        O.sample_ladies(rowptr2, col2, np.array([[1, 1]], dtype=np.int32), (1,), 1)
