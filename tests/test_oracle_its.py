"""Pins for the without-replacement rule of the GraphSAGE SAMPLE step (no GPU)."""
import itertools

import numpy as np
from scipy import stats

import brute
from oracle import bms_oracle as O


def test_removal_rule_equals_its_on_zeroed_weights_exhaustively():
    # every (deg, s) with s < deg <= 12, many keys: the oracle's rule must pick exactly the
    # positions that literal ITS with chosen weights set to zero picks
    for deg in range(2, 13):
        for s in range(1, deg):
            for t in range(12):
                key = O.rowkey(100 + t, deg % 3, s, deg * 31 + t)
                got = O.its_distinct(key, deg, s)
                assert got == brute.distinct_positions_literal(key, deg, s), (deg, s, t)
                assert got == sorted(set(got)) and got[-1] < deg and len(got) == s


def test_removal_rule_large_degree_and_fanout():
    for deg, s in ((1000, 15), (17000, 10), (200, 150), (65, 64)):
        key = O.rowkey(7, 1, 2, deg)
        got = O.its_distinct(key, deg, s)
        assert got == brute.distinct_positions_literal(key, deg, s)


def test_subsets_are_uniform_chi_square():
    # deg 5, s 2: the C(5,2) = 10 subsets are equally likely
    subsets = {c: 0 for c in itertools.combinations(range(5), 2)}
    for t in range(20000):
        subsets[tuple(O.its_distinct(O.rowkey(t, 0, 0, 3), 5, 2))] += 1
    p = stats.chisquare(list(subsets.values())).pvalue
    assert p > 1e-3, (p, subsets)
    # deg 6, s 3: 20 subsets
    subsets = {c: 0 for c in itertools.combinations(range(6), 3)}
    for t in range(30000):
        subsets[tuple(O.its_distinct(O.rowkey(11, 1, t, 9), 6, 3))] += 1
    p = stats.chisquare(list(subsets.values())).pvalue
    assert p > 1e-3, (p, subsets)


def test_single_draw_and_inclusion_marginals():
    cells = np.zeros(7)
    for t in range(14000):
        cells[O.its_distinct(O.rowkey(3, 2, 1, t), 7, 1)[0]] += 1
    assert stats.chisquare(cells).pvalue > 1e-3
    # deg 9, s 4: every position is included with probability 4/9
    inc = np.zeros(9)
    trials = 18000
    for t in range(trials):
        inc[O.its_distinct(O.rowkey(t, 0, 5, 8), 9, 4)] += 1
    z = (inc / trials - 4 / 9) / np.sqrt((4 / 9) * (5 / 9) / trials)
    assert np.abs(z).max() < 4.0, z
