"""Pins for the oracle's random stream and range reduction (no GPU)."""
import numpy as np
from scipy import stats

from oracle import bms_oracle as O

M64 = (1 << 64) - 1
GOLD64 = 0x9E3779B97F4A7C15


def test_mix64_is_the_splitmix64_output_function():
    # Published SplitMix64 streams (state += golden gamma; output = finaliser(state)).
    state, got = 0, []
    for _ in range(3):
        state = (state + GOLD64) & M64
        got.append(O.mix64(state))
    assert got == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    state, got = 1234567, []
    for _ in range(5):
        state = (state + GOLD64) & M64
        got.append(O.mix64(state))
    assert got == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                   4593380528125082431, 16408922859458223821]


def _fin32_inverse(y):
    # invert  x ^= x>>16; x *= c1; x ^= x>>15; x *= c2; x ^= x>>16  with modular inverses
    c1, c2 = 0x7FEB352D, 0x846CA68B
    i1, i2 = pow(c1, -1, 1 << 32), pow(c2, -1, 1 << 32)
    y ^= y >> 16
    y = (y * i2) & 0xFFFFFFFF
    y ^= (y >> 15) ^ (y >> 30)
    y = (y * i1) & 0xFFFFFFFF
    y ^= y >> 16
    return y


def test_fin32_is_a_bijection_with_the_stated_constants():
    rng = np.random.default_rng(0)
    xs = [0, 1, 0xFFFFFFFF, 0x80000000] + [int(v) for v in rng.integers(0, 1 << 32, size=2000)]
    for x in xs:
        assert _fin32_inverse(O.fin32(x)) == x


def test_avalanche_of_both_finalisers():
    rng = np.random.default_rng(1)
    for fn, bits in ((O.fin32, 32), (O.mix64, 64)):
        flips = np.zeros((bits, bits))
        trials = 400
        for _ in range(trials):
            x = int(rng.integers(0, 1 << 63)) & ((1 << bits) - 1)
            y = fn(x)
            for i in range(bits):
                d = y ^ fn(x ^ (1 << i))
                flips[i] += [(d >> o) & 1 for o in range(bits)]
        p = flips / trials
        assert abs(p.mean() - 0.5) < 0.01
        assert p.min() > 0.35 and p.max() < 0.65


def test_rowkey_composition_and_field_separation():
    seed, h, mb, v = 42, 2, 7, 123456
    hopkey = O.mix64(seed ^ ((GOLD64 * (h + 1)) & M64))
    assert O.rowkey(seed, h, mb, v) == O.mix64(hopkey ^ ((mb << 32) | v))
    base = O.rowkey(seed, h, mb, v)
    others = {O.rowkey(seed + 1, h, mb, v), O.rowkey(seed, h + 1, mb, v),
              O.rowkey(seed, h, mb + 1, v), O.rowkey(seed, h, mb, v + 1),
              O.rowkey(seed, h, v & 0xFFFF, mb)}
    assert base not in others and len(others) == 5


def test_draw32_and_draw64_composition():
    key = O.rowkey(9, 0, 3, 77)
    lo, hi = key & 0xFFFFFFFF, key >> 32
    for j in (0, 1, 2, 1000, 0xFFFFFFFF):
        expect = O.fin32(O.fin32((lo + j * 0x9E3779B9) & 0xFFFFFFFF) ^ hi)
        assert O.draw32(key, j) == expect
    for j in (0, 1, 5, 12345):
        assert O.draw64(key, j) == (O.draw32(key, 2 * j) << 32) | O.draw32(key, 2 * j + 1)


def test_bounded_is_floor_of_scaled_product():
    rng = np.random.default_rng(2)
    for _ in range(2000):
        x = int(rng.integers(0, 1 << 32))
        m = int(rng.integers(1, 1 << 32))
        assert O.bounded32(x, m) == (x * m) >> 32 < m
        X = (int(rng.integers(0, 1 << 32)) << 32) | x
        W = (int(rng.integers(0, 1 << 31)) << 32) | m
        assert O.bounded64(X, W) == (X * W) >> 64 < W
    assert O.bounded32(0xFFFFFFFF, 1) == 0 and O.bounded32(0xFFFFFFFF, 10) == 9
    assert O.bounded64(M64, 1) == 0 and O.bounded64(M64, 7) == 6


def test_draw_stream_is_uniform_chi_square():
    # 64 cells over many keys and counters; deterministic seeds, so no flakiness
    cells = np.zeros(64)
    for mb in range(40):
        key = O.rowkey(5, 1, mb, 1000 + mb)
        for j in range(500):
            cells[O.bounded32(O.draw32(key, j), 64)] += 1
    p = stats.chisquare(cells).pvalue
    assert p > 1e-3, p
    # consecutive counters of one key are uncorrelated in their top bit
    key = O.rowkey(1, 0, 0, 0)
    bits = np.array([O.draw32(key, j) >> 31 for j in range(4000)])
    same = (bits[1:] == bits[:-1]).mean()
    assert abs(same - 0.5) < 0.03
