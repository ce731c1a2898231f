"""Parity of the HIP forward aggregation with the CPU oracle, through the C ABI.

The kernel adds a row's entries in ascending order in fp32, the oracle in double with one final rounding.
Tolerance, from the arithmetic: a sequential fp32 sum of m terms is off by at most (m - 1) u S with
S = sum |x_e| and u = 2^-24; the mean adds one more rounding of the quotient, and the oracle's own final
rounding one more: |gpu - oracle| <= (m + 2) u S (divided by m for the mean).  Written below as `bound`.
"""
import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr

pytestmark = pytest.mark.gpu
U = 2.0 ** -24


@pytest.fixture(scope="module")
def mods():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    assert torch.cuda.is_available()
    return O, bms


def _check(O, bms, res, ref_hops, h, X, mean):
    out = bms.aggregate_hop(res, h, torch.from_numpy(X).cuda(), mean=mean).cpu().numpy()
    ref = O.aggregate(ref_hops[h], X, mean=mean)
    m = np.diff(ref_hops[h].rowptr).astype(np.float64)[:, None]
    S = O.aggregate(ref_hops[h], np.abs(X), mean=False).astype(np.float64)
    bound = (m + 2) * U * S * 1.0001
    if mean:
        bound = bound / np.maximum(m, 1.0)
    err = np.abs(out.astype(np.float64) - ref.astype(np.float64))
    assert out.shape == ref.shape
    assert np.all(err <= bound), (h, mean, float(err.max()), float(bound[err > bound].min()) if (err > bound).any() else 0)
    return out


@pytest.mark.parametrize("f", [128, 100, 7, 1, 260])
def test_nodewise_hops_mean_and_sum(mods, f):
    O, bms = mods
    rng = np.random.default_rng(f)
    rowptr, col = random_csr(20000, 14.0, rng)
    batches = random_batches(20000, 6, 100, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (10, 5), 3)
    ref = O.sample_nodewise(rowptr, col, batches, (10, 5), 3)
    for h in (0, 1):
        X = rng.standard_normal((ref[h].ncols, f)).astype(np.float32)
        for mean in (True, False):
            _check(O, bms, res, ref, h, X, mean)


def test_small_integer_features_sum_exactly(mods):
    O, bms = mods
    rng = np.random.default_rng(12)
    rowptr, col = random_csr(5000, 30.0, rng)
    batches = random_batches(5000, 4, 64, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (40, 3), 5)  # wide rows too
    ref = O.sample_nodewise(rowptr, col, batches, (40, 3), 5)
    for h in (0, 1):
        X = rng.integers(-100, 100, size=(ref[h].ncols, 12)).astype(np.float32)
        out = bms.aggregate_hop(res, h, torch.from_numpy(X).cuda(), mean=False).cpu().numpy()
        assert np.array_equal(out, O.aggregate(ref[h], X, mean=False))
    ones = np.ones((ref[0].ncols, 4), dtype=np.float32)
    out = bms.aggregate_hop(res, 0, torch.from_numpy(ones).cuda(), mean=True).cpu().numpy()
    assert np.array_equal(out, (np.diff(ref[0].rowptr) > 0)[:, None].repeat(4, axis=1).astype(np.float32))


def test_layerwise_hops_and_rows_without_entries(mods):
    O, bms = mods
    rng = np.random.default_rng(13)
    rowptr, col = random_csr(8000, 20.0, rng, symmetric=False)
    batches = random_batches(8000, 5, 50, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), (60, 60), 2)
    ref = O.sample_ladies(rowptr, col, batches, (60, 60), 2)
    assert (np.diff(ref[1].rowptr) == 0).any()
    for h in (0, 1):
        X = rng.standard_normal((ref[h].ncols, 32)).astype(np.float32)
        _check(O, bms, res, ref, h, X, True)


def test_fetch_then_aggregate_down_to_the_seeds(mods):
    # the consumer's chain (Sec. 6.2): features of the last frontier, then one aggregation per hop, last hop first
    O, bms = mods
    rng = np.random.default_rng(14)
    rowptr, col = random_csr(30000, 10.0, rng)
    batches = random_batches(30000, 8, 64, rng)
    H = rng.standard_normal((30000, 64)).astype(np.float32)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (5, 5, 5), 9)
    ref = O.sample_nodewise(rowptr, col, batches, (5, 5, 5), 9)
    X = bms.fetch_features(torch.from_numpy(H).cuda(), res.hop(2).col_vertex)
    Xr = O.fetch_features(H, ref[2].col_vertex)
    assert np.array_equal(X.cpu().numpy(), Xr)
    for h in (2, 1, 0):
        X = bms.aggregate_hop(res, h, X, mean=True)
        Xr64 = O.aggregate(ref[h], Xr, mean=True)
        # errors compound over the three levels: each level at most (m + 2) u times the mean of |inputs|
        assert np.allclose(X.cpu().numpy(), Xr64, rtol=0, atol=3 * 8 * U * np.abs(H).max())
        Xr = Xr64
    assert X.shape == (8 * 64, 64)


def test_errors(mods):
    O, bms = mods
    rng = np.random.default_rng(15)
    rowptr, col = random_csr(100, 5.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, random_batches(100, 2, 5, rng), (3,), 1)
    ncols = res.sizes()[0][2]
    X = torch.zeros((ncols, 4), device="cuda")
    with pytest.raises(bms.BmsError) as e:
        bms._check(bms.lib().bms_aggregate_hop(res.handle, 3, X.data_ptr(), 4, 1, X.data_ptr(), None))
    assert e.value.code == bms.EINVAL
    with pytest.raises(ValueError):
        bms.aggregate_hop(res, 0, torch.zeros((ncols + 1, 4), device="cuda"))
