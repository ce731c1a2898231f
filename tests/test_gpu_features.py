"""Parity of the HIP feature fetch with the CPU oracle (bit-exact copies), through the C ABI."""
import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    assert torch.cuda.is_available()
    return O, bms


def _bits(x):
    return np.ascontiguousarray(x).view(np.uint32)


@pytest.mark.parametrize("n,f,m", [(1000, 128, 5000), (1000, 100, 4999), (777, 1, 3000), (50, 37, 1), (300, 602, 1500),
                                   (4000, 4, 100001), (10, 256, 7)])
def test_fetch_matches_oracle_bit_for_bit(mods, n, f, m):
    # widths with and without 16-byte rows, rows longer than one wave moves at once, ragged tails
    O, bms = mods
    rng = np.random.default_rng(n + f + m)
    H = rng.standard_normal((n, f)).astype(np.float32)
    H.ravel()[::97] = np.nan
    H.ravel()[1::89] = -0.0
    ids = rng.integers(0, n, size=m).astype(np.int32)
    out = bms.fetch_features(torch.from_numpy(H).cuda(), torch.from_numpy(ids).cuda())
    assert np.array_equal(_bits(out.cpu().numpy()), _bits(O.fetch_features(H, ids)))


def test_unaligned_views_take_the_scalar_path(mods):
    O, bms = mods
    rng = np.random.default_rng(8)
    base = torch.from_numpy(rng.standard_normal(200 * 8 + 1).astype(np.float32)).cuda()
    H = base[1:].view(200, 8)  # 4 bytes off a 16-byte boundary
    ids = torch.from_numpy(rng.integers(0, 200, size=999).astype(np.int32)).cuda()
    out = bms.fetch_features(H, ids)
    assert np.array_equal(_bits(out.cpu().numpy()), _bits(O.fetch_features(H.cpu().numpy(), ids.cpu().numpy())))


def test_last_frontier_of_a_bulk_sample(mods):
    O, bms = mods
    rng = np.random.default_rng(9)
    rowptr, col = random_csr(20000, 12.0, rng)
    batches = random_batches(20000, 8, 128, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (10, 5), 3)
    last = res.hop(1)
    H = rng.standard_normal((20000, 100)).astype(np.float32)
    out = bms.fetch_features(torch.from_numpy(H).cuda(), last.col_vertex)
    ref_hop = O.sample_nodewise(rowptr, col, batches, (10, 5), 3)[1]
    assert np.array_equal(_bits(out.cpu().numpy()), _bits(O.fetch_features(H, ref_hop.col_vertex)))


def test_errors_and_empty(mods):
    O, bms = mods
    H = torch.arange(12, dtype=torch.float32, device="cuda").view(4, 3)
    assert bms.fetch_features(H, torch.zeros(0, dtype=torch.int32, device="cuda")).shape == (0, 3)
    for bad in ([0, 4, 1], [-1]):
        ids = torch.tensor(bad, dtype=torch.int32, device="cuda")
        out = torch.full((len(bad), 3), 7.0, device="cuda")
        with pytest.raises(bms.BmsError) as e:
            bms.fetch_features(H, ids, out=out)
        assert e.value.code == bms.ERANGE
        host = out.cpu().numpy()
        for j, v in enumerate(bad):  # rows of valid ids are still fetched, rows of bad ids are zeros
            assert host[j].tolist() == (H[v].cpu().numpy().tolist() if 0 <= v < 4 else [0.0, 0.0, 0.0])
    good = bms.fetch_features(H, torch.tensor([3, 3, 0], dtype=torch.int32, device="cuda"))
    assert good.cpu().numpy().tolist() == [[9, 10, 11], [9, 10, 11], [0, 1, 2]]
