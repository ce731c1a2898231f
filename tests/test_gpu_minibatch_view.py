"""bms_result_minibatch: one minibatch cut out of the stacked result, against the oracle's single-minibatch call
(bulk sampling equals the stack of the k minibatches, Eq. 1), for both samplers and the kept-frontier variant."""
import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr

pytestmark = pytest.mark.gpu


def _check_views(res, k, single):
    from paper_2311_02909_amd import bms
    for i in range(k):
        ref = single(i)
        for h, r in enumerate(ref):
            m = res.minibatch(h, i)
            assert (m.rows, m.nnz, m.ncols) == (r.rows, r.nnz, r.ncols), (h, i)
            assert np.array_equal(m.row_vertex.cpu().numpy(), r.row_vertex)
            assert np.array_equal((m.rowptr - m.edge0).cpu().numpy(), r.rowptr)
            assert np.array_equal(m.col.cpu().numpy(), r.col)
            assert np.array_equal(m.col_vertex.cpu().numpy(), r.col_vertex)
            if r.row_self is not None:
                assert np.array_equal(m.row_self.cpu().numpy(), r.row_self)
            else:
                assert m.row_self is None
            hop = res.hop(h)   # and the view really is a window of the stacked arrays
            assert m.row0 == int(hop.mb_rowoff[i]) and m.col0 == int(hop.mb_coloff[i])
            assert m.edge0 == int(hop.rowptr[m.row0])
    for bad in ((0, -1), (0, k), (-1, 0), (res.L, 0)):
        with pytest.raises(bms.BmsError) as e:
            res.minibatch(*bad)
        assert e.value.code == bms.EINVAL


@pytest.mark.parametrize("union_dst", [False, True])
def test_minibatch_views_nodewise(union_dst):
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(61)
    n, k, b, fan = 30000, 7, 150, (6, 4, 3)
    rowptr, col = random_csr(n, 14.0, rng)
    batches = random_batches(n, k, b, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), fan, 5, mb_base=100, union_dst=union_dst)
    _check_views(res, k, lambda i: O.sample_nodewise(rowptr, col, batches[i:i + 1], fan, 5, mb_base=100 + i,
                                                     union_dst=union_dst))
    # a recycled result drops the cached offsets: the views follow the new contents
    other = random_batches(n, k, b, rng)
    res = bms.sample_nodewise(csr, torch.from_numpy(other).cuda(), fan, 6, recycle=res, union_dst=union_dst)
    _check_views(res, k, lambda i: O.sample_nodewise(rowptr, col, other[i:i + 1], fan, 6, mb_base=i,
                                                     union_dst=union_dst))


def test_minibatch_views_ladies_and_aggregation_per_minibatch():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(62)
    n, k, b, s = 20000, 5, 64, (128, 64)
    rowptr, col = random_csr(n, 18.0, rng)
    batches = random_batches(n, k, b, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), s, 9)
    _check_views(res, k, lambda i: O.sample_ladies(rowptr, col, batches[i:i + 1], s, 9, mb_base=i))
    # A_i H_i of one minibatch from its view equals the stacked aggregation's rows of that minibatch
    hop = res.hop(1)
    X = torch.randint(-8, 9, (hop.ncols, 16), device="cuda").float()     # small integers: sums are exact
    Y = bms.aggregate_hop(res, 1, X, mean=False)
    for i in range(k):
        m = res.minibatch(1, i)
        Xi = X[m.col0:m.col0 + m.ncols]
        A = torch.zeros((m.rows, m.ncols), device="cuda")
        lens = (m.rowptr[1:] - m.rowptr[:-1])
        A[torch.arange(m.rows, device="cuda").repeat_interleave(lens), m.col.long()] = 1.0
        assert torch.equal(A @ Xi, Y[m.row0:m.row0 + m.rows])
