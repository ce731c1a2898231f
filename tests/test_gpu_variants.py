"""Parity of the node-wise variants with the CPU oracle (bit-exact), through the C ABI.

union_dst: the frontier's own vertices stay columns (next frontier = frontier + sampled vertices) and every row
reports its own column.  replace: the s draws of a row are independent and the row keeps the distinct picks."""
import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr, skewed_csr
from parity import assert_hops_equal

pytestmark = pytest.mark.gpu

EXTRACTS = (None, "sort", "buckets", "bitmap")


def _check(rowptr, col, batches, fanouts, seed, mb_base=0, extracts=EXTRACTS, **variant):
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    ref = O.sample_nodewise(rowptr, col, batches, fanouts, seed, mb_base, **variant)
    res = None
    for extract in extracts:
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), fanouts, seed, mb_base=mb_base,
                                  extract=extract, **variant)
        assert_hops_equal(res.hops(), ref, what="%s extract=%s fanouts=%s" % (variant, extract, fanouts))
    return csr, res, ref


@pytest.mark.parametrize("fanouts", [(3,), (4, 4), (8, 3, 2), (15, 10, 5), (16, 2), (32, 2), (1, 1, 1), (40, 3), (2048, 2)])
def test_union_dst_all_lane_capacities(fanouts):
    rng = np.random.default_rng(100 + sum(fanouts))
    rowptr, col = random_csr(20000, 24.0, rng)
    batches = random_batches(20000, 5, 300, rng)
    _, res, ref = _check(rowptr, col, batches, fanouts, 7, mb_base=3, union_dst=True)
    for h, hop in enumerate(res.hops()):
        # every frontier contains the one before it, and a row's own column leads back to its vertex
        own = hop.col_vertex[(hop.mb_coloff[:-1].repeat_interleave(hop.mb_rowoff[1:] - hop.mb_rowoff[:-1])
                              + hop.row_self).long()]
        assert torch.equal(own, hop.row_vertex)


def test_union_dst_full_fanout_directed_with_loops_and_isolated_rows():
    rng = np.random.default_rng(31)
    rowptr, col = random_csr(3000, 3.0, rng, symmetric=False, allow_loops=True)   # many vertices without out-edges
    assert (np.diff(rowptr) == 0).sum() > 100
    maxdeg = int(np.diff(rowptr).max())
    batches = random_batches(3000, 4, 33, rng)
    _check(rowptr, col, batches, (maxdeg, 2**31 - 1, maxdeg + 1), 1, union_dst=True)
    _check(rowptr, col, batches, (2, 1), 1, union_dst=True)


def test_union_dst_recycled_calls_and_change_of_variant():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(32)
    rowptr, col = random_csr(50000, 12.0, rng)
    batches = random_batches(50000, 8, 500, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    bt = torch.from_numpy(batches).cuda()
    fan = (6, 5, 4)
    ref_u = O.sample_nodewise(rowptr, col, batches, fan, 77, union_dst=True)
    ref_p = O.sample_nodewise(rowptr, col, batches, fan, 77)
    res = None
    for union in (True, True, True, False, False, True):   # the same result handle through both variants
        res = bms.sample_nodewise(csr, bt, fan, 77, recycle=res, union_dst=union)
        assert_hops_equal(res.hops(), ref_u if union else ref_p, what="recycled, union=%s" % union)


@pytest.mark.parametrize("extract", [None, "buckets"])
def test_union_dst_seed_out_of_range_on_the_no_round_trip_path(extract):
    # a recycled result of a remembered shape enqueues every hop before it reads the seed check back; with union_dst
    # the seed itself travels through EXTRACT as an entry, so a seed outside [0, n) must be made harmless on the
    # device: the call reports BMS_ERANGE, the recycled result is left empty, and the handles keep working
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(33)
    n = 50000
    rowptr, col = random_csr(n, 12.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    fan = (6, 5, 4)
    res = None
    for seed in (1, 2):   # the second call runs without host round trips
        batches = random_batches(n, 8, 500, rng)
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), fan, seed, recycle=res, union_dst=True,
                                  extract=extract)
        assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, batches, fan, seed, union_dst=True))
    for bad_id in (n, 2**31 - 1, -1):
        bad = random_batches(n, 8, 500, rng)
        bad[3, 17] = bad_id
        with pytest.raises(bms.BmsError) as e:
            bms.sample_nodewise(csr, torch.from_numpy(bad).cuda(), fan, 3, recycle=res, union_dst=True, extract=extract)
        assert e.value.code == bms.ERANGE
        with pytest.raises(bms.BmsError) as e:   # the recycled result is empty after the failed call
            res.hop(0)
        assert e.value.code == bms.EINVAL
        good = random_batches(n, 8, 500, rng)
        for seed in (4, 5):   # recovers, and gets back onto the no-round-trip path
            res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), fan, seed, recycle=res, union_dst=True,
                                      extract=extract)
            assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, good, fan, seed, union_dst=True))


def test_union_dst_many_small_minibatches_and_single_vertex_batches():
    rng = np.random.default_rng(33)
    rowptr, col = random_csr(4000, 8.0, rng)
    _check(rowptr, col, random_batches(4000, 700, 1, rng), (3, 3), 5, extracts=(None, "sort"), union_dst=True)
    _check(rowptr, col, random_batches(4000, 2, 1500, rng), (5, 5), 5, union_dst=True)


def test_union_dst_is_rejected_for_layerwise_sampling():
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(34)
    rowptr, col = random_csr(500, 5.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    import ctypes as C
    out = C.c_void_p()
    opts = bms._Opts(stream=None, mb_base=0, flags=bms.UNION_DST, recycle=None, scratch_limit=0)
    bt = torch.from_numpy(random_batches(500, 2, 8, rng)).cuda()
    s = (C.c_int32 * 1)(16)
    rc = bms.lib().bms_sample_ladies(csr.handle, bt.data_ptr(), 2, 8, s, 1, 1, C.byref(opts), C.byref(out))
    assert rc == bms.EINVAL and not out.value


def test_union_dst_on_the_mid_size_workload():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    g, batches, w = synth.make_workload("mid_sage", device="cuda")
    csr = bms.Csr(g.rowptr, g.col)
    res = bms.sample_nodewise(csr, batches, w["params"], synth.SAMPLING_SEED, union_dst=True)
    res = bms.sample_nodewise(csr, batches, w["params"], synth.SAMPLING_SEED, union_dst=True, recycle=res)
    print("\n  sizes", res.sizes(), flush=True)
    ref = O.sample_nodewise(g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy(), w["params"],
                            synth.SAMPLING_SEED, union_dst=True)
    assert_hops_equal(res.hops(), ref, what="mid_sage union_dst")


@pytest.mark.parametrize("variant", [dict(replace=True), dict(replace=True, union_dst=True)], ids=lambda v: "+".join(sorted(v)))
@pytest.mark.parametrize("fanouts", [(3,), (4, 4), (8, 3, 2), (15, 10, 5), (16, 2), (32, 2), (1, 1, 1), (33, 3), (40, 40),
                                     (200, 3), (2048, 2)])
def test_replace_all_lane_capacities_and_wave_sorted_rows(fanouts, variant):
    rng = np.random.default_rng(200 + sum(fanouts))
    rowptr, col = skewed_csr(6000, 100000, rng)     # some rows have thousands of entries, some none
    assert np.diff(rowptr).max() > 2048 and np.diff(rowptr).min() == 0
    batches = random_batches(6000, 3, 300, rng)
    _, res, ref = _check(rowptr, col, batches, fanouts, 11, mb_base=5, **variant)
    deg = np.diff(rowptr)
    for h, hop in enumerate(ref):   # the oracle's rows really are shorter than the plain method's somewhere
        lens = np.diff(hop.rowptr)
        assert (lens <= np.minimum(deg[hop.row_vertex], fanouts[h])).all()
    assert max(fanouts) == 1 or any((np.diff(hop.rowptr) < np.minimum(deg[hop.row_vertex], fanouts[h])).any()
                                    for h, hop in enumerate(ref))


def test_replace_recycled_calls_and_change_of_variant():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(42)
    rowptr, col = random_csr(50000, 12.0, rng)
    batches = random_batches(50000, 8, 500, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    bt = torch.from_numpy(batches).cuda()
    fan = (6, 5, 4)
    refs = {(u, r): O.sample_nodewise(rowptr, col, batches, fan, 77, union_dst=u, replace=r)
            for u in (False, True) for r in (False, True)}
    res = None
    for u, r in ((False, True), (False, True), (True, True), (True, True), (False, False), (True, False), (False, True)):
        res = bms.sample_nodewise(csr, bt, fan, 77, recycle=res, union_dst=u, replace=r)
        assert_hops_equal(res.hops(), refs[(u, r)], what="recycled, union=%s replace=%s" % (u, r))


def test_replace_limits():
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(43)
    rowptr, col = random_csr(500, 5.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    bt = torch.from_numpy(random_batches(500, 2, 8, rng)).cuda()
    with pytest.raises(bms.BmsError) as e:
        bms.sample_nodewise(csr, bt, (3, 2049), 1, replace=True)
    assert e.value.code == bms.EINVAL
    # one draw per row: with and without replacement are the same sample
    a = bms.sample_nodewise(csr, bt, (1, 1, 1), 9, replace=True)
    b = bms.sample_nodewise(csr, bt, (1, 1, 1), 9)
    for ha, hb in zip(a.hops(), b.hops()):
        assert torch.equal(ha.col, hb.col) and torch.equal(ha.col_vertex, hb.col_vertex) and torch.equal(ha.rowptr, hb.rowptr)


def test_replace_on_the_mid_size_workload():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    g, batches, w = synth.make_workload("mid_sage", device="cuda")
    csr = bms.Csr(g.rowptr, g.col)
    res = None
    for _ in range(2):
        res = bms.sample_nodewise(csr, batches, w["params"], synth.SAMPLING_SEED, replace=True, recycle=res)
    print("\n  sizes", res.sizes(), flush=True)
    ref = O.sample_nodewise(g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy(), w["params"],
                            synth.SAMPLING_SEED, replace=True)
    assert_hops_equal(res.hops(), ref, what="mid_sage replace")
