"""Parity of the HIP node-wise sampler with the CPU oracle (bit-exact), through the C ABI."""
import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr, skewed_csr
from parity import assert_hops_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    assert torch.cuda.is_available()
    return O, bms, synth


def _run_both(mods, rowptr, col, batches, fanouts, seed, mb_base=0, device_csr=True):
    """Runs every EXTRACT kernel path of the library and compares each with the oracle."""
    O, bms, _ = mods
    rp, cl = torch.from_numpy(rowptr), torch.from_numpy(col)
    if device_csr:
        rp, cl = rp.cuda(), cl.cuda()
    csr = bms.Csr(rp, cl)
    ref = O.sample_nodewise(rowptr, col, batches, fanouts, seed, mb_base)
    for extract in ("sort", "buckets", "bitmap"):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), fanouts, seed, mb_base=mb_base,
                                  extract=extract)
        assert_hops_equal(res.hops(), ref, what="extract=%s fanouts=%s seed=%d" % (extract, fanouts, seed))
    return csr, res, ref


def test_tiny_workload(mods):
    O, bms, synth = mods
    g, batches, w = synth.make_workload("tiny_sage")
    print("tiny_sage:", g.describe(), flush=True)
    _run_both(mods, g.rowptr.numpy(), g.col.numpy(), batches.numpy(), w["params"], synth.SAMPLING_SEED)


@pytest.mark.parametrize("fanouts", [(3,), (4, 4), (5, 5), (8, 3, 2), (15, 10, 5), (16, 2), (17, 3), (32, 2), (1, 1, 1)])
def test_random_graph_all_lane_capacities(mods, fanouts):
    # n and b chosen so that a minibatch spans several 256-row tiles with a ragged tail
    rng = np.random.default_rng(sum(fanouts))
    rowptr, col = random_csr(20000, 24.0, rng)
    batches = random_batches(20000, 5, 300, rng)
    _run_both(mods, rowptr, col, batches, fanouts, 7, mb_base=3)


@pytest.mark.parametrize("fanouts", [(33, 2), (40, 40), (200, 3), (2048, 2)])
def test_wide_fanouts_one_wave_per_row(mods, fanouts):
    rng = np.random.default_rng(5)
    rowptr, col = random_csr(6000, 60.0, rng)       # skewed: some rows have thousands of entries
    assert np.diff(rowptr).max() > 2048
    batches = random_batches(6000, 3, 70, rng)
    _run_both(mods, rowptr, col, batches, fanouts, 11)


def test_fanout_at_least_max_degree_is_exact(mods):
    rng = np.random.default_rng(6)
    rowptr, col = random_csr(3000, 10.0, rng)
    maxdeg = int(np.diff(rowptr).max())
    batches = random_batches(3000, 4, 33, rng)
    for fan in ((maxdeg, maxdeg), (2**31 - 1, maxdeg + 7)):
        _, res, ref = _run_both(mods, rowptr, col, batches, fan, 1)
        # no randomness: a different seed gives the same result
        _, res2, _ = _run_both(mods, rowptr, col, batches, fan, 2)
        assert torch.equal(res.hop(1).col, res2.hop(1).col)


def test_host_csr_host_batches_directed_with_loops(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(8)
    rowptr, col = random_csr(5000, 9.0, rng, symmetric=False, allow_loops=True)
    batches = random_batches(5000, 6, 40, rng)
    csr = bms.Csr(torch.from_numpy(rowptr), torch.from_numpy(col))           # host arrays, copied
    res = bms.sample_nodewise(csr, batches, (6, 4), 21)                       # host batches
    assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, batches, (6, 4), 21))


def test_bulk_equals_stack_and_recycle(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(9)
    rowptr, col = random_csr(8000, 16.0, rng)
    batches = random_batches(8000, 6, 100, rng)
    csr, bulk, ref = _run_both(mods, rowptr, col, batches, (7, 5), 5, mb_base=40)
    res = None
    for i in range(6):        # k = 1 calls with the minibatch index advanced, reusing one result
        res = bms.sample_nodewise(csr, torch.from_numpy(batches[i:i + 1]).cuda(), (7, 5), 5, mb_base=40 + i,
                                  recycle=res)
        one = O.sample_nodewise(rowptr, col, batches[i:i + 1], (7, 5), 5, 40 + i)
        assert_hops_equal(res.hops(), one, what="minibatch %d alone" % i)
        for h in range(2):
            r0, r1 = ref[h].mb_coloff[i], ref[h].mb_coloff[i + 1]
            assert np.array_equal(res.hop(h).col_vertex.cpu().numpy(), ref[h].col_vertex[r0:r1])
    # the same csr handle keeps working for a larger call afterwards (scratch regrown, sets clean)
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (7, 5), 5, mb_base=40, recycle=res)
    assert_hops_equal(res.hops(), ref)


def test_degenerate_graphs_and_empty_frontiers(mods):
    O, bms, _ = mods
    # isolated vertices, a hop whose frontier becomes empty, a graph with no edges at all
    rowptr = np.array([0, 0, 1, 1, 1], dtype=np.int64)
    col = np.array([2], dtype=np.int32)
    batches = np.array([[0, 1], [2, 0], [3, 2]], dtype=np.int32)
    _run_both(mods, rowptr, col, batches, (3, 3, 3), 1)
    rowptr0 = np.zeros(11, dtype=np.int64)
    col0 = np.zeros(0, dtype=np.int32)
    _run_both(mods, rowptr0, col0, np.array([[1, 2, 3]], dtype=np.int32), (2, 2), 1)
    # one vertex, one self-loop
    _run_both(mods, np.array([0, 1], dtype=np.int64), np.array([0], dtype=np.int32),
              np.array([[0]], dtype=np.int32), (1, 1), 1)


def test_error_codes(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(10)
    rowptr, col = random_csr(500, 8.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    good = random_batches(500, 2, 8, rng)
    for bad, code in ((np.array([[1, 2, 1, 3]], dtype=np.int32), bms.ERANGE),
                      (np.array([[1, 500]], dtype=np.int32), bms.ERANGE),
                      (np.array([[-1, 4]], dtype=np.int32), bms.ERANGE)):
        with pytest.raises(bms.BmsError) as e:
            bms.sample_nodewise(csr, bad, (2,), 1)
        assert e.value.code == code
        # the handle is still usable and the vertex sets are clean again
        res = bms.sample_nodewise(csr, good, (3, 2), 4)
        assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, good, (3, 2), 4))
    with pytest.raises(bms.BmsError) as e:
        bms.sample_nodewise(csr, good, (3, 0), 1)
    assert e.value.code == bms.EINVAL
    big = int(np.diff(rowptr).max())
    # malformed matrices are refused at load time
    unsorted = col.copy()
    v = int(np.argmax(np.diff(rowptr)))
    unsorted[rowptr[v]], unsorted[rowptr[v] + 1] = unsorted[rowptr[v] + 1], unsorted[rowptr[v]]
    dup = col.copy()
    dup[rowptr[v] + 1] = dup[rowptr[v]]
    oob = col.copy()
    oob[3] = 500
    badptr = rowptr.copy()
    badptr[5] = badptr[6] + 1
    for rp, cl in ((rowptr, unsorted), (rowptr, dup), (rowptr, oob), (badptr, col)):
        with pytest.raises(bms.BmsError) as e:
            bms.Csr(torch.from_numpy(rp).cuda(), torch.from_numpy(cl).cuda())
        assert e.value.code == bms.EFORMAT, big


def test_profile_stages_are_reported(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(12)
    rowptr, col = random_csr(4000, 12.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = bms.sample_nodewise(csr, random_batches(4000, 4, 64, rng), (5, 5), 3, profile=True)
    names = [s[0] for s in res.stages()]
    assert names.count("nw_sample") == 2 and all(s[2] >= 0 for s in res.stages())
    assert len(set(names)) > 3
    # the cheap mode times the sampling kernel only; without a profile flag nothing is recorded
    res = bms.sample_nodewise(csr, random_batches(4000, 4, 64, rng), (5, 5), 3, profile="main", recycle=res)
    assert [(s[0], s[1]) for s in res.stages()] == [("nw_sample", 0), ("nw_sample", 1)]
    assert all(s[2] > 0 for s in res.stages())
    lad = bms.sample_ladies(csr, random_batches(4000, 4, 64, rng), (20,), 3, profile="main")
    assert [s[0] for s in lad.stages()] == ["ldw_accumulate"]
    res = bms.sample_nodewise(csr, random_batches(4000, 4, 64, rng), (5, 5), 3, recycle=res)
    assert res.stages() == []


def test_bucket_extract_many_buckets_and_large_batches(mods):
    # vertex range spanning many 2^18-id buckets, sparse so that most buckets hold a few ids;
    # b above the LDS seed-sort limit exercises the vertex-set seed check next to bucket EXTRACT
    O, bms, _ = mods
    rng = np.random.default_rng(44)
    n = 3_000_000
    src = rng.integers(0, n, size=400_000)
    dst = rng.integers(0, n, size=400_000)
    keep = src != dst
    key = np.unique(np.concatenate([src[keep] * n + dst[keep], dst[keep] * n + src[keep]]))
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, key // n + 1, 1)
    rowptr = np.cumsum(rowptr)
    col = (key % n).astype(np.int32)
    nonisolated = np.nonzero(np.diff(rowptr))[0]
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    for k, b in ((3, 9000), (7, 500)):
        batches = random_batches(n, k, b, rng, candidates=nonisolated)
        ref = O.sample_nodewise(rowptr, col, batches, (3, 3, 2), 5)
        for extract in ("sort", "buckets", "bitmap", None):
            res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (3, 3, 2), 5, extract=extract)
            assert_hops_equal(res.hops(), ref, what="extract=%s k=%d b=%d" % (extract, k, b))
    # repeated seed found by the LDS sort check (b <= 8192) and by the vertex-set check (b > 8192)
    for b in (500, 9000):
        bad = random_batches(n, 2, b, rng)
        bad[1, b - 1] = bad[1, 0]
        with pytest.raises(bms.BmsError) as e:
            bms.sample_nodewise(csr, bad, (2,), 1, extract="buckets")
        assert e.value.code == bms.ERANGE
    bad = random_batches(n, 2, 100, rng)
    bad[0, 7] = n
    with pytest.raises(bms.BmsError) as e:
        bms.sample_nodewise(csr, bad, (2,), 1, extract="buckets")
    assert e.value.code == bms.ERANGE


def test_sort_extract_falls_back_when_ids_crowd_one_segment(mods):
    # directed graph whose edges all point into a narrow id range: every sampled id of a minibatch lands in one
    # id-range segment, more than a segment may hold -> the per-minibatch kernel runs
    O, bms, _ = mods
    rng = np.random.default_rng(45)
    n, m = 1_000_000, 8_000_000
    src = rng.integers(0, n, size=m)
    dst = rng.integers(1030, 2000, size=m)     # narrower than any segment the library would pick
    key = np.unique(src * n + dst)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, key // n + 1, 1)
    rowptr = np.cumsum(rowptr)
    col = (key % n).astype(np.int32)
    sources = np.nonzero(np.diff(rowptr))[0]
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    batches = random_batches(n, 3, 12000, rng, candidates=sources)
    ref = O.sample_nodewise(rowptr, col, batches, (8, 2), 9)
    per_mb = np.diff(ref[0].rowptr[ref[0].mb_rowoff])
    assert per_mb.min() > 65535       # more pairs in the one segment than a segment may hold
    for extract in ("sort", "buckets", "bitmap"):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (8, 2), 9, extract=extract)
        assert_hops_equal(res.hops(), ref, what="extract=%s" % extract)


def test_recycled_calls_without_host_round_trips(mods):
    # a recycled result of the same call shape lets the library enqueue all hops without reading sizes
    # back; the second call here samples far more edges than the first (high-degree seeds), a third
    # far fewer, so buffers must be sized by upper bounds and not by the remembered sizes
    O, bms, _ = mods
    rng = np.random.default_rng(46)
    rowptr, col = random_csr(40000, 40.0, rng)
    deg = np.diff(rowptr)
    order = np.argsort(deg)
    low, high = order[:8000], order[-8000:]
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = None
    for pool, seed in ((low, 1), (high, 2), (low, 3), (high, 3)):
        batches = random_batches(40000, 6, 256, rng, candidates=pool)
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (10, 5, 3), seed, recycle=res)
        ref = O.sample_nodewise(rowptr, col, batches, (10, 5, 3), seed)
        assert_hops_equal(res.hops(), ref, what="recycled, seed %d" % seed)
    # an invalid batch on the no-round-trip path is still reported, and the handle recovers
    bad = random_batches(40000, 6, 256, rng)
    bad[2, 5] = bad[2, 6]
    with pytest.raises(bms.BmsError) as e:
        bms.sample_nodewise(csr, torch.from_numpy(bad).cuda(), (10, 5, 3), 4, recycle=res)
    assert e.value.code == bms.ERANGE
    good = random_batches(40000, 6, 256, rng)
    res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), (10, 5, 3), 5, recycle=res)
    assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, good, (10, 5, 3), 5))


def test_sort_extract_segments_sorted_by_whole_workgroups(mods):
    # most edges point into a few id-range segments, each of which then holds more pairs than one wave
    # sorts (but few enough for one workgroup); the rest spread over the whole id range, so that waves
    # and workgroups both feed the slot lists of the same minibatch
    O, bms, _ = mods
    rng = np.random.default_rng(47)
    n, m = 3_000_000, 900_000
    src = rng.integers(0, n, size=m)
    dst = np.where(rng.random(m) < 0.7, rng.integers(1 << 16, 4 << 16, size=m), rng.integers(0, n, size=m))
    key = np.unique(src * n + dst)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, key // n + 1, 1)
    rowptr = np.cumsum(rowptr)
    col = (key % n).astype(np.int32)
    sources = np.nonzero(np.diff(rowptr))[0]
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    batches = random_batches(n, 5, 8000, rng, candidates=sources)
    ref = O.sample_nodewise(rowptr, col, batches, (3, 2), 11)
    # sampled ids of minibatch 0 per range of 2^16 ids (the segment width the library picks for this shape)
    e1 = ref[0].rowptr[ref[0].mb_rowoff[1]]
    per_segment = np.bincount(ref[0].col_vertex[ref[0].col[:e1]] >> 16)
    assert 1024 < per_segment.max() <= 4096, per_segment.max()
    for extract in ("sort", None):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (3, 2), 11, extract=extract)
        assert_hops_equal(res.hops(), ref, what="extract=%s" % extract)


def test_sort_extract_largest_workgroup_sorted_segments(mods):
    # as above with most edges into ONE id range of 2^16: its segment holds several thousand pairs (several tiles
    # of the back-split per segment), ranked by a workgroup through a bitmap in LDS
    O, bms, _ = mods
    rng = np.random.default_rng(49)
    n, m = 3_000_000, 1_200_000
    src = rng.integers(0, n, size=m)
    dst = np.where(rng.random(m) < 0.7, rng.integers(1 << 16, 2 << 16, size=m), rng.integers(0, n, size=m))
    key = np.unique(src * n + dst)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr, key // n + 1, 1)
    rowptr = np.cumsum(rowptr)
    col = (key % n).astype(np.int32)
    sources = np.nonzero(np.diff(rowptr))[0]
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    batches = random_batches(n, 5, 8000, rng, candidates=sources)
    ref = O.sample_nodewise(rowptr, col, batches, (3, 2), 12)
    for i in range(5):
        e0, e1 = ref[0].rowptr[ref[0].mb_rowoff[i]], ref[0].rowptr[ref[0].mb_rowoff[i + 1]]
        per_segment = np.bincount(ref[0].col_vertex[ref[0].mb_coloff[i] + ref[0].col[e0:e1]] >> 16)
        assert 4096 < per_segment.max() <= 16384, per_segment.max()
    for extract in ("sort", None):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (3, 2), 12, extract=extract)
        assert_hops_equal(res.hops(), ref, what="extract=%s" % extract)


def test_vertex_ids_sorted_by_degree(mods):
    # hubs first: the sampled ids of every minibatch crowd the low end of the id range, so many id-range
    # segments hold far more pairs than a wave sorts and are ranked through LDS bitmaps, others stay small
    O, bms, _ = mods
    rng = np.random.default_rng(50)
    n = 400_000
    rowptr, col = skewed_csr(n, 6_000_000, rng)
    deg = np.diff(rowptr)
    order = np.argsort(-deg, kind="stable")
    newid = np.empty(n, dtype=np.int64)
    newid[order] = np.arange(n)
    src = np.repeat(np.arange(n), deg)
    key = np.sort(newid[src] * n + newid[col])
    rowptr2 = np.zeros(n + 1, dtype=np.int64)
    np.add.at(rowptr2, key // n + 1, 1)
    rowptr2 = np.cumsum(rowptr2)
    col2 = (key % n).astype(np.int32)
    batches = random_batches(n, 6, 2000, rng, candidates=np.nonzero(np.diff(rowptr2) > 0)[0])
    ref = O.sample_nodewise(rowptr2, col2, batches, (10, 5, 3), 13)
    e1 = ref[2].rowptr[ref[2].mb_rowoff[1]]
    first = ref[2].col_vertex[ref[2].col[:e1]]                  # global ids sampled by minibatch 0 at the last hop
    assert (first < n // 100).mean() > 0.08                      # ten times denser among the top 1 % of the ids
    assert np.bincount(first >> 9).max() > 2048                  # far more than a wave sorts, in ranges of 512 ids
    csr = bms.Csr(torch.from_numpy(rowptr2).cuda(), torch.from_numpy(col2).cuda())
    res = None
    for extract in ("sort", None, "buckets"):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (10, 5, 3), 13, extract=extract, recycle=res)
        assert_hops_equal(res.hops(), ref, what="degree-sorted ids, extract=%s" % extract)


def test_minibatch_with_more_sampled_edges_than_the_slot_lists_cover(mods):
    # one minibatch whose last hop samples more than 256 * 8192 edges: its local columns are stored
    # directly instead of through the per-range slot lists
    O, bms, synth = mods
    g = synth.rmat_graph(1 << 21, 24_000_000, 0.45, 0.22, 0.22, seed=5, device="cuda")
    rowptr, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    rng = np.random.default_rng(48)
    deg = np.diff(rowptr)
    batches = random_batches(g.n, 2, 8000, rng, candidates=np.nonzero(deg >= 8)[0])
    csr = bms.Csr(g.rowptr, g.col)
    ref = O.sample_nodewise(rowptr, col, batches, (15, 10, 5), 3)
    per_mb = np.diff(ref[2].rowptr[ref[2].mb_rowoff])
    assert per_mb.max() > 256 * 8192, per_mb
    res = None
    for extract in ("sort", "buckets", "sort"):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (15, 10, 5), 3, extract=extract, recycle=res)
        assert_hops_equal(res.hops(), ref, what="extract=%s" % extract)


def test_thousands_of_small_minibatches_and_the_limit_on_k(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(49)
    rowptr, col = random_csr(60000, 9.0, rng)
    batches = random_batches(60000, 3000, 4, rng)
    csr, res, ref = _run_both(mods, rowptr, col, batches, (4, 3), 8)
    lad = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), (6, 6), 8)
    assert_hops_equal(lad.hops(), O.sample_ladies(rowptr, col, batches, (6, 6), 8), with_p=True)
    with pytest.raises(bms.BmsError) as e:
        bms.sample_nodewise(csr, torch.zeros((65536, 1), dtype=torch.int32).cuda(), (2,), 1)
    assert e.value.code == bms.EINVAL


def test_side_stream_and_graph_without_vertices(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(50)
    rowptr, col = random_csr(20000, 10.0, rng)
    batches = random_batches(20000, 6, 100, rng)
    ref = O.sample_nodewise(rowptr, col, batches, (6, 4), 2)
    lref = O.sample_ladies(rowptr, col, batches, (50, 50), 2)
    side = torch.cuda.Stream()  # default priority
    with torch.cuda.stream(side):
        csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
        dev = torch.from_numpy(batches).cuda()
        res = None
        for _ in range(3):
            res = bms.sample_nodewise(csr, dev, (6, 4), 2, recycle=res)
        lad = bms.sample_ladies(csr, dev, (50, 50), 2)
        X = bms.fetch_features(torch.ones((20000, 8), device="cuda"), res.hop(1).col_vertex)
        Y = bms.aggregate_hop(res, 1, X)
    side.synchronize()
    assert_hops_equal(res.hops(), ref, what="side stream")
    assert_hops_equal(lad.hops(), lref, with_p=True, what="side stream")
    assert torch.equal(Y.cpu(), (torch.from_numpy(np.diff(ref[1].rowptr)) > 0).float()[:, None].repeat(1, 8))
    # a matrix with no vertices loads; every seed is then out of range
    empty = bms.Csr(torch.zeros(1, dtype=torch.int64).cuda(), torch.zeros(0, dtype=torch.int32).cuda())
    for fn in (bms.sample_nodewise, bms.sample_ladies):
        with pytest.raises(bms.BmsError) as e:
            fn(empty, np.zeros((1, 1), dtype=np.int32), (2,), 1)
        assert e.value.code == bms.ERANGE


def _hub_graph(n, hub_share, rng):
    """Directed graph: every vertex points at one random vertex, and a share of them also at one hub."""
    hub = 12345
    dst = rng.integers(0, n, size=n)
    dst[dst == np.arange(n)] = (dst[dst == np.arange(n)] + 1) % n
    has_hub = rng.random(n) < hub_share
    has_hub[hub] = False
    has_hub &= dst != hub
    deg = 1 + has_hub.astype(np.int64)
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(deg)
    col = np.empty(rowptr[-1], dtype=np.int32)
    first = np.where(has_hub, np.minimum(dst, hub), dst)
    col[rowptr[:-1]] = first
    col[rowptr[:-1][has_hub] + 1] = np.maximum(dst, hub)[has_hub]
    return rowptr, col, hub


@pytest.mark.parametrize("b,hub_share,what", [
    (16000, 0.02, "one id in more than 32 rows of a segment that one workgroup ranks: handed to the bitmap kernel"),
    (16000, 0.6, "the hub's segment holds more ids than one workgroup ranks: listed for the bitmap kernel"),
    (900, 0.2, "segments wider than the bitmap kernel takes: the per-minibatch kernel redoes the hop"),
])
def test_sort_extract_one_vertex_sampled_by_many_rows(mods, b, hub_share, what):
    # sparse hop (far fewer sampled ids than vertices): the ids of a segment are ranked by counting them into buckets
    # of about one id; a hub that many rows of a minibatch sample crowds one bucket
    O, bms, _ = mods
    rng = np.random.default_rng(51)
    n = 1 << 22
    rowptr, col, hub = _hub_graph(n, hub_share, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    batches = random_batches(n, 3, b, rng)
    ref = O.sample_nodewise(rowptr, col, batches, (2, 1), 21)
    picked = ref[0].col_vertex[ref[0].col[:ref[0].rowptr[ref[0].mb_rowoff[1]]]]
    assert (picked == hub).sum() > 32, what
    for extract in ("sort", None, "buckets"):
        res = None
        for _ in range(2):   # the second call runs without host round trips
            res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (2, 1), 21, extract=extract, recycle=res)
            assert_hops_equal(res.hops(), ref, what="%s, extract=%s" % (what, extract))


def test_sort_extract_dense_hops_ranked_by_bitmap_with_many_duplicates(mods):
    # dense hop (a minibatch samples a large share of the vertices): every segment is ranked through a bitmap of
    # its id range; most ids are sampled several times, segments hold tens of thousands of ids
    O, bms, _ = mods
    rng = np.random.default_rng(52)
    n = 60000
    rowptr, col = random_csr(n, 30.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    batches = random_batches(n, 4, 6000, rng)
    ref = O.sample_nodewise(rowptr, col, batches, (8, 4), 22)
    assert ref[1].nnz / 4 > 50000 and ref[1].nnz > 2 * ref[1].ncols
    for extract in ("sort", None):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (8, 4), 22, extract=extract)
        assert_hops_equal(res.hops(), ref, what="extract=%s" % extract)


@pytest.mark.parametrize("b", [1023, 1024, 1025, 2048, 3072])
def test_sort_extract_minibatches_that_fill_tiles_of_the_cut_exactly(mods, b):
    # every vertex has 10 neighbours, fanout 8: a minibatch samples exactly 8 b ids, i.e. one short of, exactly, or
    # one more than whole tiles of 8192 positions of the cut; the second hop (fanout 2) does the same on distinct ids
    O, bms, _ = mods
    n = 150_000
    v = np.arange(n, dtype=np.int64)
    nb = np.stack([(v + d) % n for d in (-5, -4, -3, -2, -1, 1, 2, 3, 4, 5)], axis=1)
    nb.sort(axis=1)
    rowptr = np.arange(n + 1, dtype=np.int64) * 10
    col = nb.reshape(-1).astype(np.int32)
    rng = np.random.default_rng(b)
    batches = random_batches(n, 3, b, rng)
    ref = O.sample_nodewise(rowptr, col, batches, (8, 2), 31)
    assert ref[0].nnz == 3 * 8 * b
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    res = None
    for _ in range(2):
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (8, 2), 31, extract="sort", recycle=res)
        assert_hops_equal(res.hops(), ref, what="b=%d" % b)
