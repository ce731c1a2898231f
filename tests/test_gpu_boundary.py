"""The boundary's two steady-state features, through the C ABI: a caller's allocator for the result buffers, and
asynchronous calls (BMS_ASYNC) whose sizes, errors and times are read when the result is first looked at."""
import time

import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr
from parity import assert_hops_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    assert torch.cuda.is_available()
    return O, bms


def test_result_buffers_come_from_the_callers_allocator(mods):
    O, bms = mods
    rng = np.random.default_rng(80)
    n = 40000
    rowptr, col = random_csr(n, 14.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    al = bms.TorchAllocator()
    batches = random_batches(n, 6, 400, rng)
    res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (8, 4, 3), 5, allocator=al)
    ref = O.sample_nodewise(rowptr, col, batches, (8, 4, 3), 5)
    assert_hops_equal(res.hops(), ref, what="allocator")
    assert al.calls >= 3 * 4 and len(al.live) >= 3 * 4   # at least rowptr, col, mb_coloff, col_vertex per hop
    for hop in res.hops():                                # every exposed pointer lies inside a tensor the allocator gave
        for t in (hop.rowptr, hop.col, hop.mb_coloff, hop.col_vertex, hop.mb_rowoff, hop.row_vertex):
            if t.numel():
                p = t.data_ptr()
                assert any(base <= p < base + buf.numel() for base, buf in al.live.items())
    # recycled with a larger call: buffers grow through the same allocator; the union_dst variant adds row_self
    big = random_batches(n, 6, 800, rng)
    res = bms.sample_nodewise(csr, torch.from_numpy(big).cuda(), (8, 4, 3), 6, recycle=res, union_dst=True)
    assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, big, (8, 4, 3), 6, union_dst=True), what="regrown")
    lad = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), (64, 32), 7, allocator=al)
    assert_hops_equal(lad.hops(), O.sample_ladies(rowptr, col, batches, (64, 32), 7), with_p=True, what="ladies")
    res.free()
    lad.free()
    assert len(al.live) == 0, "buffers not returned: %d" % len(al.live)
    # an allocator that runs dry is an error code, not a crash
    dry = bms.TorchAllocator()
    dry.alloc = bms.ALLOC_FN(lambda nbytes, ctx: None)
    with pytest.raises(bms.BmsError) as e:
        bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (8, 4, 3), 5, allocator=dry)
    assert e.value.code == bms.ENOMEM


def test_async_calls_overlap_with_the_consumers_of_the_previous_bulk(mods):
    # Sec. 6 of the paper trains on the minibatches of one bulk while the next bulk is sampled.  Two results, two
    # streams: bulk j + 1 is sampled asynchronously on one stream while bulk j's features are fetched and
    # aggregated on the other; every bulk is checked against the oracle.
    O, bms = mods
    rng = np.random.default_rng(81)
    n, k, b, fan, f = 400_000, 32, 512, (10, 8, 4), 32
    rowptr, col = random_csr(n, 20.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    H = torch.randint(0, 100, (n, f), device="cuda").float()
    bulks = [random_batches(n, k, b, rng) for _ in range(6)]
    dev = [torch.from_numpy(x).cuda() for x in bulks]
    sample_stream, train_stream = torch.cuda.Stream(), torch.cuda.Stream()
    results = [None, None]
    for j in range(2):      # the first two calls of a shape are synchronous: they size the buffers
        results[j] = bms.sample_nodewise(csr, dev[j], fan, 100 + j, stream=sample_stream.cuda_stream)
        results[j] = bms.sample_nodewise(csr, dev[j], fan, 100 + j, stream=sample_stream.cuda_stream, recycle=results[j])
    t0 = time.perf_counter()
    bms.sample_nodewise(csr, dev[1], fan, 101, stream=sample_stream.cuda_stream, recycle=results[1])
    t_sync = time.perf_counter() - t0
    returned_early = 0
    t_async = []
    outs = {}
    for j in range(1, 6):
        # sample bulk j into the buffer that bulk j - 2 no longer needs, then consume bulk j - 1 meanwhile
        t0 = time.perf_counter()
        cur = bms.sample_nodewise(csr, dev[j], fan, 100 + j, stream=sample_stream.cuda_stream, recycle=results[j % 2],
                                  async_=True)
        t_async.append(time.perf_counter() - t0)
        returned_early += 0 if cur.ready() else 1
        prev = results[(j - 1) % 2]
        if j > 1:
            last = prev.hop(len(fan) - 1)            # first look at bulk j - 1: waits for it, not for bulk j
            X = bms.fetch_features(H, last.col_vertex, stream=train_stream.cuda_stream)
            outs[j - 1] = (bms.aggregate_hop(prev, len(fan) - 1, X, mean=False, stream=train_stream.cuda_stream),
                           [h.to_host() for h in prev.hops()])
        results[j % 2] = cur
    results[5 % 2].wait()
    train_stream.synchronize()
    outs[5] = (None, [h.to_host() for h in results[1].hops()])
    for j in range(1, 6):
        ref = O.sample_nodewise(rowptr, col, bulks[j], fan, 100 + j)
        agg, hops = outs[j]
        assert_hops_equal(hops, ref, what="bulk %d" % j)
        if agg is not None:
            want = O.aggregate(ref[-1], O.fetch_features(H.cpu().numpy(), ref[-1].col_vertex), mean=False)
            assert np.array_equal(agg.cpu().numpy(), want), "aggregation of bulk %d" % j
    print("sync call %.3f ms, async calls returned after %s ms, %d of 5 before their kernels had finished"
          % (t_sync * 1e3, ["%.3f" % (t * 1e3) for t in t_async], returned_early), flush=True)
    assert returned_early >= 1, "no asynchronous call returned before its kernels had finished"


def test_async_errors_arrive_with_the_first_look_at_the_result(mods):
    O, bms = mods
    rng = np.random.default_rng(82)
    n = 60000
    rowptr, col = random_csr(n, 12.0, rng)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    fan = (6, 4)
    good = random_batches(n, 5, 300, rng)
    res = None
    for seed in (1, 2):
        res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), fan, seed, recycle=res)
    bad = good.copy()
    bad[2, 9] = n + 5
    res = bms.sample_nodewise(csr, torch.from_numpy(bad).cuda(), fan, 3, recycle=res, async_=True)   # returns OK
    with pytest.raises(bms.BmsError) as e:
        res.wait()
    assert e.value.code == bms.ERANGE
    with pytest.raises(bms.BmsError) as e:
        res.hop(0)                       # the result is empty now
    assert e.value.code == bms.EINVAL
    for seed in (4, 5, 6):               # recovers; the third call is asynchronous again
        res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), fan, seed, recycle=res, async_=seed == 6)
        assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, good, fan, seed), what="seed %d" % seed)
    # a pending result may be recycled or freed without having been looked at
    res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), fan, 7, recycle=res, async_=True)
    res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), fan, 8, recycle=res, async_=True)
    assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, good, fan, 8), what="recycled while pending")
    res = bms.sample_nodewise(csr, torch.from_numpy(good).cuda(), fan, 9, recycle=res, async_=True)
    res.free()


def test_async_call_that_meets_crowded_ids_asks_to_be_repeated(mods):
    # the remembered shape ran on segments of equal width; the asynchronous call then samples a hub from many rows,
    # which that path cannot rank: BMS_EAGAIN at the first look, and the repeated call takes the next path
    O, bms = mods
    from test_gpu_nodewise import _hub_graph
    rng = np.random.default_rng(83)
    n = 1 << 22
    rowptr, col, hub = _hub_graph(n, 0.2, rng)
    deg = np.diff(rowptr)
    plain, with_hub = np.nonzero(deg == 1)[0], np.nonzero(deg == 2)[0]
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    fan = (2, 1)
    calm = random_batches(n, 3, 900, rng, candidates=plain)
    res = None
    for seed in (1, 2):
        res = bms.sample_nodewise(csr, torch.from_numpy(calm).cuda(), fan, seed, recycle=res, extract="sort")
        assert_hops_equal(res.hops(), O.sample_nodewise(rowptr, col, calm, fan, seed))
    crowded = random_batches(n, 3, 900, rng, candidates=with_hub)
    res = bms.sample_nodewise(csr, torch.from_numpy(crowded).cuda(), fan, 3, recycle=res, extract="sort", async_=True)
    with pytest.raises(bms.BmsError) as e:
        res.wait()
    assert e.value.code == bms.EAGAIN
    ref = O.sample_nodewise(rowptr, col, crowded, fan, 3)
    for attempt in range(3):   # repeated (asynchronously even): each attempt moves the hop one path on
        res = bms.sample_nodewise(csr, torch.from_numpy(crowded).cuda(), fan, 3, recycle=res, extract="sort", async_=True)
        try:
            res.wait()
            break
        except bms.BmsError as err:
            assert err.code == bms.EAGAIN and attempt < 2
    assert_hops_equal(res.hops(), ref, what="after the repeat")
