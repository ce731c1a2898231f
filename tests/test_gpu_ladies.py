"""Parity of the HIP layer-wise (LADIES) sampler with the CPU oracle (bit-exact), through the C ABI."""
import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr
from parity import assert_hops_equal

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mods():
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    assert torch.cuda.is_available()
    return O, bms, synth


def _run_both(mods, rowptr, col, batches, s_per_layer, seed, mb_base=0, squared=False, csr=None):
    O, bms, _ = mods
    if csr is None:
        csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    ref = O.sample_ladies(rowptr, col, batches, s_per_layer, seed, mb_base, squared)
    # the kernel paths: counters in HBM; counters in LDS windows, the rows' window boundaries found per hop;
    # the same with the boundaries copied from the per-graph index (built by the first call that may use it)
    for dense, index in ((True, True), (False, False), (False, True)):
        res = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), s_per_layer, seed, mb_base=mb_base,
                                squared=squared, dense=dense, index=index)
        assert_hops_equal(res.hops(), ref, with_p=True,
                          what="s=%s seed=%d squared=%s dense=%s index=%s" % (s_per_layer, seed, squared, dense, index))
    return csr, res, ref


def test_tiny_graph_layerwise(mods):
    O, bms, synth = mods
    g, batches, _ = synth.make_workload("tiny_sage")
    _run_both(mods, g.rowptr.numpy(), g.col.numpy(), batches.numpy(), (64, 64), synth.SAMPLING_SEED)


@pytest.mark.parametrize("s,squared", [((1,), False), ((16, 16), False), ((100, 50, 25), False), ((512, 512, 512), False),
                                       ((64, 64), True), ((3000, 10), True), ((4096, 4097, 5), False)])
def test_random_graph(mods, s, squared):
    # gathered order spans many 4096-entry tiles with a ragged tail; P spans several chunks and tiles
    rng = np.random.default_rng(len(s) * 100 + s[0])
    rowptr, col = random_csr(30000, 30.0, rng)
    batches = random_batches(30000, 5, 200, rng)
    _run_both(mods, rowptr, col, batches, s, 17, mb_base=2, squared=squared)


@pytest.mark.parametrize("s,squared", [((400, 300, 200), False), ((2000, 50), True)])
def test_many_id_windows(mods, s, squared):
    # vertex ids span several 2^16-id windows; a skewed graph, so hub rows cross every window and
    # leaf rows cross none
    O, bms, synth = mods
    g = synth.rmat_graph(300_000, 2_000_000, 0.55, 0.2, 0.2, seed=9, device="cuda")
    rowptr, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    rng = np.random.default_rng(s[0])
    batches = random_batches(g.n, 6, 300, rng)
    _run_both(mods, rowptr, col, batches, s, 23, mb_base=1, squared=squared, csr=bms.Csr(g.rowptr, g.col))


def test_directed_with_loops_and_host_inputs(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(31)
    rowptr, col = random_csr(5000, 9.0, rng, symmetric=False, allow_loops=True)
    batches = random_batches(5000, 6, 40, rng)
    csr = bms.Csr(torch.from_numpy(rowptr), torch.from_numpy(col))
    res = bms.sample_ladies(csr, batches, (30, 30), 21)
    assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, batches, (30, 30), 21), with_p=True)


def test_bulk_equals_stack_recycle_and_mixed_calls(mods):
    O, bms, _ = mods
    rng = np.random.default_rng(32)
    rowptr, col = random_csr(8000, 16.0, rng)
    batches = random_batches(8000, 4, 64, rng)
    csr, bulk, ref = _run_both(mods, rowptr, col, batches, (40, 40), 5, mb_base=9)
    res = None
    for i in range(4):
        res = bms.sample_ladies(csr, torch.from_numpy(batches[i:i + 1]).cuda(), (40, 40), 5, mb_base=9 + i, recycle=res)
        assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, batches[i:i + 1], (40, 40), 5, 9 + i), with_p=True)
    # node-wise and layer-wise calls share the handle's vertex sets: interleave them
    nw = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), (5, 5), 3)
    assert_hops_equal(nw.hops(), O.sample_nodewise(rowptr, col, batches, (5, 5), 3))
    _run_both(mods, rowptr, col, batches, (40, 40), 6, csr=csr)


def test_degenerate_inputs_and_errors(mods):
    O, bms, _ = mods
    rowptr = np.array([0, 0, 0, 1, 2], dtype=np.int64)
    col = np.array([3, 2], dtype=np.int32)
    _run_both(mods, rowptr, col, np.array([[0, 1], [2, 0]], dtype=np.int32), (2, 2, 2), 1)
    _run_both(mods, np.zeros(6, dtype=np.int64), np.zeros(0, dtype=np.int32), np.array([[1, 2]], dtype=np.int32),
              (3, 3), 1)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    for bad in (np.array([[1, 1]], dtype=np.int32), np.array([[0, 4]], dtype=np.int32)):
        with pytest.raises(bms.BmsError) as e:
            bms.sample_ladies(csr, bad, (2,), 1)
        assert e.value.code == bms.ERANGE
    _run_both(mods, rowptr, col, np.array([[3, 2]], dtype=np.int32), (1,), 1, csr=csr)
    with pytest.raises(bms.BmsError) as e:
        bms.sample_ladies(csr, np.array([[3, 2]], dtype=np.int32), (1,), 1, scratch_limit=8)
    assert e.value.code == bms.ENOMEM


def test_paper_worked_example_on_the_gpu(mods):
    # Sec. 2.2: batch {1,5}; e = [1,0,1,1,2,0]; with squared weights the array is [1,0,1,1,4,0]/7
    O, bms, _ = mods
    edges = [(0, 1), (2, 1), (3, 5), (4, 1), (4, 5)]
    A = np.zeros((6, 6), dtype=np.int64)
    for u, v in edges:
        A[u, v] = A[v, u] = 1
    rowptr = np.concatenate([[0], np.cumsum(A.sum(axis=1))]).astype(np.int64)
    col = np.concatenate([np.nonzero(A[v])[0] for v in range(6)]).astype(np.int32)
    batch = np.array([[1, 5]], dtype=np.int32)
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    for seed in range(20):
        res = bms.sample_ladies(csr, batch, (2,), seed, squared=True)
        hop = res.hop(0).to_host()
        e = np.zeros(6, dtype=np.int64)
        e[hop.p_col] = hop.p_cnt
        assert e.tolist() == [1, 0, 1, 1, 2, 0]
        assert_hops_equal([hop], O.sample_ladies(rowptr, col, batch, (2,), seed, squared=True), with_p=True)


@pytest.mark.parametrize("b", [8192, 9000])
def test_largest_batches_of_each_kernel_path(mods, b):
    # b = 8192 is the most the LDS-window path takes (seed check by an LDS sort, 16-bit counters); larger batches
    # run on the dense-counter path by themselves
    O, bms, synth = mods
    g = synth.rmat_graph(120_000, 700_000, 0.5, 0.2, 0.2, seed=11, device="cuda")
    rowptr, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    rng = np.random.default_rng(b)
    batches = random_batches(g.n, 2, b, rng)
    ref = O.sample_ladies(rowptr, col, batches, (300, 100), 4)
    res = bms.sample_ladies(bms.Csr(g.rowptr, g.col), torch.from_numpy(batches).cuda(), (300, 100), 4)
    assert_hops_equal(res.hops(), ref, with_p=True, what="b=%d" % b)


def test_window_index_is_built_once_when_it_fits_and_left_out_when_it_does_not(mods):
    # the index of where adjacency lists cross the window boundaries: n * (windows + 1) 32-bit words held by the
    # handle after the first call that may build it; not built under BMS_LADIES_NO_INDEX, with a scratch limit
    # whose quarter it exceeds, or for a graph whose column array is less than half its size; same results always
    O, bms, synth = mods
    g = synth.rmat_graph(300_000, 2_000_000, 0.55, 0.2, 0.2, seed=5, device="cuda")
    rowptr, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    rng = np.random.default_rng(77)
    batches = random_batches(g.n, 4, 200, rng)
    s = (150, 100)
    ref = O.sample_ladies(rowptr, col, batches, s, 8)
    index_bytes = g.n * ((g.n + 65535) // 65536 + 1) * 4
    dev_batches = torch.from_numpy(batches).cuda()

    csr = bms.Csr(g.rowptr, g.col)
    res = bms.sample_ladies(csr, dev_batches, s, 8, index=False)
    assert_hops_equal(res.hops(), ref, with_p=True, what="no index")
    without = csr.held_bytes()
    res = bms.sample_ladies(csr, dev_batches, s, 8)
    assert_hops_equal(res.hops(), ref, with_p=True, what="index built by this call")
    held = csr.held_bytes()
    assert held >= without + index_bytes - (g.n * 6 * 4) // 2  # the per-hop lists shrink to half without their row-major copy
    res = bms.sample_ladies(csr, dev_batches, s, 8, recycle=res)
    assert_hops_equal(res.hops(), ref, with_p=True, what="index reused")
    assert held <= csr.held_bytes() < held + index_bytes  # (scratch sized with a margin by the recycled call, no second index)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        res = bms.sample_ladies(csr, dev_batches, s, 9, stream=stream.cuda_stream)
    assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, batches, s, 9), with_p=True, what="index on another stream")

    small = bms.Csr(g.rowptr, g.col)
    res = bms.sample_ladies(small, dev_batches, s, 8, scratch_limit=3 * index_bytes)
    assert_hops_equal(res.hops(), ref, with_p=True, what="scratch limit of three times the index")
    assert small.held_bytes() < index_bytes + without

    # average degree 0.5: the index would be four times the column array
    rng = np.random.default_rng(78)
    rp, cl = random_csr(70_000, 0.5, rng)
    bt = random_batches(70_000, 3, 100, rng)
    sparse = bms.Csr(torch.from_numpy(rp).cuda(), torch.from_numpy(cl).cuda())
    res = bms.sample_ladies(sparse, torch.from_numpy(bt).cuda(), (50, 50), 3)
    assert_hops_equal(res.hops(), O.sample_ladies(rp, cl, bt, (50, 50), 3), with_p=True, what="sparse graph")
    plain = bms.Csr(torch.from_numpy(rp).cuda(), torch.from_numpy(cl).cuda())
    bms.sample_ladies(plain, torch.from_numpy(bt).cuda(), (50, 50), 3, index=False)
    assert sparse.held_bytes() == plain.held_bytes()


def test_recycled_calls_without_size_read_backs_and_their_fallback(mods):
    # a recycled result remembers what its call shape needed (gathered neighbours, nnz(P), kept neighbours per hop):
    # the next call of that shape sizes its buffers from it and checks on the device; when the new seeds need more
    # (hubs instead of leaves) the device flag goes up and the call is repeated with read-backs.  Same results.
    O, bms, synth = mods
    g = synth.rmat_graph(200_000, 3_000_000, 0.57, 0.19, 0.19, seed=21, device="cuda")
    rowptr, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    deg = np.diff(rowptr)
    order = np.argsort(deg, kind="stable")
    k, b, s = 4, 128, (96, 64)
    leaves = order[deg[order] > 0][:k * b].astype(np.int32).reshape(k, b)
    hubs = order[-k * b:].astype(np.int32).reshape(k, b)
    rng = np.random.default_rng(5)
    mixed = random_batches(g.n, k, b, rng)
    csr = bms.Csr(g.rowptr, g.col)
    res = None
    attempts = []
    for step, (batches, seed) in enumerate([(leaves, 1), (leaves, 2), (mixed, 3), (hubs, 4), (hubs, 5), (leaves, 6)]):
        res = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), s, seed, recycle=res)
        attempts.append(res.attempts())
        assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, batches, s, seed), with_p=True, what="step %d" % step)
    # leaves gather a few hundred neighbours at the first hop, hubs far more than the margin over that allows: that
    # call repeats itself; the same seeds again then fit what is remembered
    assert attempts[0] == 1 and attempts[1] == 1 and attempts[3] == 2 and attempts[4] == 1, attempts
    assert set(attempts) <= {1, 2}
    # errors on the path without read-backs arrive at the end of the call; the handle recovers
    bad = leaves.copy()
    bad[1, 3] = g.n
    with pytest.raises(bms.BmsError) as e:
        bms.sample_ladies(csr, torch.from_numpy(bad).cuda(), s, 7, recycle=res)
    assert e.value.code == bms.ERANGE
    res = bms.sample_ladies(csr, torch.from_numpy(hubs).cuda(), s, 8)
    res = bms.sample_ladies(csr, torch.from_numpy(hubs).cuda(), s, 9, recycle=res)
    assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, hubs, s, 9), with_p=True, what="after the error")
    # another shape on the same result: nothing remembered applies
    res = bms.sample_ladies(csr, torch.from_numpy(hubs[:2]).cuda(), s, 10, recycle=res)
    assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, hubs[:2], s, 10), with_p=True, what="other shape")


def test_shapes_around_the_window_and_part_boundaries(mods):
    # vertex counts just below, at and above one and two id windows (2^16); one seed per minibatch; one draw;
    # as many draws as the LDS path takes; recycled calls (sizes remembered) in between
    rng = np.random.default_rng(99)
    cases = [(65535, 3, 7, (5, 3)), (65536, 2, 1, (1, 1, 1)), (65537, 4, 33, (64, 1)), (131071, 1, 50, (200,)),
             (131072, 5, 20, (4096, 17)), (131073, 2, 64, (100, 100, 100)), (4097, 3, 16, (33, 9)), (70, 2, 5, (4, 4))]
    for n, k, b, s in cases:
        rowptr, col = random_csr(n, 12.0, rng)
        batches = random_batches(n, k, b, rng)
        csr, res, _ = _run_both(mods, rowptr, col, batches, s, 40 + k, mb_base=k, squared=bool(b & 1))
        O, bms, _ = mods
        for seed in (1, 2):
            res = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), s, seed, squared=bool(b & 1), recycle=res)
            assert_hops_equal(res.hops(), O.sample_ladies(rowptr, col, batches, s, seed, 0, bool(b & 1)), with_p=True,
                              what="n=%d k=%d b=%d s=%s seed=%d" % (n, k, b, s, seed))
