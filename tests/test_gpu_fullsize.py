"""Full-size parity: the six benchmark workloads, generated on the GPU exactly as bench.py does,
sampled through the C ABI in bench.py's launch configuration and compared with the oracle on every
array of every hop (bit-exact).  The oracle runs the complete workload (seconds on the host cores)."""
import time

import pytest
import torch

from parity import assert_hops_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny_sage", "mid_sage", "mid_ladies", "large_sage", "dense_sage", "dense_ladies"])
def test_workload_matches_oracle(name):
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    t0 = time.time()
    g, batches, w = synth.make_workload(name, device="cuda")
    print("\n%s: %s (%.1f s)" % (name, g.describe(), time.time() - t0), flush=True)
    target = {"tiny_sage": 2.0e5, "mid_sage": 1.237e8, "mid_ladies": 1.237e8, "large_sage": 1.6e9,
              "dense_sage": 1.3e9, "dense_ladies": 1.3e9}[name]
    assert abs(g.nnz - target) <= 0.05 * target
    csr = bms.Csr(g.rowptr, g.col)
    nodewise = w["sampler"] == "nodewise"
    fn = bms.sample_nodewise if nodewise else bms.sample_ladies
    res = fn(csr, batches, w["params"], synth.SAMPLING_SEED, profile=True)
    res = fn(csr, batches, w["params"], synth.SAMPLING_SEED, recycle=res, profile=True)   # steady state, as timed
    print("  sizes", res.sizes(), flush=True)
    rp, cl, bt = g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy()
    del g
    torch.cuda.empty_cache()
    t0 = time.time()
    ofn = O.sample_nodewise if nodewise else O.sample_ladies
    ref = ofn(rp, cl, bt, w["params"], synth.SAMPLING_SEED)
    print("  oracle %.1f s on %d threads" % (time.time() - t0, O.set_threads(0)), flush=True)
    assert_hops_equal(res.hops(), ref, with_p=not nodewise, what=name)
    # properties that hold at any size
    for h, hop in enumerate(ref):
        assert hop.rows <= w["k"] * w["batch"] * (1 if h == 0 else max(w["params"][:h]) ** h * 10**6)
        if not nodewise:
            assert ((hop.mb_coloff[1:] - hop.mb_coloff[:-1]) <= w["params"][h]).all()


@pytest.mark.parametrize("name", ["mid_sage", "large_sage"])
def test_workload_with_ids_sorted_by_degree_matches_oracle(name):
    """The same graphs with their vertices renumbered hubs first: the sampled ids of every minibatch crowd the low end
    of the id range, EXTRACT falls back from segments of equal width to segments dealt by a table (built in the
    first call, reused by the recycled ones).  Three calls: the one that finds out, the one that builds the table,
    and steady state."""
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    g, batches, w = synth.make_workload(name, device="cuda", relabel="degree")
    deg = g.rowptr[1:] - g.rowptr[:-1]
    assert bool((deg[:-1] >= deg[1:]).all())
    csr = bms.Csr(g.rowptr, g.col)
    rp, cl, bt = g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy()
    ref = O.sample_nodewise(rp, cl, bt, w["params"], synth.SAMPLING_SEED)
    res = None
    attempts = []
    for call in range(3):
        res = bms.sample_nodewise(csr, batches, w["params"], synth.SAMPLING_SEED, recycle=res, profile=True)
        attempts.append(res.attempts())
        assert_hops_equal(res.hops(), ref, what="%s by degree, call %d" % (name, call))
    assert attempts[0] > 1 and attempts[2] == 1, attempts  # the first call repeats itself, the steady state does not
    stages = {s for s, _, _ in res.stages()}
    assert "dd_unsplit" in stages, "no hop of the steady-state call went through the segment kernels: %s" % sorted(stages)
    # other batches of the same split keep using the table
    other = synth.train_batches(g.n, w["frac"], 8, w["batch"], synth.SPLIT_SEED, "cuda", first=w["k"]) \
        if name == "mid_sage" else None
    if other is not None:
        r2 = bms.sample_nodewise(csr, other, w["params"], 7)
        assert_hops_equal(r2.hops(), O.sample_nodewise(rp, cl, other.cpu().numpy(), w["params"], 7), what="other batches")


def test_fetch_and_aggregate_at_full_size_on_sampled_outputs():
    """The two consumer steps on the mid-size node-wise workload at its real shape (f = 100 as in Table 3),
    in the launch configuration bench.py times; checked on outputs the oracle computes one by one:
    100 000 random fetched rows, and every aggregated row of three whole minibatches."""
    import numpy as np
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    g, batches, w = synth.make_workload("mid_sage", device="cuda")
    f = w["features"]
    csr = bms.Csr(g.rowptr, g.col)
    res = bms.sample_nodewise(csr, batches, w["params"], synth.SAMPLING_SEED)
    last_h = len(w["params"]) - 1
    last = res.hop(last_h)
    gen = torch.Generator(device="cuda").manual_seed(7)
    H = torch.randn((g.n, f), dtype=torch.float32, device="cuda", generator=gen)
    X = bms.fetch_features(H, last.col_vertex)
    assert X.shape == (last.ncols, f)
    # every expected value below comes from the oracle's own sample of the same workload
    ref_last = O.sample_nodewise(g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy(), w["params"],
                                 synth.SAMPLING_SEED)[last_h]
    rng = np.random.default_rng(1)
    sel = np.sort(rng.integers(0, ref_last.ncols, size=100_000))
    Hh = H.cpu().numpy()
    got = X[torch.from_numpy(sel).cuda()].cpu().numpy()
    assert np.array_equal(got.view(np.uint32), O.fetch_features(Hh, ref_last.col_vertex[sel]).view(np.uint32))
    out = bms.aggregate_hop(res, last_h, X, mean=True)
    assert out.shape == (ref_last.rows, f)
    hop = ref_last
    u = 2.0 ** -24
    for i in (0, w["k"] // 2, w["k"] - 1):
        r0, r1 = int(hop.mb_rowoff[i]), int(hop.mb_rowoff[i + 1])
        c0, c1 = int(hop.mb_coloff[i]), int(hop.mb_coloff[i + 1])
        e0, e1 = int(hop.rowptr[r0]), int(hop.rowptr[r1])
        sub = O.Hop(rows=r1 - r0, nnz=e1 - e0, ncols=c1 - c0, mb_rowoff=np.array([0, r1 - r0], dtype=np.int64),
                    row_vertex=hop.row_vertex[r0:r1], rowptr=hop.rowptr[r0:r1 + 1] - e0, col=hop.col[e0:e1],
                    mb_coloff=np.array([0, c1 - c0], dtype=np.int64), col_vertex=hop.col_vertex[c0:c1])
        Xi = O.fetch_features(Hh, hop.col_vertex[c0:c1])
        ref = O.aggregate(sub, Xi, mean=True).astype(np.float64)
        m = np.diff(sub.rowptr).astype(np.float64)[:, None]
        bound = (m + 2) * u * O.aggregate(sub, np.abs(Xi), mean=False).astype(np.float64) / np.maximum(m, 1.0) * 1.0001
        err = np.abs(out[r0:r1].cpu().numpy().astype(np.float64) - ref)
        assert np.all(err <= bound), (i, float(err.max()))


def test_layerwise_on_the_largest_graph():
    """LADIES on the 111 M-vertex graph (1 694 id windows per minibatch, most of them empty; dense per-minibatch
    counters would not fit in the scratch limit there), against the complete oracle result."""
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms, synth
    g, batches, w = synth.make_workload("large_sage", device="cuda")
    batches = batches[:16, :512].contiguous()
    csr = bms.Csr(g.rowptr, g.col)
    s = (512, 256, 128)
    res = bms.sample_ladies(csr, batches, s, synth.SAMPLING_SEED, mb_base=3)
    res = bms.sample_ladies(csr, batches, s, synth.SAMPLING_SEED, mb_base=3, recycle=res)
    print("\n  sizes", res.sizes(), flush=True)
    ref = O.sample_ladies(g.rowptr.cpu().numpy(), g.col.cpu().numpy(), batches.cpu().numpy(), s, synth.SAMPLING_SEED, 3)
    assert_hops_equal(res.hops(), ref, with_p=True, what="ladies on the largest graph")


def test_vertex_ids_up_to_the_int32_limit():
    """Maximum size of the id space: n = 2^31 - 1 vertices (ids up to 2^31 - 2, rowptr of 17 GB), edges among two
    million of them spread over the whole range including both ends.  Node-wise sampling (per-minibatch bitmaps in
    HBM are the only EXTRACT path for an id range this wide) and LADIES by LDS windows (32 768 windows per
    minibatch), each against the complete oracle result."""
    import numpy as np
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    n = 2**31 - 1
    gen = torch.Generator(device="cuda").manual_seed(5)
    active = torch.randint(0, n, (2_000_000,), device="cuda", generator=gen)
    active = torch.unique(torch.cat([active, torch.tensor([0, 1, n - 2, n - 1, 2**30 - 1, 2**30], device="cuda")]))
    m = 6_000_000
    src = active[torch.randint(0, active.numel(), (m,), device="cuda", generator=gen)]
    dst = active[(torch.rand(m, device="cuda", generator=gen) ** 2 * active.numel()).long()]   # a few hubs
    key = torch.unique(torch.cat([src * n + dst, dst * n + src]))
    src, dst = key // n, key % n
    del key
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device="cuda")
    rowptr[1:] = torch.cumsum(torch.bincount(src, minlength=n), 0)
    col = dst.to(torch.int32)
    del src, dst
    print("\n  n=%d nnz=%d max degree=%d" % (n, col.numel(), int((rowptr[1:] - rowptr[:-1]).max())), flush=True)
    csr = bms.Csr(rowptr, col)
    k, b = 2, 64
    pick = torch.randperm(active.numel(), device="cuda", generator=gen)[:k * b - 2]
    batches = torch.cat([active[pick], torch.tensor([0, n - 1], device="cuda")]).to(torch.int32).reshape(k, b).contiguous()
    rp, cl, bt = rowptr.cpu().numpy(), col.cpu().numpy(), batches.cpu().numpy()
    for variant in (dict(), dict(union_dst=True)):
        res = bms.sample_nodewise(csr, batches, (4, 3), 17, **variant)
        print("  node-wise", variant, res.sizes(), flush=True)
        ref = O.sample_nodewise(rp, cl, bt, (4, 3), 17, **variant)
        assert_hops_equal(res.hops(), ref, what="n = 2^31 - 1, node-wise %s" % variant)
        assert int(res.hop(1).col_vertex.max()) > 2**30
    res = bms.sample_ladies(csr, batches, (64, 32), 17)
    print("  ladies", res.sizes(), flush=True)
    ref = O.sample_ladies(rp, cl, bt, (64, 32), 17)
    assert_hops_equal(res.hops(), ref, with_p=True, what="n = 2^31 - 1, ladies")
