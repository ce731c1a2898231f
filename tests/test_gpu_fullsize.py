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
