"""Randomised shapes: both samplers against the oracle on graphs, batch shapes and sampling parameters drawn
from a seeded stream (skewed and uniform graphs, directed and symmetric, tiny to mid-size frontiers)."""
import os

import numpy as np
import pytest
import torch

from conftest import random_batches, random_csr, skewed_csr
from parity import assert_hops_equal

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("case", range(int(os.environ.get("BMS_RANDOM_CASES", "40"))))
def test_random_case(case):
    from oracle import bms_oracle as O
    from paper_2311_02909_amd import bms
    rng = np.random.default_rng(1000 + case)
    n = int(rng.choice([300, 5_000, 70_000, 400_000]))
    if rng.random() < 0.5:
        rowptr, col = skewed_csr(n, int(n * rng.uniform(2, 12)), rng)
    else:
        rowptr, col = random_csr(n, float(rng.uniform(1, 20)), rng, symmetric=bool(rng.random() < 0.5))
    k = int(rng.integers(1, 9))
    b = int(min(n, rng.choice([1, 7, 64, 300, 1500])))
    L = int(rng.integers(1, 4))
    csr = bms.Csr(torch.from_numpy(rowptr).cuda(), torch.from_numpy(col).cuda())
    batches = random_batches(n, k, b, rng)
    seed, mb_base = int(rng.integers(0, 2**62)), int(rng.integers(0, 1000))
    fanouts = tuple(int(x) for x in rng.choice([1, 2, 3, 5, 8, 15, 20, 40], size=L))
    ref = O.sample_nodewise(rowptr, col, batches, fanouts, seed, mb_base)
    res = None
    for extract in (None, "buckets", "sort", None):   # recycled calls of the same shape skip the size read-backs
        res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), fanouts, seed, mb_base=mb_base,
                                  extract=extract, recycle=res)
        assert_hops_equal(res.hops(), ref, what="case %d nodewise fanouts=%s extract=%s" % (case, fanouts, extract))
    variant = dict(union_dst=bool(rng.random() < 0.5), replace=bool(rng.random() < 0.5))
    if any(variant.values()):
        vref = O.sample_nodewise(rowptr, col, batches, fanouts, seed, mb_base, **variant)
        for extract in (None, "bitmap", None):   # the last one recycles: no size read-backs
            res = bms.sample_nodewise(csr, torch.from_numpy(batches).cuda(), fanouts, seed, mb_base=mb_base,
                                      extract=extract, recycle=res, **variant)
            assert_hops_equal(res.hops(), vref, what="case %d nodewise %s fanouts=%s extract=%s" % (
                case, variant, fanouts, extract))
    s = tuple(int(x) for x in rng.choice([1, 4, 33, 200, 1000, 4096], size=L))
    squared = bool(rng.random() < 0.3)
    lref = O.sample_ladies(rowptr, col, batches, s, seed, mb_base, squared)
    for dense in (False, True):
        lres = bms.sample_ladies(csr, torch.from_numpy(batches).cuda(), s, seed, mb_base=mb_base, squared=squared,
                                 dense=dense)
        assert_hops_equal(lres.hops(), lref, with_p=True, what="case %d ladies s=%s dense=%s" % (case, s, dense))
