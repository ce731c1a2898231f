"""The library driven from a plain C program (tests/c_abi/bms_c_client.c, built by paper_2311_02909_amd/build.py):
host arrays in, device views copied back with the HIP runtime, compared with the oracle bit for bit."""
import os
import subprocess

import numpy as np
import pytest

from conftest import random_batches, random_csr

pytestmark = pytest.mark.gpu
CLIENT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "bms_c_client")


@pytest.mark.parametrize("variant", [dict(), dict(union_dst=True), dict(replace=True)], ids=["plain", "union_dst", "replace"])
def test_c_client_matches_oracle(tmp_path, variant):
    from oracle import bms_oracle as O
    assert os.path.exists(CLIENT), "build the C client first: python paper_2311_02909_amd/build.py"
    rng = np.random.default_rng(77)
    n, k, b, fanouts, seed = 50_000, 5, 200, (7, 4, 3), 123456789
    rowptr, col = random_csr(n, 11.0, rng)
    batches = random_batches(n, k, b, rng)
    problem, result = tmp_path / "problem.bin", tmp_path / "result.bin"
    with open(problem, "wb") as f:
        np.array([n, col.shape[0], k, b, len(fanouts), seed], dtype=np.int64).tofile(f)
        rowptr.astype(np.int64).tofile(f)
        col.astype(np.int32).tofile(f)
        batches.astype(np.int32).tofile(f)
        np.array(fanouts, dtype=np.int32).tofile(f)
    flags = (128 if variant.get("union_dst") else 0) | (256 if variant.get("replace") else 0)   # values of include/bms.h
    run = subprocess.run([CLIENT, str(problem), str(result), str(flags)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip() == "ok", (run.returncode, run.stdout, run.stderr)
    ref = O.sample_nodewise(rowptr, col, batches, fanouts, seed, **variant)
    with open(result, "rb") as f:
        for h, hop in enumerate(ref):
            rows, nnz, ncols = np.fromfile(f, dtype=np.int64, count=3)
            assert (rows, nnz, ncols) == (hop.rows, hop.nnz, hop.ncols), h
            for name, dtype, count in (("mb_rowoff", np.int64, k + 1), ("row_vertex", np.int32, rows),
                                       ("rowptr", np.int64, rows + 1), ("col", np.int32, nnz),
                                       ("mb_coloff", np.int64, k + 1), ("col_vertex", np.int32, ncols)) + (
                    (("row_self", np.int32, rows),) if variant.get("union_dst") else ()):
                got = np.fromfile(f, dtype=dtype, count=int(count))
                assert np.array_equal(got, getattr(hop, name)), (h, name)
        assert f.read() == b""


def test_c_client_drives_the_consumer_calls_and_the_layerwise_sampler(tmp_path):
    """bms_result_minibatch, bms_fetch_features, bms_aggregate_hop and bms_sample_ladies from plain C, each compared with
    the oracle (features are small integers, so the sums are exact in fp32)."""
    from oracle import bms_oracle as O
    from parity import slice_minibatch
    rng = np.random.default_rng(78)
    n, k, b, fanouts, seed, f = 30_000, 4, 150, (6, 3), 987654321, 8
    rowptr, col = random_csr(n, 9.0, rng)
    batches = random_batches(n, k, b, rng)
    problem, result = tmp_path / "problem.bin", tmp_path / "result.bin"
    with open(problem, "wb") as fh:
        np.array([n, col.shape[0], k, b, len(fanouts), seed], dtype=np.int64).tofile(fh)
        rowptr.astype(np.int64).tofile(fh)
        col.astype(np.int32).tofile(fh)
        batches.astype(np.int32).tofile(fh)
        np.array(fanouts, dtype=np.int32).tofile(fh)
    run = subprocess.run([CLIENT, str(problem), str(result), "0", "consumers"], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and run.stdout.strip() == "ok", (run.returncode, run.stdout, run.stderr)
    ref = O.sample_nodewise(rowptr, col, batches, fanouts, seed)
    lref = O.sample_ladies(rowptr, col, batches, tuple(8 * s for s in fanouts), seed)
    fields = (("mb_rowoff", np.int64, lambda h: k + 1), ("row_vertex", np.int32, lambda h: h.rows),
              ("rowptr", np.int64, lambda h: h.rows + 1), ("col", np.int32, lambda h: h.nnz),
              ("mb_coloff", np.int64, lambda h: k + 1), ("col_vertex", np.int32, lambda h: h.ncols))
    with open(result, "rb") as fh:
        for h, hop in enumerate(ref):
            assert tuple(np.fromfile(fh, dtype=np.int64, count=3)) == (hop.rows, hop.nnz, hop.ncols)
            for name, dtype, count in fields:
                assert np.array_equal(np.fromfile(fh, dtype=dtype, count=int(count(hop))), getattr(hop, name)), (h, name)
        for h, hop in enumerate(ref):
            for i in range(k):
                six = np.fromfile(fh, dtype=np.int64, count=6)
                m = slice_minibatch(hop, i)
                r0, c0 = int(hop.mb_rowoff[i]), int(hop.mb_coloff[i])
                assert tuple(six) == (m.rows, m.nnz, m.ncols, r0, int(hop.rowptr[r0]), c0), (h, i)
        H = ((31 * np.arange(n, dtype=np.int64)[:, None] + 7 * np.arange(f, dtype=np.int64)[None, :]) % 997).astype(np.float32)
        last = ref[-1]
        X = np.fromfile(fh, dtype=np.float32, count=last.ncols * f).reshape(last.ncols, f)
        assert np.array_equal(X, O.fetch_features(H, last.col_vertex))
        agg = np.fromfile(fh, dtype=np.float32, count=last.rows * f).reshape(last.rows, f)
        assert np.array_equal(agg, O.aggregate(last, X, mean=False))
        for h, hop in enumerate(lref):
            assert tuple(np.fromfile(fh, dtype=np.int64, count=3)) == (hop.rows, hop.nnz, hop.ncols)
            for name, dtype, count in fields:
                assert np.array_equal(np.fromfile(fh, dtype=dtype, count=int(count(hop))), getattr(hop, name)), (h, name)
            pnnz = int(np.fromfile(fh, dtype=np.int64, count=1)[0])
            assert pnnz == hop.p_col.shape[0]
            assert np.array_equal(np.fromfile(fh, dtype=np.int64, count=k + 1), hop.p_off)
            assert np.array_equal(np.fromfile(fh, dtype=np.int32, count=pnnz), hop.p_col)
            assert np.array_equal(np.fromfile(fh, dtype=np.uint32, count=pnnz), hop.p_cnt)
        assert fh.read() == b""
