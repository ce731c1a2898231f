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
