"""The seeded input generators (shared by the library's tests and the oracle; they hold none of the method)."""
import numpy as np
import pytest
import torch

from paper_2311_02909_amd import synth


def _check_graph(g):
    rowptr, col = g.rowptr.cpu().numpy(), g.col.cpu().numpy()
    n = g.n
    assert rowptr.shape == (n + 1,) and rowptr[0] == 0 and rowptr[-1] == col.shape[0] == g.nnz
    assert np.all(np.diff(rowptr) >= 0)
    assert col.min() >= 0 and col.max() < n
    src = np.repeat(np.arange(n), np.diff(rowptr))
    assert np.all(src != col)                                   # no self-loops
    key = src.astype(np.int64) * n + col
    assert np.all(np.diff(key) > 0)                             # rows ascending, no duplicates
    assert np.array_equal(np.sort(col.astype(np.int64) * n + src), key)   # symmetric


def test_tiny_workload_shape_and_determinism():
    g, batches, w = synth.make_workload("tiny_sage")
    _check_graph(g)
    assert g.n == 10_000 and abs(g.nnz - 200_000) <= 10_000
    assert batches.shape == (4, 64) and batches.dtype == torch.int32
    b = batches.numpy()
    assert len(np.unique(b)) == b.size and b.min() >= 0 and b.max() < g.n   # drawn without replacement
    g2, batches2, _ = synth.make_workload("tiny_sage")
    assert torch.equal(g.rowptr, g2.rowptr) and torch.equal(g.col, g2.col) and torch.equal(batches, batches2)


def test_generation_does_not_depend_on_chunking():
    a = synth.rmat_graph(5000, 60_000, 0.5, 0.2, 0.2, seed=3)
    b = synth.rmat_graph(5000, 60_000, 0.5, 0.2, 0.2, seed=3, chunk=7777)
    c = synth.rmat_graph(5000, 60_000, 0.5, 0.2, 0.2, seed=4)
    _check_graph(a)
    assert torch.equal(a.rowptr, b.rowptr) and torch.equal(a.col, b.col)
    assert not torch.equal(a.col[:1000], c.col[:1000])
    deg = (a.rowptr[1:] - a.rowptr[:-1]).numpy()
    assert deg.max() > 8 * deg.mean()                            # heavy tail


def test_train_split_is_a_prefix_of_a_seeded_permutation():
    p = synth.seeded_permutation(1000, 5, "cpu").numpy()
    assert np.array_equal(np.sort(p), np.arange(1000))
    assert not np.array_equal(p, synth.seeded_permutation(1000, 6, "cpu").numpy())
    b = synth.train_batches(1000, 0.2, 3, 50, 5, "cpu").numpy()
    assert len(np.unique(b)) == 150                              # seeds distinct across the whole split
    later = synth.train_batches(1000, 0.2, 2, 50, 5, "cpu", first=1).numpy()
    assert np.array_equal(later, b[1:3])                         # minibatch i = entries [i b, (i+1) b) of the split
    with pytest.raises(Exception):
        synth.train_batches(1000, 0.1, 3, 50, 5, "cpu")          # split smaller than k * b


@pytest.mark.gpu
def test_cpu_and_gpu_generation_agree():
    for name in ("tiny_sage",):
        gc, bc, _ = synth.make_workload(name, device="cpu")
        gg, bg, _ = synth.make_workload(name, device="cuda")
        assert torch.equal(gc.rowptr, gg.rowptr.cpu()) and torch.equal(gc.col, gg.col.cpu()) and torch.equal(bc, bg.cpu())
    a = synth.rmat_graph(200_000, 1_500_000, 0.5, 0.17, 0.17, seed=1, device="cpu")
    b = synth.rmat_graph(200_000, 1_500_000, 0.5, 0.17, 0.17, seed=1, device="cuda")
    assert torch.equal(a.rowptr, b.rowptr.cpu()) and torch.equal(a.col, b.col.cpu())
