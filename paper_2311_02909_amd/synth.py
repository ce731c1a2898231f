"""Seeded synthetic inputs: R-MAT graphs in CSR form and train-split minibatches.

This module serves both the HIP library's tests/benchmark and the CPU oracle's
tests.  It holds none of the sampler's arithmetic: it only manufactures inputs
(a {0,1} adjacency matrix A in CSR, and k x b seed-vertex batches) with the shapes
and degree skew of the workloads in Table 3 / Table 4 of the paper, whose datasets
themselves are not available here.

Everything is a pure function of integer seeds through a stateless 64-bit mixing
hash, written with torch integer ops only, so the same graph comes out on the CPU
and on the GPU (the large graphs are only ever generated on the GPU).

Recipe (R-MAT, Chakrabarti et al. 2004):
  * scale = ceil(log2 n); edge e picks, at each of `scale` levels, one quadrant
    (a, b, c, d) from a 32-bit hash of (seed, e, level); bits accumulate into
    (src, dst);
  * pairs with an endpoint >= n or src == dst are dropped;
  * vertex ids are relabelled through a seeded permutation of [0, n) so that degree
    is uncorrelated with id;
  * both directions are emitted, sorted, duplicates removed; rowptr is int64,
    col is int32 and ascending within a row.
Train split: the first ceil(frac * n) entries of a second seeded permutation;
minibatch i is entries [i*b, (i+1)*b) of it, so seeds are distinct within a batch.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

_M64 = (1 << 64)
_C1 = 0xBF58476D1CE4E5B9 - _M64  # as signed int64
_C2 = 0x94D049BB133111EB - _M64
_GOLD = 0x9E3779B97F4A7C15 - _M64


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x: torch.Tensor) -> torch.Tensor:
    """64-bit mixing hash on int64 tensors (wrapping arithmetic)."""
    x = x ^ _lsr(x, 30)
    x = x * _C1
    x = x ^ _lsr(x, 27)
    x = x * _C2
    x = x ^ _lsr(x, 31)
    return x


def _scalar_mix(x: int) -> int:
    x &= _M64 - 1
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & (_M64 - 1)
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & (_M64 - 1)
    x ^= x >> 31
    return x


def _signed(x: int) -> int:
    x &= _M64 - 1
    return x - _M64 if x >= (1 << 63) else x


def seeded_permutation(n: int, seed: int, device="cpu") -> torch.Tensor:
    """A permutation of [0, n) (int64) determined by `seed`: stable argsort of hashed ids."""
    base = _signed(_scalar_mix(seed * 2 + 1))
    keys = _lsr(_mix(torch.arange(n, dtype=torch.int64, device=device) * _GOLD + base), 1)
    return torch.sort(keys, stable=True).indices


def _rmat_pairs(e0: int, e1: int, scale: int, a: float, b: float, c: float, seed: int, device) -> Tuple[torch.Tensor, torch.Tensor]:
    """(src, dst) in [0, 2^scale) for edge counters e0..e1-1."""
    ta = int(a * 4294967296.0)
    tab = int((a + b) * 4294967296.0)
    tabc = int((a + b + c) * 4294967296.0)
    e = torch.arange(e0, e1, dtype=torch.int64, device=device)
    src = torch.zeros_like(e)
    dst = torch.zeros_like(e)
    base = _signed(_scalar_mix(seed * 2))
    nhash = (scale + 1) // 2
    for q in range(nhash):
        hsh = _mix((e * nhash + q) * _GOLD + base)
        for half in range(2):
            lvl = 2 * q + half
            if lvl >= scale:
                break
            u = _lsr(hsh, 32) if half == 0 else (hsh & 0xFFFFFFFF)
            sbit = (u >= tab).to(torch.int64)                       # quadrants c, d: lower half of rows
            dbit = ((u >= ta) & (u < tab) | (u >= tabc)).to(torch.int64)  # quadrants b, d: right half of columns
            src = src * 2 + sbit
            dst = dst * 2 + dbit
    return src, dst


@dataclass
class Graph:
    n: int
    nnz: int
    rowptr: torch.Tensor  # int64, n+1
    col: torch.Tensor     # int32, nnz
    max_degree: int
    isolated: int

    @property
    def mean_degree(self) -> float:
        return self.nnz / max(self.n, 1)

    def describe(self) -> str:
        return "n=%d nnz=%d mean_deg=%.2f max_deg=%d isolated=%d" % (
            self.n, self.nnz, self.mean_degree, self.max_degree, self.isolated)


def rmat_graph(n: int, pairs: int, a: float, b: float, c: float, seed: int, device="cpu",
               chunk: int = 1 << 25, parts: Optional[int] = None) -> Graph:
    """Symmetric, loop-free, duplicate-free R-MAT graph on n vertices from `pairs` generated pairs."""
    scale = max(1, math.ceil(math.log2(max(n, 2))))
    perm = seeded_permutation(n, seed + 1000003, device)
    keys = []
    for e0 in range(0, pairs, chunk):
        e1 = min(pairs, e0 + chunk)
        src, dst = _rmat_pairs(e0, e1, scale, a, b, c, seed, device)
        keep = (src < n) & (dst < n) & (src != dst)
        src = perm[src[keep]]
        dst = perm[dst[keep]]
        keys.append(torch.cat([src * n + dst, dst * n + src]))
        del src, dst, keep
    total = sum(int(x.numel()) for x in keys)
    if parts is None:
        parts = max(1, math.ceil(total / (1 << 28)))
    span = (n + parts - 1) // parts
    counts = torch.zeros(n, dtype=torch.int64, device=device)
    cols = []
    for p in range(parts):
        lo, hi = p * span, min(n, (p + 1) * span)
        if lo >= hi:
            break
        if parts == 1:
            seg = keys[0] if len(keys) == 1 else torch.cat(keys)
        else:
            seg = torch.cat([x[(x >= lo * n) & (x < hi * n)] for x in keys])
        seg = torch.unique_consecutive(torch.sort(seg).values)
        rows = torch.div(seg, n, rounding_mode="floor")
        cols.append((seg - rows * n).to(torch.int32))
        counts[lo:hi] = torch.bincount(rows - lo, minlength=hi - lo)
        del seg, rows
    del keys
    col = torch.cat(cols) if cols else torch.zeros(0, dtype=torch.int32, device=device)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    rowptr[1:] = torch.cumsum(counts, 0)
    return Graph(n=n, nnz=int(col.numel()), rowptr=rowptr, col=col,
                 max_degree=int(counts.max().item()) if n else 0,
                 isolated=int((counts == 0).sum().item()))


def relabel_by_degree(g: Graph, parts: Optional[int] = None) -> Graph:
    """The same graph with its vertices renumbered by descending degree (hubs first, ties by old id): the id
    layout of datasets whose ids correlate with degree, the opposite of rmat_graph's random relabelling."""
    n, device = g.n, g.rowptr.device
    deg = g.rowptr[1:] - g.rowptr[:-1]
    order = torch.sort(deg, descending=True, stable=True).indices          # new id -> old id
    newid = torch.empty(n, dtype=torch.int64, device=device)
    newid[order] = torch.arange(n, dtype=torch.int64, device=device)
    keys = torch.repeat_interleave(newid, deg) * n                           # new source of every entry
    keys += newid[g.col.long()] if g.nnz < (1 << 28) else torch.index_select(newid, 0, g.col)
    if parts is None:
        parts = max(1, math.ceil(g.nnz / (1 << 28)))
    span = (n + parts - 1) // parts
    cols = []
    for p in range(parts):
        lo, hi = p * span, min(n, (p + 1) * span)
        if lo >= hi:
            break
        seg = keys if parts == 1 else keys[(keys >= lo * n) & (keys < hi * n)]
        seg = torch.sort(seg).values
        cols.append((seg % n).to(torch.int32))
        del seg
    del keys
    col = torch.cat(cols) if cols else torch.zeros(0, dtype=torch.int32, device=device)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    rowptr[1:] = torch.cumsum(deg[order], 0)
    return Graph(n=n, nnz=g.nnz, rowptr=rowptr, col=col, max_degree=g.max_degree, isolated=g.isolated)


def train_batches(n: int, frac: float, k: int, b: int, seed: int, device="cpu", first: int = 0) -> torch.Tensor:
    """k x b int32 seed vertices: minibatches first..first+k-1 of the seeded train split."""
    ntrain = int(math.ceil(frac * n))
    if (first + k) * b > ntrain:
        raise ValueError("train split of %d vertices holds fewer than %d batches of %d" % (ntrain, first + k, b))
    perm = seeded_permutation(n, seed + 2000003, device)
    return perm[first * b:(first + k) * b].to(torch.int32).reshape(k, b).contiguous()


# The five workloads (graph recipe + sampler parameters).  `pairs` is the only tuned
# number: how many R-MAT pairs to generate so that nnz lands near the target.
# `features` = length f of a vertex's feature vector in the dataset the workload stands in for (Table 3)
WORKLOADS = {
    # Tiny node-wise
    "tiny_sage": dict(graph=dict(n=10_000, pairs=148_000, a=0.57, b=0.19, c=0.19, seed=1),
                      sampler="nodewise", params=(5, 5), batch=64, k=4, frac=0.10, features=16),
    # Mid node-wise: stands in for the Products-sized row of Table 3
    "mid_sage": dict(graph=dict(n=2_450_000, pairs=94_000_000, a=0.50, b=0.17, c=0.17, seed=1),
                     sampler="nodewise", params=(15, 10, 5), batch=1024, k=64, frac=0.08, features=100),
    # Layer-wise on the same graph
    "mid_ladies": dict(graph=dict(n=2_450_000, pairs=94_000_000, a=0.50, b=0.17, c=0.17, seed=1),
                       sampler="ladies", params=(512, 512, 512), batch=512, k=32, frac=0.08, features=100),
    # Large node-wise: stands in for the Papers-sized row of Table 3
    "large_sage": dict(graph=dict(n=111_000_000, pairs=861_000_000, a=0.52, b=0.18, c=0.18, seed=1),
                       sampler="nodewise", params=(15, 10, 5), batch=1024, k=256, frac=0.011, features=128),
    # Dense-ish large: stands in for the Protein-sized row of Table 3
    "dense_sage": dict(graph=dict(n=8_700_000, pairs=1_280_000_000, a=0.45, b=0.22, c=0.22, seed=1),
                       sampler="nodewise", params=(15, 10, 5), batch=1024, k=128, frac=0.12, features=128),
    "dense_ladies": dict(graph=dict(n=8_700_000, pairs=1_280_000_000, a=0.45, b=0.22, c=0.22, seed=1),
                         sampler="ladies", params=(2048, 2048, 2048), batch=1024, k=64, frac=0.12, features=128),
}

SPLIT_SEED = 2
SAMPLING_SEED = 42


def make_workload(name: str, device="cpu", relabel: Optional[str] = None) -> Tuple[Graph, torch.Tensor, dict]:
    """(graph, batches k x b int32, workload dict) for one named workload.  relabel="degree": vertex ids sorted by
    descending degree instead of the recipe's random relabelling."""
    w = WORKLOADS[name]
    g = rmat_graph(device=device, **w["graph"])
    if relabel == "degree":
        g = relabel_by_degree(g)
    elif relabel is not None:
        raise ValueError("unknown relabel %r" % relabel)
    batches = train_batches(g.n, w["frac"], w["k"], w["batch"], SPLIT_SEED, device)
    return g, batches, w
