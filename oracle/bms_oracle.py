"""ctypes front end of the plain CPU oracle (oracle/bms_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  Nothing in the product package imports it, and it
imports nothing from the product package.

All arithmetic is in the C file; this module only compiles it with gcc when no
built library is present, marshals numpy arrays in and copies the result arrays out.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bms_oracle.c")
_LIB = os.path.join(_HERE, "libbms_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over minibatches). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", tmp, _SRC]
        )
        os.replace(tmp, _LIB)
    return _LIB


class _Hop(C.Structure):
    _fields_ = [
        ("rows", C.c_int64),
        ("nnz", C.c_int64),
        ("ncols", C.c_int64),
        ("pnnz", C.c_int64),
        ("mb_rowoff", C.POINTER(C.c_int64)),
        ("row_vertex", C.POINTER(C.c_int32)),
        ("rowptr", C.POINTER(C.c_int64)),
        ("col", C.POINTER(C.c_int32)),
        ("mb_coloff", C.POINTER(C.c_int64)),
        ("col_vertex", C.POINTER(C.c_int32)),
        ("p_off", C.POINTER(C.c_int64)),
        ("p_col", C.POINTER(C.c_int32)),
        ("p_cnt", C.POINTER(C.c_uint32)),
        ("row_self", C.POINTER(C.c_int32)),
    ]


_lib: Optional[C.CDLL] = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.orc_mix64.restype = C.c_uint64
        L.orc_mix64.argtypes = [C.c_uint64]
        L.orc_fin32.restype = C.c_uint32
        L.orc_fin32.argtypes = [C.c_uint32]
        L.orc_rowkey.restype = C.c_uint64
        L.orc_rowkey.argtypes = [C.c_uint64, C.c_int32, C.c_uint32, C.c_uint32]
        L.orc_draw32.restype = C.c_uint32
        L.orc_draw32.argtypes = [C.c_uint64, C.c_uint32]
        L.orc_draw64.restype = C.c_uint64
        L.orc_draw64.argtypes = [C.c_uint64, C.c_uint32]
        L.orc_bounded32.restype = C.c_uint32
        L.orc_bounded32.argtypes = [C.c_uint32, C.c_uint32]
        L.orc_bounded64.restype = C.c_uint64
        L.orc_bounded64.argtypes = [C.c_uint64, C.c_uint64]
        L.orc_its_distinct.restype = None
        L.orc_its_distinct.argtypes = [C.c_uint64, C.c_uint32, C.c_int32, C.POINTER(C.c_uint32)]
        common = [C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32,
                  C.c_uint64, C.c_int32]
        L.orc_sample_nodewise.restype = C.c_int
        L.orc_sample_nodewise.argtypes = common + [C.POINTER(C.c_void_p)]
        L.orc_sample_nodewise_variant.restype = C.c_int
        L.orc_sample_nodewise_variant.argtypes = common + [C.c_int, C.POINTER(C.c_void_p)]
        L.orc_its_replace.restype = C.c_int32
        L.orc_its_replace.argtypes = [C.c_uint64, C.c_uint32, C.c_int32, C.POINTER(C.c_uint32)]
        L.orc_sample_ladies.restype = C.c_int
        L.orc_sample_ladies.argtypes = common + [C.c_int, C.POINTER(C.c_void_p)]
        L.orc_result_hop.restype = C.POINTER(_Hop)
        L.orc_result_hop.argtypes = [C.c_void_p, C.c_int32]
        L.orc_result_free.restype = None
        L.orc_result_free.argtypes = [C.c_void_p]
        L.orc_fetch_features.restype = C.c_int
        L.orc_fetch_features.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
        L.orc_aggregate.restype = None
        L.orc_aggregate.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                    C.c_int, C.c_void_p]
        L.orc_set_threads.restype = C.c_int
        L.orc_set_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


# ---- scalar access to the random stream (used by the brute-force pins) ----
def mix64(x: int) -> int:
    return lib().orc_mix64(x & 0xFFFFFFFFFFFFFFFF)


def fin32(x: int) -> int:
    return lib().orc_fin32(x & 0xFFFFFFFF)


def rowkey(seed: int, hop: int, mb: int, vertex: int) -> int:
    return lib().orc_rowkey(seed & 0xFFFFFFFFFFFFFFFF, hop, mb & 0xFFFFFFFF, vertex & 0xFFFFFFFF)


def draw32(key: int, j: int) -> int:
    return lib().orc_draw32(key, j)


def draw64(key: int, j: int) -> int:
    return lib().orc_draw64(key, j)


def bounded32(x: int, m: int) -> int:
    return lib().orc_bounded32(x, m)


def bounded64(x: int, w: int) -> int:
    return lib().orc_bounded64(x, w)


def its_distinct(key: int, deg: int, s: int) -> List[int]:
    buf = (C.c_uint32 * max(s, 1))()
    lib().orc_its_distinct(key, deg, s, buf)
    return [int(buf[i]) for i in range(s)]


def its_replace(key: int, deg: int, s: int) -> List[int]:
    """Distinct positions picked by s independent draws in [0, deg), ascending."""
    buf = (C.c_uint32 * max(s, 1))()
    c = lib().orc_its_replace(key, deg, s, buf)
    return [int(buf[i]) for i in range(c)]


def set_threads(nthreads: int = 0) -> int:
    """Set (if > 0) and return the number of threads of the loop over minibatches."""
    return int(lib().orc_set_threads(nthreads))


def fetch_features(H: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """Rows of the n x f fp32 feature matrix H for the listed vertex ids (Sec. 6.2); raises on an id outside [0, n)."""
    H = np.ascontiguousarray(H, dtype=np.float32)
    ids = np.ascontiguousarray(ids, dtype=np.int32)
    n, f = H.shape
    out = np.empty((ids.shape[0], f), dtype=np.float32)
    rc = lib().orc_fetch_features(H.ctypes.data, n, f, ids.ctypes.data, ids.shape[0], out.ctypes.data)
    if rc != 0:
        raise ValueError("vertex id outside [0, %d)" % n)
    return out


def aggregate(hop, X: np.ndarray, mean: bool = True) -> np.ndarray:
    """Forward aggregation of one hop (Sec. 6.2): out[r] = mean (or sum) of X over row r's sampled columns.

    `hop` is a Hop of a bulk sample; X has one fp32 row per stacked column (hop.ncols x f)."""
    X = np.ascontiguousarray(X, dtype=np.float32)
    assert X.shape[0] == hop.ncols
    f = X.shape[1]
    mb_rowoff = np.ascontiguousarray(hop.mb_rowoff, dtype=np.int64)
    rowptr = np.ascontiguousarray(hop.rowptr, dtype=np.int64)
    col = np.ascontiguousarray(hop.col, dtype=np.int32)
    mb_coloff = np.ascontiguousarray(hop.mb_coloff, dtype=np.int64)
    out = np.empty((hop.rows, f), dtype=np.float32)
    lib().orc_aggregate(mb_rowoff.ctypes.data, mb_rowoff.shape[0] - 1, rowptr.ctypes.data, col.ctypes.data,
                        mb_coloff.ctypes.data, X.ctypes.data, f, 1 if mean else 0, out.ctypes.data)
    return out


NOVERTEX = 0xFFFFFFFF


@dataclass
class Hop:
    """One hop of a bulk sample, every array a host numpy copy (same fields as the C struct)."""
    rows: int
    nnz: int
    ncols: int
    mb_rowoff: np.ndarray
    row_vertex: np.ndarray
    rowptr: np.ndarray
    col: np.ndarray
    mb_coloff: np.ndarray
    col_vertex: np.ndarray
    p_off: Optional[np.ndarray] = None
    p_col: Optional[np.ndarray] = None
    p_cnt: Optional[np.ndarray] = None
    row_self: Optional[np.ndarray] = None   # union_dst only: local column of each row's own vertex


def _copy(ptr, count, dtype):
    if count == 0:
        return np.zeros(0, dtype=dtype)
    return np.ctypeslib.as_array(ptr, shape=(count,)).astype(dtype, copy=True)


def _collect(handle, k: int, L: int, with_p: bool) -> List[Hop]:
    hops = []
    for h in range(L):
        hp = lib().orc_result_hop(handle, h).contents
        hop = Hop(
            rows=int(hp.rows), nnz=int(hp.nnz), ncols=int(hp.ncols),
            mb_rowoff=_copy(hp.mb_rowoff, k + 1, np.int64),
            row_vertex=_copy(hp.row_vertex, hp.rows, np.int32),
            rowptr=_copy(hp.rowptr, hp.rows + 1, np.int64),
            col=_copy(hp.col, hp.nnz, np.int32),
            mb_coloff=_copy(hp.mb_coloff, k + 1, np.int64),
            col_vertex=_copy(hp.col_vertex, hp.ncols, np.int32),
        )
        if hp.row_self:
            hop.row_self = _copy(hp.row_self, hp.rows, np.int32)
        if with_p:
            hop.p_off = _copy(hp.p_off, k + 1, np.int64)
            hop.p_col = _copy(hp.p_col, hp.pnnz, np.int32)
            hop.p_cnt = _copy(hp.p_cnt, hp.pnnz, np.uint32)
        hops.append(hop)
    return hops


def _prep(rowptr, col, batches, params):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    batches = np.ascontiguousarray(batches, dtype=np.int32)
    if batches.ndim != 2:
        raise ValueError("batches must be a k x b array")
    params = np.ascontiguousarray(params, dtype=np.int32)
    return rowptr, col, batches, params


UNION_DST, REPLACE = 1, 2


def sample_nodewise(rowptr, col, batches, fanouts: Sequence[int], seed: int, mb_base: int = 0,
                    collect: bool = True, union_dst: bool = False, replace: bool = False) -> Optional[List[Hop]]:
    """Bulk GraphSAGE sampling (Sec. 4.1, Eq. 1). With collect=False only runs it (for timing).

    union_dst: the frontier's own vertices stay columns (next frontier = frontier + sampled), Hop.row_self filled.
    replace: the s draws of a row are independent; the row keeps the distinct picks."""
    rowptr, col, batches, fan = _prep(rowptr, col, batches, fanouts)
    k, b = batches.shape
    out = C.c_void_p()
    variant = (UNION_DST if union_dst else 0) | (REPLACE if replace else 0)
    rc = lib().orc_sample_nodewise_variant(rowptr.ctypes.data, col.ctypes.data, rowptr.size - 1, batches.ctypes.data,
                                           k, b, fan.ctypes.data, fan.size, seed & 0xFFFFFFFFFFFFFFFF, mb_base,
                                           variant, C.byref(out))
    if rc:
        raise ValueError("oracle rejected the input (code %d)" % rc)
    try:
        return _collect(out, k, fan.size, False) if collect else None
    finally:
        lib().orc_result_free(out)


def sample_ladies(rowptr, col, batches, s_per_layer: Sequence[int], seed: int, mb_base: int = 0,
                  squared: bool = False, collect: bool = True) -> Optional[List[Hop]]:
    """Bulk LADIES sampling (Sec. 4.2)."""
    rowptr, col, batches, sp = _prep(rowptr, col, batches, s_per_layer)
    k, b = batches.shape
    out = C.c_void_p()
    rc = lib().orc_sample_ladies(rowptr.ctypes.data, col.ctypes.data, rowptr.size - 1, batches.ctypes.data, k, b,
                                 sp.ctypes.data, sp.size, seed & 0xFFFFFFFFFFFFFFFF, mb_base, int(squared),
                                 C.byref(out))
    if rc:
        raise ValueError("oracle rejected the input (code %d)" % rc)
    try:
        return _collect(out, k, sp.size, True) if collect else None
    finally:
        lib().orc_result_free(out)
