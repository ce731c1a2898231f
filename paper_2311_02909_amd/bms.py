"""Thin binding over the C ABI of libbms.so (include/bms.h).

Argument marshalling only: every step of the sampling path runs in the library's HIP
kernels.  PyTorch supplies device memory for the inputs, the current stream, and
zero-copy tensor views of the result buffers.  There is no CPU fallback: if the
library has not been built, importing any entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbms.so")

OK, EINVAL, ERANGE, EFORMAT, ENOMEM, EHIP, EAGAIN = 0, -1, -2, -3, -4, -5, -6
HOST, DEVICE_BORROW, DEVICE_COPY = 0, 1, 2
LADIES_SQUARED, PROFILE, EXTRACT_BUCKETS, EXTRACT_BITMAP, EXTRACT_SORT, LADIES_DENSE, PROFILE_MAIN = 1, 2, 4, 8, 16, 32, 64
UNION_DST, NODEWISE_REPLACE, ASYNC, LADIES_NO_INDEX = 128, 256, 512, 1024
NOALLOC_MAX_K = 16383


class BmsError(RuntimeError):
    def __init__(self, code: int, detail: str):
        super().__init__("bms error %d: %s" % (code, detail))
        self.code = code


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p)
DEALLOC_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class _Opts(C.Structure):
    _fields_ = [("stream", C.c_void_p), ("mb_base", C.c_int32), ("flags", C.c_uint32),
                ("recycle", C.c_void_p), ("scratch_limit", C.c_int64),
                ("alloc", ALLOC_FN), ("dealloc", DEALLOC_FN), ("alloc_ctx", C.c_void_p)]


class TorchAllocator:
    """bms_opts.alloc / dealloc served by torch.empty: the result's buffers then live in PyTorch's caching
    allocator.  Keep the object alive as long as any result created with it."""

    def __init__(self, device="cuda"):
        self.device = device
        self.live = {}
        self.calls = 0

        def _alloc(nbytes, _ctx):
            try:
                t = torch.empty(int(nbytes), dtype=torch.uint8, device=self.device)
            except RuntimeError:
                return None
            self.live[t.data_ptr()] = t
            self.calls += 1
            return t.data_ptr()

        def _dealloc(ptr, _ctx):
            self.live.pop(ptr, None)

        self.alloc, self.dealloc = ALLOC_FN(_alloc), DEALLOC_FN(_dealloc)


class _HopView(C.Structure):
    _fields_ = [("rows", C.c_int64), ("nnz", C.c_int64), ("ncols", C.c_int64), ("pnnz", C.c_int64),
                ("mb_rowoff", C.c_void_p), ("row_vertex", C.c_void_p), ("rowptr", C.c_void_p), ("col", C.c_void_p),
                ("mb_coloff", C.c_void_p), ("col_vertex", C.c_void_p), ("p_off", C.c_void_p), ("p_col", C.c_void_p),
                ("p_cnt", C.c_void_p), ("row_self", C.c_void_p)]


class _MbView(C.Structure):
    _fields_ = [("rows", C.c_int64), ("nnz", C.c_int64), ("ncols", C.c_int64), ("row0", C.c_int64),
                ("edge0", C.c_int64), ("col0", C.c_int64), ("row_vertex", C.c_void_p), ("rowptr", C.c_void_p),
                ("col", C.c_void_p), ("col_vertex", C.c_void_p), ("row_self", C.c_void_p)]


_lib = None


def lib() -> C.CDLL:
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                              "or `python -m paper_2311_02909_amd.build` first" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        L.bms_csr_load.restype = C.c_int
        L.bms_csr_load.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.POINTER(C.c_void_p)]
        L.bms_csr_held_bytes.restype = C.c_int
        L.bms_csr_held_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_int64)]
        L.bms_csr_info.restype = C.c_int
        L.bms_csr_info.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
        for fn in (L.bms_sample_nodewise, L.bms_sample_ladies):
            fn.restype = C.c_int
            fn.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_uint64,
                           C.POINTER(_Opts), C.POINTER(C.c_void_p)]
        L.bms_result_wait.restype = C.c_int
        L.bms_result_wait.argtypes = [C.c_void_p]
        L.bms_result_ready.restype = C.c_int
        L.bms_result_ready.argtypes = [C.c_void_p]
        L.bms_result_attempts.restype = C.c_int
        L.bms_result_attempts.argtypes = [C.c_void_p, C.POINTER(C.c_int32)]
        L.bms_result_info.restype = C.c_int
        L.bms_result_info.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
        L.bms_result_hop.restype = C.c_int
        L.bms_result_hop.argtypes = [C.c_void_p, C.c_int32, C.POINTER(_HopView)]
        L.bms_result_minibatch.restype = C.c_int
        L.bms_result_minibatch.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(_MbView)]
        L.bms_result_minibatch_offsets.restype = C.c_int
        L.bms_result_minibatch_offsets.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.bms_result_stage.restype = C.c_int
        L.bms_result_stage.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_int32),
                                       C.POINTER(C.c_float)]
        L.bms_free.restype = None
        L.bms_free.argtypes = [C.c_void_p]
        L.bms_aggregate_hop.restype = C.c_int
        L.bms_aggregate_hop.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int, C.c_void_p, C.c_void_p]
        L.bms_fetch_features.restype = C.c_int
        L.bms_fetch_features.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p]
        L.bms_strerror.restype = C.c_char_p
        L.bms_strerror.argtypes = [C.c_int]
        L.bms_last_error.restype = C.c_char_p
        L.bms_last_error.argtypes = []
        _lib = L
    return _lib


def _check(rc: int):
    if rc != OK:
        detail = lib().bms_last_error().decode() or lib().bms_strerror(rc).decode()
        raise BmsError(rc, detail)


class _DevArray:
    """A device buffer owned by a result, exposed through the CUDA array interface."""

    def __init__(self, ptr: int, count: int, typestr: str, owner):
        self.owner = owner
        self.__cuda_array_interface__ = {"shape": (count,), "typestr": typestr, "data": (ptr, False), "version": 2}


def _view(ptr, count: int, dtype: torch.dtype, owner) -> torch.Tensor:
    if count == 0 or not ptr:
        return torch.empty(0, dtype=dtype, device="cuda")
    typestr = {torch.int32: "<i4", torch.int64: "<i8"}[dtype]
    return torch.as_tensor(_DevArray(int(ptr), int(count), typestr, owner), device="cuda")


@dataclass
class Hop:
    """One hop of a bulk sample (see bms_hop_view in include/bms.h). Tensors are views of
    device memory owned by the result; p_cnt holds uint32 values in an int32 tensor."""
    rows: int
    nnz: int
    ncols: int
    pnnz: int
    mb_rowoff: torch.Tensor
    row_vertex: torch.Tensor
    rowptr: torch.Tensor
    col: torch.Tensor
    mb_coloff: torch.Tensor
    col_vertex: torch.Tensor
    p_off: Optional[torch.Tensor]
    p_col: Optional[torch.Tensor]
    p_cnt: Optional[torch.Tensor]
    row_self: Optional[torch.Tensor] = None   # union_dst only: local column of each row's own vertex

    def to_host(self) -> "HostHop":
        def cp(t, dt=None):
            if t is None:
                return None
            a = t.cpu().numpy()
            return a.view(dt) if dt is not None else a
        return HostHop(self.rows, self.nnz, self.ncols, cp(self.mb_rowoff), cp(self.row_vertex), cp(self.rowptr),
                       cp(self.col), cp(self.mb_coloff), cp(self.col_vertex), cp(self.p_off), cp(self.p_col),
                       cp(self.p_cnt, np.uint32), cp(self.row_self))


@dataclass
class Minibatch:
    """One minibatch of one hop (bms_mb_view): views into the stacked arrays; A_i is the CSR
    (rowptr - edge0, col) over `ncols` local columns whose vertices are col_vertex."""
    rows: int
    nnz: int
    ncols: int
    row0: int
    edge0: int
    col0: int
    row_vertex: torch.Tensor
    rowptr: torch.Tensor
    col: torch.Tensor
    col_vertex: torch.Tensor
    row_self: Optional[torch.Tensor] = None


@dataclass
class HostHop:
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
    row_self: Optional[np.ndarray] = None


class Csr:
    """Adjacency matrix resident on the device (bms_csr_load)."""

    def __init__(self, rowptr: torch.Tensor, col: torch.Tensor):
        if rowptr.dtype != torch.int64 or col.dtype != torch.int32:
            raise TypeError("rowptr must be int64 and col int32")
        rowptr, col = rowptr.contiguous(), col.contiguous()
        n, nnz = rowptr.numel() - 1, col.numel()
        if rowptr.is_cuda != col.is_cuda:
            raise ValueError("rowptr and col must live on the same side")
        self._keep = (rowptr, col)          # borrowed device arrays must stay alive
        loc = DEVICE_BORROW if rowptr.is_cuda else HOST
        h = C.c_void_p()
        _check(lib().bms_csr_load(rowptr.data_ptr(), col.data_ptr() if nnz else None, n, nnz, loc, C.byref(h)))
        self.handle = h
        if loc == HOST:
            self._keep = None
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        _check(lib().bms_csr_info(h, C.byref(a), C.byref(b), C.byref(c)))
        self.n, self.nnz, self.max_degree = a.value, b.value, c.value

    def held_bytes(self) -> int:
        """bms_csr_held_bytes: device memory the handle holds beyond the caller's arrays."""
        v = C.c_int64()
        _check(lib().bms_csr_held_bytes(self.handle, C.byref(v)))
        return v.value

    def free(self):
        if getattr(self, "handle", None):
            lib().bms_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Result:
    """Owner of the device buffers of one bulk sample (bms_result)."""

    def __init__(self, handle):
        self.handle = handle
        k, L = C.c_int32(), C.c_int32()
        _check(lib().bms_result_info(handle, C.byref(k), C.byref(L)))
        self.k, self.L = k.value, L.value

    def wait(self):
        """bms_result_wait: blocks until an asynchronous call has completed; raises its deferred error."""
        _check(lib().bms_result_wait(self.handle))

    def ready(self) -> bool:
        """bms_result_ready: False while an asynchronous call still runs."""
        return lib().bms_result_ready(self.handle) == 1

    def attempts(self) -> int:
        """bms_result_attempts: how many times the call that wrote this result enqueued its kernels."""
        v = C.c_int32()
        _check(lib().bms_result_attempts(self.handle, C.byref(v)))
        return v.value

    def hop(self, h: int) -> Hop:
        v = _HopView()
        _check(lib().bms_result_hop(self.handle, h, C.byref(v)))
        k = self.k
        has_p = bool(v.p_off)
        return Hop(
            rows=v.rows, nnz=v.nnz, ncols=v.ncols, pnnz=v.pnnz,
            mb_rowoff=_view(v.mb_rowoff, k + 1, torch.int64, self),
            row_vertex=_view(v.row_vertex, v.rows, torch.int32, self),
            rowptr=_view(v.rowptr, v.rows + 1, torch.int64, self),
            col=_view(v.col, v.nnz, torch.int32, self),
            mb_coloff=_view(v.mb_coloff, k + 1, torch.int64, self),
            col_vertex=_view(v.col_vertex, v.ncols, torch.int32, self),
            p_off=_view(v.p_off, k + 1, torch.int64, self) if has_p else None,
            p_col=_view(v.p_col, v.pnnz, torch.int32, self) if has_p else None,
            p_cnt=_view(v.p_cnt, v.pnnz, torch.int32, self) if has_p else None,
            row_self=_view(v.row_self, v.rows, torch.int32, self) if v.row_self else None,
        )

    def minibatch(self, h: int, i: int) -> Minibatch:
        """bms_result_minibatch: minibatch i of hop h cut out of the stack (no copies of the arrays)."""
        v = _MbView()
        _check(lib().bms_result_minibatch(self.handle, h, i, C.byref(v)))
        return Minibatch(
            rows=v.rows, nnz=v.nnz, ncols=v.ncols, row0=v.row0, edge0=v.edge0, col0=v.col0,
            row_vertex=_view(v.row_vertex, v.rows, torch.int32, self),
            rowptr=_view(v.rowptr, v.rows + 1, torch.int64, self),
            col=_view(v.col, v.nnz, torch.int32, self),
            col_vertex=_view(v.col_vertex, v.ncols, torch.int32, self),
            row_self=_view(v.row_self, v.rows, torch.int32, self) if v.row_self else None,
        )

    def minibatch_offsets(self, h: int, out: Optional[np.ndarray] = None, stream=None) -> np.ndarray:
        """bms_result_minibatch_offsets: the (row, entry, column) offsets of every minibatch of hop h as a
        3 x (k+1) int64 host array (filled in place when `out` is given); the library allocates nothing."""
        if out is None:
            out = np.empty((3, self.k + 1), dtype=np.int64)
        if out.dtype != np.int64 or out.shape != (3, self.k + 1) or not out.flags.c_contiguous:
            raise TypeError("out must be a C-contiguous 3 x (k+1) int64 array")
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        _check(lib().bms_result_minibatch_offsets(self.handle, h, out[0].ctypes.data, out[1].ctypes.data,
                                                  out[2].ctypes.data, stream))
        return out

    def hops(self) -> List[Hop]:
        return [self.hop(h) for h in range(self.L)]

    def sizes(self) -> List[Tuple[int, int, int]]:
        """(rows, nnz, ncols) per hop without creating tensor views."""
        out = []
        v = _HopView()
        for h in range(self.L):
            _check(lib().bms_result_hop(self.handle, h, C.byref(v)))
            out.append((v.rows, v.nnz, v.ncols))
        return out

    def stages(self) -> List[Tuple[str, int, float]]:
        """(stage name, hop, milliseconds) in launch order; empty unless sampled with profile=True."""
        out, i = [], 0
        name, hop, ms = C.c_char_p(), C.c_int32(), C.c_float()
        while lib().bms_result_stage(self.handle, i, C.byref(name), C.byref(hop), C.byref(ms)) == OK:
            out.append((name.value.decode(), hop.value, ms.value))
            i += 1
        return out

    def free(self):
        if getattr(self, "handle", None):
            lib().bms_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _profile_flag(profile) -> int:
    """profile=True: every stage timed; profile="main": only the sampler's main kernel stage (cheaper)."""
    if profile == "main":
        return PROFILE_MAIN
    return PROFILE if profile else 0


def _sample(fn, csr: Csr, batches, params: Sequence[int], seed: int, mb_base, stream, recycle, flags, scratch_limit,
            allocator=None):
    if isinstance(batches, np.ndarray):
        batches = torch.from_numpy(np.ascontiguousarray(batches, dtype=np.int32))
    if batches.dtype != torch.int32 or batches.dim() != 2:
        raise TypeError("batches must be a k x b int32 tensor")
    batches = batches.contiguous()
    k, b = batches.shape
    par = (C.c_int32 * len(params))(*[int(p) for p in params])
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    opts = _Opts(stream=stream, mb_base=mb_base, flags=flags,
                 recycle=recycle.handle if recycle is not None else None, scratch_limit=scratch_limit)
    if allocator is not None:
        opts.alloc, opts.dealloc = allocator.alloc, allocator.dealloc
    out = C.c_void_p()
    _check(fn(csr.handle, batches.data_ptr(), k, b, par, len(params), seed & 0xFFFFFFFFFFFFFFFF, C.byref(opts),
              C.byref(out)))
    if recycle is not None:
        recycle.k, recycle.L = k, len(params)
        return recycle
    r = Result(out)
    r._allocator = allocator   # the callbacks must outlive the result
    return r


def sample_nodewise(csr: Csr, batches, fanouts: Sequence[int], seed: int, *, mb_base: int = 0, stream=None,
                    recycle: Optional[Result] = None, profile: bool = False, scratch_limit: int = 0,
                    extract: Optional[str] = None, union_dst: bool = False, replace: bool = False,
                    allocator=None, async_: bool = False) -> Result:
    """bms_sample_nodewise: bulk GraphSAGE sampling of the k x b seed batches.
    extract: None (library's choice), "sort", "buckets" or "bitmap" -- which EXTRACT kernels run; same result.
    union_dst: BMS_UNION_DST, every frontier contains the one before it and Hop.row_self is filled.
    replace: BMS_NODEWISE_REPLACE, independent draws per row, the distinct picks kept.
    allocator: e.g. TorchAllocator(): where the result's buffers come from (bms_opts.alloc / dealloc).
    async_: BMS_ASYNC, a recycled call of a remembered shape returns before its kernels have run."""
    flags = _profile_flag(profile) | {None: 0, "buckets": EXTRACT_BUCKETS, "bitmap": EXTRACT_BITMAP,
                                           "sort": EXTRACT_SORT}[extract] | (UNION_DST if union_dst else 0) | (
        NODEWISE_REPLACE if replace else 0) | (ASYNC if async_ else 0)
    return _sample(lib().bms_sample_nodewise, csr, batches, fanouts, seed, mb_base, stream, recycle, flags,
                   scratch_limit, allocator)


def sample_ladies(csr: Csr, batches, s_per_layer: Sequence[int], seed: int, *, mb_base: int = 0, squared: bool = False,
                  stream=None, recycle: Optional[Result] = None, profile: bool = False,
                  scratch_limit: int = 0, dense: bool = False, allocator=None, index: bool = True) -> Result:
    """bms_sample_ladies: bulk LADIES sampling of the k x b seed batches.  index=False: BMS_LADIES_NO_INDEX.

    dense=True picks the kernel path with per-minibatch counters in HBM (same results)."""
    flags = _profile_flag(profile) | (LADIES_SQUARED if squared else 0) | (LADIES_DENSE if dense else 0) | (0 if index else LADIES_NO_INDEX)
    return _sample(lib().bms_sample_ladies, csr, batches, s_per_layer, seed, mb_base, stream, recycle, flags,
                   scratch_limit, allocator)


def fetch_features(H: torch.Tensor, ids: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """bms_fetch_features: out[j, :] = H[ids[j], :] (device tensors; H n x f fp32, ids int32)."""
    if H.dtype != torch.float32 or H.dim() != 2 or not H.is_cuda or not H.is_contiguous():
        raise TypeError("H must be a contiguous n x f float32 device tensor")
    if ids.dtype != torch.int32 or ids.dim() != 1 or not ids.is_cuda or not ids.is_contiguous():
        raise TypeError("ids must be a contiguous int32 device vector")
    n, f = H.shape
    m = ids.shape[0]
    if out is None:
        out = torch.empty((m, f), dtype=torch.float32, device=H.device)
    elif out.dtype != torch.float32 or tuple(out.shape) != (m, f) or not out.is_cuda or not out.is_contiguous():
        raise TypeError("out must be a contiguous m x f float32 device tensor")
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().bms_fetch_features(H.data_ptr(), n, f, ids.data_ptr(), m, out.data_ptr(), stream))
    return out


def aggregate_hop(res: "Result", hop: int, X: torch.Tensor, mean: bool = True, out: Optional[torch.Tensor] = None,
                  stream=None) -> torch.Tensor:
    """bms_aggregate_hop: out[r, :] = mean (or sum) of X over the sampled columns of stacked row r of `hop`."""
    if X.dtype != torch.float32 or X.dim() != 2 or not X.is_cuda or not X.is_contiguous():
        raise TypeError("X must be a contiguous ncols x f float32 device tensor")
    rows, _, ncols = res.sizes()[hop]
    if X.shape[0] != ncols:
        raise ValueError("X has %d rows, the hop has %d columns" % (X.shape[0], ncols))
    f = X.shape[1]
    if out is None:
        out = torch.empty((rows, f), dtype=torch.float32, device=X.device)
    elif out.dtype != torch.float32 or tuple(out.shape) != (rows, f) or not out.is_cuda or not out.is_contiguous():
        raise TypeError("out must be a contiguous rows x f float32 device tensor")
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    _check(lib().bms_aggregate_hop(res.handle, hop, X.data_ptr(), f, 1 if mean else 0, out.data_ptr(), stream))
    return out
