"""ctypes binding of include/tofu.h: same names, argument marshalling only.

The library is loaded from the in-tree build (paper_1807_08887_amd/libtofu.so).  If it has not
been built this module builds it once with hipcc; if that is impossible it raises -- there is no
CPU fallback for any entry point.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

TOFU_MAX_DIMS = 6
STATIC_SCRATCH_BYTES = 32 << 20      # TOFU_STATIC_SCRATCH_BYTES of include/tofu.h
OP_MATMUL, OP_CONV2D, OP_CONV2D_WGRAD, OP_CONV2D_DGRAD, OP_LSTM_CELL, OP_CONV1D = 0, 1, 2, 3, 4, 5
LSTM_DIM_B, LSTM_DIM_H = 0, 1
CONV1D_DIM_B, CONV1D_DIM_CO, CONV1D_DIM_X, CONV1D_DIM_CI = 0, 1, 2, 3
MM_DIM_M, MM_DIM_N, MM_DIM_K = 0, 1, 2
CONV_DIM_N, CONV_DIM_CO, CONV_DIM_H, CONV_DIM_W, CONV_DIM_CI = 0, 1, 2, 3, 4
WGRAD_DIM_CO, WGRAD_DIM_CI, WGRAD_DIM_N = 0, 1, 2
DGRAD_DIM_N, DGRAD_DIM_CI, DGRAD_DIM_H, DGRAD_DIM_W, DGRAD_DIM_CO = 0, 1, 2, 3, 4

_i64x = ctypes.c_int64 * TOFU_MAX_DIMS


class Region(ctypes.Structure):
    _fields_ = [("ndim", ctypes.c_int32), ("lo", _i64x), ("hi", _i64x)]

    def box(self):
        return [(int(self.lo[d]), int(self.hi[d])) for d in range(self.ndim)]

    @staticmethod
    def from_box(box) -> "Region":
        r = Region()
        r.ndim = len(box)
        for d, (lo, hi) in enumerate(box):
            r.lo[d], r.hi[d] = lo, hi
        return r


class Tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("extent", Region), ("stride", _i64x)]


class Split(ctypes.Structure):
    _fields_ = [("dim", ctypes.c_int32), ("k", ctypes.c_int32), ("shard", ctypes.c_int32)]


class OpDesc(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
                ("batch", ctypes.c_int64), ("c_in", ctypes.c_int64), ("c_out", ctypes.c_int64), ("H", ctypes.c_int64),
                ("W", ctypes.c_int64), ("KH", ctypes.c_int64), ("KW", ctypes.c_int64), ("stride", ctypes.c_int64),
                ("pad", ctypes.c_int64)]


class TofuError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"tofu status {status}: {message}")
        self.status = status


_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libtofu.so")
_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load libtofu.so, building it first when no built library exists or when the sources it was
    built from are not the present ones (their hash is kept beside the library)."""
    global _lib
    if _lib is not None:
        return _lib
    from .build import build, is_current
    if not is_current():
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    P = ctypes.POINTER
    lib.tofu_last_error.restype = ctypes.c_char_p
    lib.tofu_last_error.argtypes = []
    lib.tofu_shard_range.argtypes = [i64, i32, i32, P(i64), P(i64)]
    lib.tofu_op_regions.argtypes = [P(OpDesc), P(Split), i32, P(Region), P(Region), P(i64), P(i64), P(i32)]
    lib.tofu_workspace_bytes.restype = sz
    lib.tofu_workspace_bytes.argtypes = [P(OpDesc), P(Split), i32]
    lib.tofu_region_fetch.argtypes = [P(Tensor), P(Tensor), i32, vp]
    shard_calls = ("tofu_shard_matmul", "tofu_shard_conv2d", "tofu_shard_conv2d_wgrad", "tofu_shard_conv2d_dgrad", "tofu_shard_conv1d")
    accumulate_calls = tuple(n + "_accumulate" for n in shard_calls)
    for name in shard_calls + accumulate_calls:
        getattr(lib, name).argtypes = [P(OpDesc), P(Split), i32, P(Tensor), P(Tensor), P(Tensor), vp, sz, vp]
    lib.tofu_shard_matmul_noalloc.argtypes = [P(OpDesc), P(Split), i32, P(Tensor), P(Tensor), P(Tensor), vp]
    lib.tofu_shard_matmul_noalloc.restype = ctypes.c_int
    lib.tofu_shard_conv2d_fused.argtypes = [P(OpDesc), P(Split), i32, P(Tensor), i32, P(Tensor), P(Tensor), vp, sz, vp]
    lib.tofu_partition_reduce.argtypes = [vp, P(vp), i32, i64, vp]
    lib.tofu_shard_lstm_cell.argtypes = [P(OpDesc), P(Split), i32, P(Tensor), P(Tensor), P(Tensor), P(Tensor), vp]
    lib.tofu_partition_reduce_ex.argtypes = [vp, P(vp), i32, i64, i32, i32, vp]
    lib.tofu_partition_reduce_scatter.argtypes = [vp, P(vp), i32, i64, i32, i32, i32, i32, vp]
    lib.tofu_probe_mfma.argtypes = [vp, i32, i32, vp]
    lib.tofu_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.tofu_probe_read.argtypes = [vp, sz, vp, vp]
    lib.tofu_probe_stream.argtypes = [vp, P(vp), i32, sz, vp]
    lib.tofu_probe_read.restype = lib.tofu_probe_stream.restype = ctypes.c_int
    for name in ("tofu_shard_range", "tofu_op_regions", "tofu_region_fetch", "tofu_shard_matmul", "tofu_shard_conv2d",
                 "tofu_shard_conv2d_wgrad", "tofu_partition_reduce", "tofu_probe_mfma", "tofu_probe_copy", "tofu_shard_conv2d_fused", "tofu_shard_conv2d_dgrad", "tofu_partition_reduce_ex", "tofu_shard_lstm_cell",
                 "tofu_partition_reduce_scatter") + accumulate_calls:
        getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def last_error() -> str:
    return load().tofu_last_error().decode()


def _check(status: int) -> None:
    if status != 0:
        raise TofuError(status, last_error())


def _splits(splits: Sequence) -> tuple:
    arr = (Split * max(1, len(splits)))()
    for i, s in enumerate(splits):
        arr[i].dim, arr[i].k, arr[i].shard = (s.dim, s.k, s.shard) if isinstance(s, Split) else s
    return arr, len(splits)


def matmul_desc(M: int, N: int, K: int) -> OpDesc:
    d = OpDesc()
    d.kind, d.M, d.N, d.K = OP_MATMUL, M, N, K
    return d


def conv2d_desc(batch, c_in, c_out, H, W, KH=3, KW=3, stride=1, pad=1, kind=OP_CONV2D) -> OpDesc:
    d = OpDesc()
    d.kind = kind
    d.batch, d.c_in, d.c_out, d.H, d.W, d.KH, d.KW, d.stride, d.pad = batch, c_in, c_out, H, W, KH, KW, stride, pad
    return d


def wgrad_desc(batch, c_in, c_out, H, W, KH=3, KW=3, stride=1, pad=1) -> OpDesc:
    return conv2d_desc(batch, c_in, c_out, H, W, KH, KW, stride, pad, kind=OP_CONV2D_WGRAD)


def lstm_cell_desc(batch: int, hidden: int) -> OpDesc:
    d = OpDesc()
    d.kind, d.M, d.N = OP_LSTM_CELL, batch, hidden
    return d


def dgrad_desc(batch, c_in, c_out, H, W, KH=3, KW=3, stride=1, pad=1) -> OpDesc:
    """Data gradient of the convolution whose INPUT is [batch, c_in, H, W]."""
    return conv2d_desc(batch, c_in, c_out, H, W, KH, KW, stride, pad, kind=OP_CONV2D_DGRAD)


def tensor(t, lo: Optional[Sequence[int]] = None) -> Tensor:
    """Descriptor of a CUDA float32 torch tensor holding the global box [lo, lo + t.shape)."""
    import torch
    if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or not t.is_cuda:
        raise TypeError("tofu tensors must be float32 torch tensors in device memory")
    lo = list(lo) if lo is not None else [0] * t.dim()
    if len(lo) != t.dim() or t.dim() > TOFU_MAX_DIMS:
        raise ValueError("lo must give one coordinate per tensor dimension (at most 6)")
    if t.numel() > 1 and all(t.stride(i) == 0 for i in range(t.dim()) if t.shape[i] > 1):
        raise ValueError("a fully expanded (all strides zero) tensor cannot be described: all-zero strides mean dense row-major; "
                         "materialise it first")
    d = Tensor()
    d.data = t.data_ptr()
    d.extent.ndim = t.dim()
    for i in range(t.dim()):
        d.extent.lo[i] = lo[i]
        d.extent.hi[i] = lo[i] + t.shape[i]
        d.stride[i] = t.stride(i)
    return d


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return ctypes.c_void_p(int(stream))


def shard_range(extent: int, k: int, shard: int):
    lo, hi = ctypes.c_int64(), ctypes.c_int64()
    _check(load().tofu_shard_range(extent, k, shard, ctypes.byref(lo), ctypes.byref(hi)))
    return lo.value, hi.value


def op_regions(op: OpDesc, splits: Sequence):
    """-> dict(out_box, in_boxes, pad_lo, pad_hi, is_partial) with boxes as [(lo, hi), ...]."""
    arr, n = _splits(splits)
    out, ins = Region(), (Region * 2)()
    plo, phi, part = (ctypes.c_int64 * 2)(), (ctypes.c_int64 * 2)(), ctypes.c_int32()
    _check(load().tofu_op_regions(ctypes.byref(op), arr, n, ctypes.byref(out), ins, plo, phi, ctypes.byref(part)))
    return dict(out_box=out.box(), in_boxes=[ins[0].box(), ins[1].box()], pad_lo=list(plo), pad_hi=list(phi),
                is_partial=bool(part.value))


def workspace_bytes(op: OpDesc, splits: Sequence) -> int:
    """tofu_workspace_bytes; an invalid operator or plan (0 with an error text) raises."""
    arr, n = _splits(splits)
    need = int(load().tofu_workspace_bytes(ctypes.byref(op), arr, n))
    if need == 0 and last_error():
        raise TofuError(-1, last_error())
    return need


def region_fetch(dst: Tensor, srcs: Sequence[Tensor], stream=None) -> None:
    arr = (Tensor * max(1, len(srcs)))(*srcs)
    _check(load().tofu_region_fetch(ctypes.byref(dst), arr, len(srcs), _stream(stream)))


def _shard(fn, op, splits, a, b, c, workspace, stream):
    arr, n = _splits(splits)
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (workspace.data_ptr(), workspace.numel() * workspace.element_size())
    _check(fn(ctypes.byref(op), arr, n, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c), ws_ptr, ws_bytes, _stream(stream)))


def shard_matmul(op, splits, A: Tensor, B: Tensor, C: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_matmul, op, splits, A, B, C, workspace, stream)


def shard_matmul_noalloc(op, splits, A: Tensor, B: Tensor, C: Tensor, stream=None) -> None:
    """tofu_shard_matmul_noalloc: the K slices go to the library's built-in device array."""
    arr, n = _splits(splits)
    _check(load().tofu_shard_matmul_noalloc(ctypes.byref(op), arr, n, ctypes.byref(A), ctypes.byref(B), ctypes.byref(C), _stream(stream)))


def shard_conv2d(op, splits, x: Tensor, w: Tensor, y: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv2d, op, splits, x, w, y, workspace, stream)


def shard_conv2d_fused(op, splits, x_srcs: Sequence[Tensor], w: Tensor, y: Tensor, workspace=None, stream=None) -> None:
    """tofu_shard_conv2d_fused: the input region is read from the blocks `x_srcs` that hold it."""
    sp, n = _splits(splits)
    arr = (Tensor * max(1, len(x_srcs)))(*x_srcs)
    ws_ptr, ws_bytes = (None, 0) if workspace is None else (ctypes.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size())
    _check(load().tofu_shard_conv2d_fused(ctypes.byref(op), sp, n, arr, len(x_srcs), ctypes.byref(w), ctypes.byref(y), ws_ptr, ws_bytes,
                                          _stream(stream)))


def shard_conv2d_wgrad(op, splits, x: Tensor, dy: Tensor, dw: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv2d_wgrad, op, splits, x, dy, dw, workspace, stream)


def shard_conv2d_dgrad(op, splits, dy: Tensor, w: Tensor, dx: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv2d_dgrad, op, splits, dy, w, dx, workspace, stream)


def shard_matmul_accumulate(op, splits, A: Tensor, B: Tensor, C: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_matmul_accumulate, op, splits, A, B, C, workspace, stream)


def shard_conv2d_accumulate(op, splits, x: Tensor, w: Tensor, y: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv2d_accumulate, op, splits, x, w, y, workspace, stream)


def shard_conv2d_wgrad_accumulate(op, splits, x: Tensor, dy: Tensor, dw: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv2d_wgrad_accumulate, op, splits, x, dy, dw, workspace, stream)


def shard_conv2d_dgrad_accumulate(op, splits, dy: Tensor, w: Tensor, dx: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv2d_dgrad_accumulate, op, splits, dy, w, dx, workspace, stream)


def conv1d_desc(batch: int, c_in: int, c_out: int, length: int, window: int = 3) -> OpDesc:
    """Fig. 1's conv1d: data [batch, c_in, length], filters [c_in, c_out, window], out [batch, c_out, length - window + 1]."""
    d = OpDesc()
    d.kind, d.batch, d.c_in, d.c_out, d.W, d.KW = OP_CONV1D, batch, c_in, c_out, length, window
    d.H, d.KH, d.stride, d.pad = 1, 1, 1, 0
    return d


def shard_conv1d(op, splits, data: Tensor, filters: Tensor, out: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv1d, op, splits, data, filters, out, workspace, stream)


def shard_conv1d_accumulate(op, splits, data: Tensor, filters: Tensor, out: Tensor, workspace=None, stream=None) -> None:
    _shard(load().tofu_shard_conv1d_accumulate, op, splits, data, filters, out, workspace, stream)


def shard_lstm_cell(op, splits, gates: Tensor, c_prev: Tensor, c_new: Tensor, h_new: Tensor, stream=None) -> None:
    sp, n = _splits(splits)
    _check(load().tofu_shard_lstm_cell(ctypes.byref(op), sp, n, ctypes.byref(gates), ctypes.byref(c_prev), ctypes.byref(c_new),
                                       ctypes.byref(h_new), _stream(stream)))


REDUCE_SUM, REDUCE_MAX, REDUCE_MIN, REDUCE_PROD = 0, 1, 2, 3
ORDER_LINEAR, ORDER_TREE = 0, 1


def _addr(t) -> int:
    if isinstance(t, int):
        return t
    if not t.is_cuda or t.dtype.itemsize != 4 or not t.is_contiguous():
        raise TypeError("partition_reduce needs contiguous float32 device tensors")
    return t.data_ptr()


def partition_reduce_scatter(dst, partials: Sequence, shares: int, share: int, count: Optional[int] = None, stream=None,
                             reducer: int = REDUCE_SUM, order: int = ORDER_LINEAR) -> None:
    """tofu_partition_reduce_scatter: combine only share `share` of `shares` of the flat index range."""
    if count is None:
        count = dst.numel()
    ptrs = (ctypes.c_void_p * max(1, len(partials)))(*[_addr(p) for p in partials])
    _check(load().tofu_partition_reduce_scatter(ctypes.c_void_p(_addr(dst)), ptrs, len(partials), count, shares, share, reducer, order,
                                                _stream(stream)))


def partition_reduce(dst, partials: Sequence, count: Optional[int] = None, stream=None, reducer: Optional[int] = None,
                     order: int = ORDER_LINEAR) -> None:
    """dst, partials: CUDA float32 torch tensors (contiguous) or raw device addresses.
    With `reducer` given the call goes to tofu_partition_reduce_ex."""
    addr = _addr
    if count is None:
        count = dst.numel()
    ptrs = (ctypes.c_void_p * max(1, len(partials)))(*[addr(p) for p in partials])
    if reducer is None:
        _check(load().tofu_partition_reduce(ctypes.c_void_p(addr(dst)), ptrs, len(partials), count, _stream(stream)))
    else:
        _check(load().tofu_partition_reduce_ex(ctypes.c_void_p(addr(dst)), ptrs, len(partials), count, reducer, order, _stream(stream)))


def probe_mfma(sink, iters: int, workgroups: int, stream=None) -> None:
    """include/tofu_probe.h: register-only fp32 MFMA loop; FLOP = workgroups * 4 * iters * 8 * 4096."""
    _check(load().tofu_probe_mfma(ctypes.c_void_p(sink.data_ptr()), iters, workgroups, _stream(stream)))


def probe_copy(dst, src, nbytes: Optional[int] = None, stream=None) -> None:
    """include/tofu_probe.h: plain 16-byte-vector copy between two device tensors."""
    if nbytes is None:
        nbytes = src.numel() * src.element_size()
    _check(load().tofu_probe_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), nbytes, _stream(stream)))


def probe_read(src, sink, nbytes: Optional[int] = None, stream=None) -> None:
    """include/tofu_probe.h: read-only nontemporal stream over a device tensor."""
    if nbytes is None:
        nbytes = src.numel() * src.element_size()
    _check(load().tofu_probe_read(ctypes.c_void_p(src.data_ptr()), nbytes, ctypes.c_void_p(sink.data_ptr()), _stream(stream)))


def probe_stream(dst, srcs: Sequence, nbytes: Optional[int] = None, stream=None) -> None:
    """include/tofu_probe.h: k:1 read:write stream, dst = sum of the k sources (k in 1, 2, 4, 8)."""
    if nbytes is None:
        nbytes = dst.numel() * dst.element_size()
    ptrs = (ctypes.c_void_p * max(1, len(srcs)))(*[t.data_ptr() for t in srcs])
    _check(load().tofu_probe_stream(ctypes.c_void_p(dst.data_ptr()), ptrs, len(srcs), nbytes, _stream(stream)))
