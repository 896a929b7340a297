"""TEST INFRASTRUCTURE (oracle side): ctypes access to the fp64 loop nests in tofu_oracle.c.

Inputs are float32 numpy arrays holding the UNPARTITIONED tensors (dense, row-major);
outputs are (value, abs_sum) float64 arrays.  See tofu_oracle.c for what each routine
computes and which passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tofu_oracle.c")
_LIB = os.path.join(_HERE, "libtofu_oracle.so")
_lib = None

_i64 = ctypes.c_int64
_fp = ctypes.POINTER(ctypes.c_float)
_dp = ctypes.POINTER(ctypes.c_double)
_ip = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = True) -> str:
    """Compile tofu_oracle.c with gcc (OpenMP).  No fast-math: fp64 sums keep source order."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_LIB)
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_fp)


def _out(n):
    v, s = np.empty(n, dtype=np.float64), np.empty(n, dtype=np.float64)
    return v, s, v.ctypes.data_as(_dp), s.ctypes.data_as(_dp)


def _pts(pts, nd):
    p = np.ascontiguousarray(pts, dtype=np.int64).reshape(-1, nd)
    return p, p.ctypes.data_as(_ip)


def _box(box):
    lo = (ctypes.c_int64 * 4)(*[b[0] for b in box])
    hi = (ctypes.c_int64 * 4)(*[b[1] for b in box])
    return lo, hi


def threads() -> int:
    return int(_load().oracle_threads())


def matmul_box(A, B, box=None, krange=None):
    """C over box [(m0,m1),(n0,n1)] (default all), summing k over krange (default all)."""
    A, pa = _f32(A); B, pb = _f32(B)
    M, K = A.shape; K2, N = B.shape
    assert K == K2
    (m0, m1), (n0, n1) = box or ((0, M), (0, N))
    k0, k1 = krange or (0, K)
    v, s, pv, ps = _out((m1 - m0) * (n1 - n0))
    _load().oracle_matmul_box(pa, pb, _i64(M), _i64(N), _i64(K), _i64(m0), _i64(m1), _i64(n0), _i64(n1),
                              _i64(k0), _i64(k1), pv, ps)
    return v.reshape(m1 - m0, n1 - n0), s.reshape(m1 - m0, n1 - n0)


def matmul_pts(A, B, pts, krange=None):
    A, pa = _f32(A); B, pb = _f32(B)
    M, K = A.shape; _, N = B.shape
    k0, k1 = krange or (0, K)
    p, pp = _pts(pts, 2)
    v, s, pv, ps = _out(len(p))
    _load().oracle_matmul_pts(pa, pb, _i64(M), _i64(N), _i64(K), _i64(len(p)), pp, _i64(k0), _i64(k1), pv, ps)
    return v, s


def _conv_dims(x, c_out, KH, KW, stride, pad):
    batch, c_in, H, W = x.shape
    ho = (H + 2 * pad - KH) // stride + 1
    wo = (W + 2 * pad - KW) // stride + 1
    args = [_i64(v) for v in (batch, c_in, c_out, H, W, KH, KW, stride, pad)]
    return args, (batch, c_in, ho, wo)


def conv2d_box(x, w, stride=1, pad=0, box=None, cirange=None):
    """y over box [(n),(co),(h),(w)] (default all), summing ci over cirange (default all)."""
    x, px = _f32(x); w, pw = _f32(w)
    c_out, c_in, KH, KW = w.shape
    assert x.shape[1] == c_in
    args, (batch, _, ho, wo) = _conv_dims(x, c_out, KH, KW, stride, pad)
    box = box or ((0, batch), (0, c_out), (0, ho), (0, wo))
    shape = [b[1] - b[0] for b in box]
    c0, c1 = cirange or (0, c_in)
    lo, hi = _box(box)
    v, s, pv, ps = _out(int(np.prod(shape)))
    _load().oracle_conv2d_box(px, pw, *args, lo, hi, _i64(c0), _i64(c1), pv, ps)
    return v.reshape(shape), s.reshape(shape)


def conv2d_pts(x, w, pts, stride=1, pad=0, cirange=None):
    x, px = _f32(x); w, pw = _f32(w)
    c_out, c_in, KH, KW = w.shape
    args, _ = _conv_dims(x, c_out, KH, KW, stride, pad)
    c0, c1 = cirange or (0, c_in)
    p, pp = _pts(pts, 4)
    v, s, pv, ps = _out(len(p))
    _load().oracle_conv2d_pts(px, pw, *args, _i64(len(p)), pp, _i64(c0), _i64(c1), pv, ps)
    return v, s


def conv1d_box(data, filters, box=None, cirange=None):
    """Fig. 1's conv1d over box [(b),(co),(x)] (default all): data [B, CI, X + DX - 1], filters [CI, CO, DX]."""
    data, pd = _f32(data); filters, pf = _f32(filters)
    batch, c_in, L = data.shape
    assert filters.shape[0] == c_in
    c_out, DX = filters.shape[1], filters.shape[2]
    X = L - DX + 1
    box = box or ((0, batch), (0, c_out), (0, X))
    shape = [b[1] - b[0] for b in box]
    c0, c1 = cirange or (0, c_in)
    lo = (ctypes.c_int64 * 3)(*[b[0] for b in box])
    hi = (ctypes.c_int64 * 3)(*[b[1] for b in box])
    v, s, pv, ps = _out(int(np.prod(shape)))
    _load().oracle_conv1d_box(pd, pf, _i64(batch), _i64(c_in), _i64(c_out), _i64(X), _i64(DX), lo, hi, _i64(c0), _i64(c1), pv, ps)
    return v.reshape(shape), s.reshape(shape)


def wgrad_box(x, dy, KH, KW, stride=1, pad=0, box=None, nrange=None):
    """dw over box [(co),(ci),(kh),(kw)] (default all), summing n over nrange (default all)."""
    x, px = _f32(x); dy, pd = _f32(dy)
    c_out = dy.shape[1]
    args, (batch, c_in, ho, wo) = _conv_dims(x, c_out, KH, KW, stride, pad)
    assert dy.shape == (batch, c_out, ho, wo)
    box = box or ((0, c_out), (0, c_in), (0, KH), (0, KW))
    shape = [b[1] - b[0] for b in box]
    n0, n1 = nrange or (0, batch)
    lo, hi = _box(box)
    v, s, pv, ps = _out(int(np.prod(shape)))
    _load().oracle_wgrad_box(px, pd, *args, lo, hi, _i64(n0), _i64(n1), pv, ps)
    return v.reshape(shape), s.reshape(shape)


def wgrad_pts(x, dy, KH, KW, pts, stride=1, pad=0, nrange=None):
    x, px = _f32(x); dy, pd = _f32(dy)
    c_out = dy.shape[1]
    args, (batch, _, _, _) = _conv_dims(x, c_out, KH, KW, stride, pad)
    n0, n1 = nrange or (0, batch)
    p, pp = _pts(pts, 4)
    v, s, pv, ps = _out(len(p))
    _load().oracle_wgrad_pts(px, pd, *args, _i64(len(p)), pp, _i64(n0), _i64(n1), pv, ps)
    return v, s


def _dgrad_dims(dy, w, H, W, stride, pad):
    c_out, c_in, KH, KW = w.shape
    batch = dy.shape[0]
    ho = (H + 2 * pad - KH) // stride + 1
    wo = (W + 2 * pad - KW) // stride + 1
    assert dy.shape == (batch, c_out, ho, wo), "dy must have the forward output's shape"
    return [_i64(v) for v in (batch, c_in, c_out, H, W, KH, KW, stride, pad)], (batch, c_in, c_out)


def dgrad_box(dy, w, H, W, stride=1, pad=0, box=None, corange=None):
    """dx over box [(n),(ci),(h),(w)] of the H x W input (default all), summing co over corange (default all)."""
    dy, pd = _f32(dy); w, pw = _f32(w)
    args, (batch, c_in, c_out) = _dgrad_dims(dy, w, H, W, stride, pad)
    box = box or ((0, batch), (0, c_in), (0, H), (0, W))
    shape = [b[1] - b[0] for b in box]
    c0, c1 = corange or (0, c_out)
    lo, hi = _box(box)
    v, s, pv, ps = _out(int(np.prod(shape)))
    _load().oracle_dgrad_box(pd, pw, *args, lo, hi, _i64(c0), _i64(c1), pv, ps)
    return v.reshape(shape), s.reshape(shape)


def dgrad_pts(dy, w, H, W, pts, stride=1, pad=0, corange=None):
    dy, pd = _f32(dy); w, pw = _f32(w)
    args, (_, _, c_out) = _dgrad_dims(dy, w, H, W, stride, pad)
    c0, c1 = corange or (0, c_out)
    p, pp = _pts(pts, 4)
    v, s, pv, ps = _out(len(p))
    _load().oracle_dgrad_pts(pd, pw, *args, _i64(len(p)), pp, _i64(c0), _i64(c1), pv, ps)
    return v, s


def reduce(partials):
    """Element-wise sum of a list of equally shaped float32 arrays -> (value, abs_sum)."""
    arrs = [np.ascontiguousarray(p, dtype=np.float32) for p in partials]
    shape = arrs[0].shape
    assert all(a.shape == shape for a in arrs)
    ptrs = (_fp * len(arrs))(*[a.ctypes.data_as(_fp) for a in arrs])
    v, s, pv, ps = _out(arrs[0].size)
    _load().oracle_reduce(ptrs, _i64(len(arrs)), _i64(arrs[0].size), pv, ps)
    return v.reshape(shape), s.reshape(shape)


REDUCERS = {"sum": 0, "max": 1, "min": 2, "prod": 3}


def reduce_op(partials, reducer="sum"):
    """Element-wise Sum / Max / Min / Prod of equally shaped float32 arrays -> (value, scale)."""
    if reducer == "sum":
        return reduce(partials)
    arrs = [np.ascontiguousarray(p, dtype=np.float32) for p in partials]
    shape = arrs[0].shape
    assert all(a.shape == shape for a in arrs)
    ptrs = (_fp * len(arrs))(*[a.ctypes.data_as(_fp) for a in arrs])
    v, s, pv, ps = _out(arrs[0].size)
    _load().oracle_reduce_op(ptrs, _i64(len(arrs)), _i64(arrs[0].size), _i64(REDUCERS[reducer]), pv, ps)
    return v.reshape(shape), s.reshape(shape)


def lstm_cell(gates, c_prev):
    """gates [..., 4] (input, forget, cell, output pre-activations), c_prev [...] ->
    (c_new, h_new, scale_c) float64 arrays of c_prev's shape."""
    g, pg = _f32(gates); c, pc = _f32(c_prev)
    assert g.shape == c.shape + (4,)
    n = c.size
    cn, hn, sc = (np.empty(n, dtype=np.float64) for _ in range(3))
    _load().oracle_lstm_cell(pg, pc, _i64(n), cn.ctypes.data_as(_dp), hn.ctypes.data_as(_dp), sc.ctypes.data_as(_dp))
    return cn.reshape(c.shape), hn.reshape(c.shape), sc.reshape(c.shape)
