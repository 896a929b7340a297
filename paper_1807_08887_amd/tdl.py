"""ctypes binding of include/tofu_tdl.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes
from typing import Dict, List, Sequence, Tuple

from .binding import TOFU_MAX_DIMS, OpDesc, Region, Split, _check, _splits, load

MAX_VARS, MAX_INPUTS = 8, 4
_i64 = ctypes.c_int64


class Index(ctypes.Structure):
    _fields_ = [("coef", _i64 * MAX_VARS), ("offset", _i64)]


class Access(ctypes.Structure):
    _fields_ = [("ndim", ctypes.c_int32), ("size", _i64 * TOFU_MAX_DIMS), ("index", Index * TOFU_MAX_DIMS)]


class TdlOp(ctypes.Structure):
    _fields_ = [("n_vars", ctypes.c_int32), ("n_out", ctypes.c_int32), ("extent", _i64 * MAX_VARS),
                ("n_inputs", ctypes.c_int32), ("input", Access * MAX_INPUTS)]


class Interval(ctypes.Structure):
    _fields_ = [("lower_num", _i64 * MAX_VARS), ("upper_num", _i64 * MAX_VARS), ("den", _i64), ("constant", _i64)]


_ready = False


def _lib():
    global _ready
    lib = load()
    if not _ready:
        P = ctypes.POINTER
        i32 = ctypes.c_int32
        lib.tofu_tdl_from_op.argtypes = [P(OpDesc), P(TdlOp)]
        lib.tofu_tdl_symbolic.argtypes = [P(TdlOp), i32, i32, i32, i32, P(Interval)]
        lib.tofu_tdl_regions.argtypes = [P(TdlOp), P(Split), i32, P(Region), P(Region), P(_i64), P(_i64), P(i32)]
        lib.tofu_tdl_fetch_elements.argtypes = [P(TdlOp), i32, i32, i32, i32, P(_i64)]
        for n in ("tofu_tdl_from_op", "tofu_tdl_symbolic", "tofu_tdl_regions", "tofu_tdl_fetch_elements"):
            getattr(lib, n).restype = ctypes.c_int
        _ready = True
    return lib


def describe(extents: Sequence[int], n_out: int, inputs: Sequence[Tuple[Sequence[int], Sequence[Dict]]]) -> TdlOp:
    """extents: one per variable (output variables first); inputs: (tensor shape, [index per
    dimension]) with an index given as {variable position: coefficient, "c": constant}."""
    op = TdlOp()
    op.n_vars, op.n_out, op.n_inputs = len(extents), n_out, len(inputs)
    for v, e in enumerate(extents):
        op.extent[v] = e
    for i, (shape, exprs) in enumerate(inputs):
        op.input[i].ndim = len(shape)
        for d, (size, e) in enumerate(zip(shape, exprs)):
            op.input[i].size[d] = size
            for v, c in e.items():
                if v == "c":
                    op.input[i].index[d].offset = c
                else:
                    op.input[i].index[d].coef[v] = c
    return op


def from_op(desc: OpDesc) -> TdlOp:
    out = TdlOp()
    _check(_lib().tofu_tdl_from_op(ctypes.byref(desc), ctypes.byref(out)))
    return out


def symbolic(op: TdlOp, split_var: int, half: int, input_index: int, dim: int):
    """-> (lower numerators, upper numerators, denominator, constant), numerators per variable."""
    iv = Interval()
    _check(_lib().tofu_tdl_symbolic(ctypes.byref(op), split_var, half, input_index, dim, ctypes.byref(iv)))
    return [int(iv.lower_num[v]) for v in range(op.n_vars)], [int(iv.upper_num[v]) for v in range(op.n_vars)], int(iv.den), int(iv.constant)


def regions(op: TdlOp, splits: Sequence):
    sp, n = _splits(splits)
    out_box = Region()
    in_boxes = (Region * MAX_INPUTS)()
    cut_lo, cut_hi = (_i64 * (MAX_INPUTS * TOFU_MAX_DIMS))(), (_i64 * (MAX_INPUTS * TOFU_MAX_DIMS))()
    partial = ctypes.c_int32(0)
    _check(_lib().tofu_tdl_regions(ctypes.byref(op), sp, n, ctypes.byref(out_box), in_boxes, cut_lo, cut_hi, ctypes.byref(partial)))
    nd = [op.input[i].ndim for i in range(op.n_inputs)]
    return dict(out_box=out_box.box(), in_boxes=[in_boxes[i].box() for i in range(op.n_inputs)],
                cut_lo=[[int(cut_lo[i * TOFU_MAX_DIMS + d]) for d in range(nd[i])] for i in range(op.n_inputs)],
                cut_hi=[[int(cut_hi[i * TOFU_MAX_DIMS + d]) for d in range(nd[i])] for i in range(op.n_inputs)],
                is_partial=bool(partial.value))


def fetch_elements(op: TdlOp, var: int, k: int, input_index: int, part_dim: int) -> int:
    out = _i64(0)
    _check(_lib().tofu_tdl_fetch_elements(ctypes.byref(op), var, k, input_index, part_dim, ctypes.byref(out)))
    return int(out.value)
