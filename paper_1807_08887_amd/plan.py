"""ctypes binding of include/tofu_plan.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes
from typing import List, Sequence, Tuple

from .binding import _check, load
from .tdl import MAX_INPUTS, TdlOp

_i32, _i64 = ctypes.c_int32, ctypes.c_int64


class PlanOp(ctypes.Structure):
    _fields_ = [("desc", TdlOp), ("input_tensor", _i32 * MAX_INPUTS), ("output_tensor", _i32), ("group", _i32)]


class PlanGraph(ctypes.Structure):
    _fields_ = [("n_tensors", _i32), ("n_ops", _i32), ("ops", ctypes.POINTER(PlanOp))]


_ready = False


def _lib():
    global _ready
    lib = load()
    if not _ready:
        P = ctypes.POINTER
        lib.tofu_plan_strategy_cost.argtypes = [P(PlanGraph), _i32, _i32, _i32, P(_i32), P(_i64)]
        lib.tofu_plan_cost.argtypes = [P(PlanGraph), _i32, P(_i32), P(_i32), P(_i64)]
        lib.tofu_plan_basic.argtypes = [P(PlanGraph), _i32, P(_i32), P(_i32), P(_i64), P(_i64)]
        lib.tofu_plan_recursive.argtypes = [P(PlanGraph), P(_i32), _i32, P(_i32), P(_i32), P(_i64), P(_i64)]
        from .binding import Split
        lib.tofu_plan_worker_splits.argtypes = [P(_i32), _i32, P(_i32), _i32, _i32, _i64, P(Split)]
        for n in ("tofu_plan_strategy_cost", "tofu_plan_cost", "tofu_plan_basic", "tofu_plan_recursive", "tofu_plan_worker_splits"):
            getattr(lib, n).restype = ctypes.c_int
        _ready = True
    return lib


def graph(n_tensors: int, ops: Sequence[Tuple[TdlOp, Sequence[int], int, int]]) -> PlanGraph:
    """ops: (description, input tensor ids, output tensor id, group) in group order."""
    arr = (PlanOp * max(1, len(ops)))()
    for o, (desc, ins, out, group) in enumerate(ops):
        arr[o].desc = desc
        for i, t in enumerate(ins):
            arr[o].input_tensor[i] = t
        arr[o].output_tensor, arr[o].group = out, group
    g = PlanGraph()
    g.n_tensors, g.n_ops, g.ops = n_tensors, len(ops), arr
    g._keep = arr            # the C struct holds only a pointer
    return g


def _ints(values: Sequence[int]):
    return (_i32 * max(1, len(values)))(*values)


def strategy_cost(g: PlanGraph, op: int, var: int, k: int, tensor_dim: Sequence[int]) -> int:
    out = _i64(0)
    _check(_lib().tofu_plan_strategy_cost(ctypes.byref(g), op, var, k, _ints(tensor_dim), ctypes.byref(out)))
    return int(out.value)


def cost(g: PlanGraph, k: int, tensor_dim: Sequence[int], op_var: Sequence[int]) -> int:
    out = _i64(0)
    _check(_lib().tofu_plan_cost(ctypes.byref(g), k, _ints(tensor_dim), _ints(op_var), ctypes.byref(out)))
    return int(out.value)


def basic(g: PlanGraph, k: int):
    """-> dict(tensor_dim, op_var, elements, configurations)."""
    dims, vars_ = (_i32 * g.n_tensors)(), (_i32 * g.n_ops)()
    el, conf = _i64(0), _i64(0)
    _check(_lib().tofu_plan_basic(ctypes.byref(g), k, dims, vars_, ctypes.byref(el), ctypes.byref(conf)))
    return dict(tensor_dim=list(dims), op_var=list(vars_), elements=int(el.value), configurations=int(conf.value))


def recursive(g: PlanGraph, ks: Sequence[int]):
    """-> dict(tensor_dim[step][tensor], op_var[step][op], step_elements[step], total)."""
    m = len(ks)
    dims, vars_ = (_i32 * (m * g.n_tensors))(), (_i32 * (m * g.n_ops))()
    steps, total = (_i64 * max(1, m))(), _i64(0)
    _check(_lib().tofu_plan_recursive(ctypes.byref(g), _ints(ks), m, dims, vars_, steps, ctypes.byref(total)))
    return dict(tensor_dim=[list(dims[s * g.n_tensors:(s + 1) * g.n_tensors]) for s in range(m)],
                op_var=[list(vars_[s * g.n_ops:(s + 1) * g.n_ops]) for s in range(m)],
                step_elements=[int(steps[s]) for s in range(m)], total=int(total.value))


def worker_splits(op_var_steps: Sequence[Sequence[int]], ks: Sequence[int], op: int, worker: int) -> List[Tuple[int, int, int]]:
    """tofu_plan_worker_splits: the split list of `worker`'s shard of operator `op` under a recursive plan."""
    from .binding import Split
    m, n_ops = len(ks), len(op_var_steps[0]) if op_var_steps else 0
    flat = _ints([v for step in op_var_steps for v in step])
    out = (Split * max(1, m))()
    _check(_lib().tofu_plan_worker_splits(flat, n_ops, _ints(ks), m, op, worker, out))
    return [(out[s].dim, out[s].k, out[s].shard) for s in range(m)]
