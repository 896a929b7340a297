"""CPU tests of the library's region analysis for operators in tensor-description form
(include/tofu_tdl.h) against the oracle's independent versions (oracle/tdl.py), the paper's
examples, and the hard-coded regions of the built-in operators.  No device call is made."""
import itertools
import os
from fractions import Fraction as F

import pytest

import paper_1807_08887_amd as tofu
from paper_1807_08887_amd import tdl as T
from oracle import tdl as O

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _to_lib(op):
    """The oracle's description dict as a library description."""
    names = [n for n, _ in op["vars"]]
    inputs = []
    for shape, exprs in op["inputs"]:
        inputs.append((shape, [{("c" if v == 1 else names.index(v)): c for v, c in e.items()} for e in exprs]))
    return T.describe([e for _, e in op["vars"]], op["n_out"], inputs)


OPS = [O.shift_two(10), O.conv1d(4, 6, 8, 12, 3), O.matmul(6, 8, 10), O.conv2d(2, 4, 4, 8, 6, 3, 3, 1, 1),
       O.conv2d(2, 2, 2, 9, 9, 2, 2, 2, 0),
       dict(vars=[("h", 8), ("kh", 3)], n_out=1, inputs=[((8,), [{"h": 1, "kh": -1, 1: 1}])])]


@pytest.mark.parametrize("op", OPS, ids=lambda o: "-".join(n for n, _ in o["vars"]))
def test_symbolic_vectors_match_the_oracle(op):
    lib = _to_lib(op)
    names = [n for n, _ in op["vars"]]
    for var, half in itertools.product([None] + names, range(2)):
        sym = O.symbolic_regions(op, var, half)
        for t, (shape, _) in enumerate(op["inputs"]):
            for d in range(len(shape)):
                lo, up, den, c = T.symbolic(lib, -1 if var is None else names.index(var), half, t, d)
                assert [F(v, den) for v in lo] + [F(v, den) for v in up] + [F(c)] == sym[t][d].vector(), (var, half, t, d)


@pytest.mark.parametrize("op", OPS, ids=lambda o: "-".join(n for n, _ in o["vars"]))
def test_concrete_regions_match_touched_coordinates(op):
    """Every one-step plan (k up to 3) and a sample of two-step plans: the library's clipped
    boxes are the bounding boxes of the coordinates the oracle's loop nest marks."""
    lib = _to_lib(op)
    names = [n for n, _ in op["vars"]]
    steps = [(n, k, s) for n, e in op["vars"] for k in range(1, min(e, 3) + 1) for s in range(k)]
    plans = [[st] for st in steps] + [[a, b] for a, b in itertools.product(steps[::3], steps[1::4])]
    for plan in plans:
        try:
            masks = O.touched(op, plan)
        except ZeroDivisionError:
            continue
        share = O._share(op, plan)
        if any(hi <= lo for lo, hi in share.values()):
            continue
        try:
            reg = T.regions(lib, [(names.index(n), k, s) for n, k, s in plan])
        except tofu.TofuError:
            # the library refuses to cut a range into more parts than it has elements
            assert any(k > 1 for _, k, _ in plan)
            continue
        assert reg["out_box"] == [share[n] for n in names[:op["n_out"]]]
        assert reg["is_partial"] == any(names.index(n) >= op["n_out"] and k > 1 for n, k, _ in plan)
        for t in range(len(op["inputs"])):
            if masks[t].any():
                box = O.bbox(masks[t])
                unit = all(abs(c) <= 1 for e in op["inputs"][t][1] for v, c in e.items() if v != 1)
                if unit:
                    assert reg["in_boxes"][t] == box, (plan, t)
                else:    # with a stride the last window of a range may stop short of the interval's end
                    assert all(a[0] <= b[0] and b[1] <= a[1] for a, b in zip(reg["in_boxes"][t], box))


def test_shift_two_and_cut_counts():
    lib = _to_lib(O.shift_two(10))
    rows = [[int(v) for v in l.split()] for l in open(os.path.join(GOLD, "shift_two.txt")) if l.strip() and not l.startswith("#")]
    for half, (_, _, in_lo, in_hi) in enumerate(rows):
        assert T.regions(lib, [(0, 2, half)])["in_boxes"][0] == [(in_lo, in_hi + 1)]
    # reads outside the tensor are reported, not hidden: conv 3x3 pad 1 reaches one row above and below
    cv = T.from_op(tofu.conv2d_desc(2, 3, 4, 8, 8))
    r = T.regions(cv, [])
    assert r["cut_lo"][0] == [0, 0, 1, 1] and r["cut_hi"][0] == [0, 0, 1, 1] and r["cut_lo"][1] == [0, 0, 0, 0]


def _builtin_ops():
    return [("matmul", tofu.matmul_desc(13, 9, 21), {0: 0, 1: 1, 2: 2}),
            ("conv2d", tofu.conv2d_desc(5, 7, 6, 11, 9), {0: 0, 1: 1, 2: 2, 3: 3, 4: 4}),
            ("conv2d-s2", tofu.conv2d_desc(4, 4, 4, 12, 13, KH=5, KW=3, stride=2, pad=2), {0: 0, 1: 1, 2: 2, 3: 3, 4: 4}),
            ("wgrad", tofu.wgrad_desc(6, 5, 7, 8, 10), {0: 0, 1: 1, 2: 4}),
            ("dgrad", tofu.dgrad_desc(5, 7, 6, 11, 9), {0: 0, 1: 1, 2: 2, 3: 3, 4: 4}),
            ("dgrad-p0", tofu.dgrad_desc(4, 4, 4, 9, 9, pad=0), {0: 0, 1: 1, 2: 2, 3: 3, 4: 4}),
            ("lstm", tofu.lstm_cell_desc(6, 10), {0: 0, 1: 1})]


@pytest.mark.parametrize("name,desc,var_of_dim", _builtin_ops(), ids=[n for n, _, _ in _builtin_ops()])
def test_builtin_operators_derive_the_hard_coded_regions(name, desc, var_of_dim):
    """tofu_op_regions' boxes and residual padding follow from the operator's description alone."""
    lib = T.from_op(desc)
    ext = {d: lib.extent[v] for d, v in var_of_dim.items()}
    steps = [(d, k, s) for d in var_of_dim for k in range(1, min(ext[d], 4) + 1) for s in range(k)]
    plans = [[]] + [[st] for st in steps] + [[a, b] for a, b in itertools.product(steps[::2], steps[::3])]
    for plan in plans:
        try:
            hard = tofu.op_regions(desc, plan)
        except tofu.TofuError:
            with pytest.raises(tofu.TofuError):
                T.regions(lib, [(var_of_dim[d], k, s) for d, k, s in plan])
            continue
        got = T.regions(lib, [(var_of_dim[d], k, s) for d, k, s in plan])
        assert got["in_boxes"] == hard["in_boxes"], (name, plan)
        assert got["is_partial"] == hard["is_partial"]
        assert got["out_box"] == hard["out_box"], (name, plan)
        if name not in ("matmul", "lstm"):     # residual padding = what the unclipped range cuts off, rows then columns
            assert got["cut_lo"][0][2:4] == hard["pad_lo"] and got["cut_hi"][0][2:4] == hard["pad_hi"], (name, plan)


def test_fetch_elements_match_the_oracle_and_the_lemma():
    for op in [O.matmul(8, 12, 16), O.conv1d(2, 4, 6, 12, 3), O.conv2d(2, 4, 4, 8, 6, 3, 3, 1, 1)]:
        lib = _to_lib(op)
        names = [n for n, _ in op["vars"]]
        for var, k in itertools.product(names, (2, 3)):
            if dict(op["vars"])[var] < k:
                continue
            for t, (shape, _) in enumerate(op["inputs"]):
                for d in range(len(shape)):
                    if shape[d] < k:
                        continue
                    assert T.fetch_elements(lib, names.index(var), k, t, d) == O.fetch_elements(op, var, k, t, d), (var, k, t, d)
    mm = _to_lib(O.matmul(8, 12, 16))
    assert T.fetch_elements(mm, 0, 2, 0, 0) == 0 and T.fetch_elements(mm, 0, 2, 0, 1) == 2 * (8 * 16) // 4
    assert T.fetch_elements(mm, 0, 2, 1, 0) == 2 * (16 * 12) // 2


def test_tdl_error_paths():
    bad = T.describe([4], 1, [((4,), [{0: 1}])])
    bad.n_vars = 0
    with pytest.raises(tofu.TofuError):
        T.regions(bad, [])
    ok = T.describe([4], 1, [((4,), [{0: 1}])])
    with pytest.raises(tofu.TofuError):
        T.regions(ok, [(1, 2, 0)])            # no such variable
    with pytest.raises(tofu.TofuError):
        T.symbolic(ok, 0, 2, 0, 0)            # half must be 0 or 1
    with pytest.raises(tofu.TofuError) as e:
        T.from_op(tofu.dgrad_desc(2, 2, 2, 9, 9, stride=2))
    assert e.value.status == -6
