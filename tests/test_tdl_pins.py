"""Pins of the oracle's region analysis for operators in tensor-description form (oracle/tdl.py):
the paper's worked examples, the symbolic interval arithmetic against brute-force marking of
touched coordinates, and the 1/2 and 1/4 communication fractions of Appendix A.3.  No GPU."""
import os
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import tdl

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    return [l.split() for l in open(os.path.join(GOLD, name)) if l.strip() and not l.startswith("#")]


def _ints(lo, hi):
    """Integer points of the real interval [lo, hi] as an inclusive pair."""
    return int(np.ceil(float(lo))), int(np.floor(float(hi)))


def test_shift_two_example_symbolic_and_brute_force():
    op = tdl.shift_two(10)
    rows = [[int(v) for v in r] for r in _rows("shift_two.txt")]
    for half, (out_lo, out_hi, in_lo, in_hi) in enumerate(rows):
        box = tdl.bbox(tdl.touched(op, [("i", 2, half)])[0])
        assert box == [(in_lo, in_hi + 1)]
        iv = tdl.symbolic_regions(op, "i", half)[0][0]
        # <l_i, u_i, c>: A is read over [l X + 2, u X + 2] with (l, u) = (0, 1/2) or (1/2, 1)
        assert iv.vector() == ([F(0), F(1, 2), F(2)] if half == 0 else [F(1, 2), F(1), F(2)])
        assert _ints(*iv.concrete({"i": 9})) == (in_lo, in_hi)


def test_conv1d_strategies_symbolic():
    """Sec. 4.2 Case-1 / Case-2 on Fig. 3's conv1d: the symbolic vectors say "half of data on b,
    all of filters", "half of data on ci and half of filters on ci", and the x split's halo."""
    op = tdl.conv1d(4, 6, 8, 12, 3)
    names = [n for n, _ in op["vars"]]
    col = {"data_b": (0, 0, "b"), "data_ci": (0, 1, "ci"), "data_x": (0, 2, "x"),
           "filters_ci": (1, 0, "ci"), "filters_co": (1, 1, "co"), "filters_dx": (1, 2, "dx")}
    keys = ["data_b", "data_ci", "data_x", "filters_ci", "filters_co", "filters_dx"]
    for row in _rows("conv1d_strategies.txt"):
        split, which = row[0], dict(zip(keys, row[1:7]))
        for half in range(2):
            sym = tdl.symbolic_regions(op, split, half)
            for key, (t, d, var) in col.items():
                iv = sym[t][d]
                lo_c, hi_c = (F(0), F(1, 2)) if half == 0 else (F(1, 2), F(1))
                if which[key] == "all":
                    want_l, want_u = {}, {var: F(1)}
                    if key == "data_x":
                        want_u = {"x": F(1), "dx": F(1)}
                elif which[key] == "half":
                    want_l, want_u = {var: lo_c}, {var: hi_c}
                else:   # halo: the worker's half of x widened by the whole window dx
                    want_l, want_u = {"x": lo_c}, {"x": hi_c, "dx": F(1)}
                nz = lambda d: {n: v for n, v in d.items() if v}
                assert nz(iv.l) == nz(want_l), (split, key, half)
                assert nz(iv.u) == nz(want_u), (split, key, half)
                assert iv.c == 0
    assert len(names) == 5


@pytest.mark.parametrize("op,even_vars", [
    (tdl.conv1d(4, 6, 8, 12, 4), ["b", "ci", "co", "x", "dx"]),
    (tdl.matmul(6, 8, 10), ["m", "n", "k"]),
    (tdl.conv2d(2, 4, 4, 8, 6, 3, 3, 1, 1), ["n", "co", "h", "w", "ci"]),
    (tdl.conv2d(2, 2, 2, 9, 9, 2, 2, 2, 0), ["n", "co", "h", "w", "ci", "kh", "kw"]),
    # an index that runs backwards (the data gradient's dy[h + pad - kh]): exercises scaling by -1
    (dict(vars=[("h", 8), ("kh", 3)], n_out=1, inputs=[((8,), [{"h": 1, "kh": -1, 1: 1}])]), ["h"]),
])
def test_symbolic_intervals_contain_and_match_touched_boxes(op, even_vars):
    """For every 2-way strategy the integer points of the symbolic interval, clipped to the
    tensor, contain the bounding box of the coordinates the loop nest touches, and are exactly
    that box when every index coefficient is +-1 (with a stride the real-valued half X/2 of an
    odd X over-approximates by less than one stride)."""
    upper = {n: e - 1 for n, e in op["vars"]}
    for var in even_vars:
        for half in range(2):
            sym = tdl.symbolic_regions(op, var, half)
            masks = tdl.touched(op, [(var, 2, half)])
            for t, (shape, _) in enumerate(op["inputs"]):
                box = tdl.bbox(masks[t])
                for d, size in enumerate(shape):
                    lo, hi = _ints(*sym[t][d].concrete(upper))
                    got = (max(lo, 0), min(hi, size - 1) + 1)
                    unit = all(abs(c) == 1 for v, c in op["inputs"][t][1][d].items() if v != 1)
                    if unit:
                        assert got == box[d], (var, half, t, d)
                    else:
                        stride = max(abs(c) for v, c in op["inputs"][t][1][d].items() if v != 1)
                        assert got[0] <= box[d][0] and box[d][1] <= got[1] and got[1] - box[d][1] < stride and box[d][0] - got[0] < stride


def test_interval_arithmetic_rules():
    names = ["x", "y"]
    x, y = tdl.Interval.variable(names, "x"), tdl.Interval.variable(names, "y")
    assert x.shift(3).vector() == [0, 0, 1, 0, 3]
    assert x.scale(2).add(y).shift(-1).vector() == [0, 0, 2, 1, -1]
    assert x.scale(F(1, 2)).vector() == [0, 0, F(1, 2), 0, 0]
    # scaling by a negative constant exchanges the ends: -x over [0, X] is [-X, 0]
    assert x.scale(-1).vector() == [-1, 0, 0, 0, 0]
    assert x.scale(-1).concrete({"x": 5, "y": 0}) == (-5, 0)
    with pytest.raises(ValueError):
        x.mul(y)


def test_fetch_fractions_of_the_cost_lemma():
    """Appendix A.3: per worker a 2-way strategy fetches 1/2 of an input it needs whole and
    1/4 of an input it needs half of along another dimension than the one it is held by;
    nothing when the two dimensions agree.  fetch_elements sums the two workers."""
    op = tdl.matmul(8, 12, 16)
    SA, SB = 8 * 16, 16 * 12
    assert tdl.fetch_elements(op, "m", 2, 0, 0) == 0                 # A needed by rows, held by rows
    assert tdl.fetch_elements(op, "m", 2, 0, 1) == 2 * SA // 4       # A needed by rows, held by columns
    assert tdl.fetch_elements(op, "m", 2, 1, 0) == 2 * SB // 2       # all of B needed, half held
    assert tdl.fetch_elements(op, "m", 2, 1, 1) == 2 * SB // 2
    assert tdl.fetch_elements(op, "k", 2, 0, 1) == 0 and tdl.fetch_elements(op, "k", 2, 1, 0) == 0
    # halo: the x split of conv1d with data held by x fetches only the window overlap (DX - 1 columns per worker)
    c = tdl.conv1d(2, 3, 4, 12, 3)
    assert tdl.fetch_elements(c, "x", 2, 0, 2) == 2 * 3 * (1 + 1)    # worker 0 lacks 1 column, worker 1 lacks 1
