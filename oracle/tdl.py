"""TEST INFRASTRUCTURE (oracle side): region analysis of operators given in the paper's tensor
description form (arXiv 1807.08887 Sec. 4.1-4.2), written out two ways that share nothing
with the HIP library:

  * brute force: run the operator's loop nest over a worker's share of the iteration space and
    mark every input coordinate it reads;
  * the symbolic interval arithmetic of Sec. 4.2 (Eq. 1 and the arithmetic table that follows
    it): an interval is <l_1..l_n, u_1..u_n, c> = [sum_i l_i X_i + c, sum_i u_i X_i + c] over the
    symbolic upper bounds X_i of the index variables; intervals can be shifted, scaled and added,
    products of intervals are an error.

An operator is a dict:
  vars    : list of (name, extent)            index variables, output ones first
  n_out   : how many of them index the output (the rest are reduction variables)
  inputs  : list of (tensor_shape, [index expression per tensor dimension]); an index expression
            is a dict {var_name: coefficient, ..., 1: constant} (an affine form, which is all the
            interval arithmetic can represent)

Reading where the paper's table is silent: scaling by a negative constant swaps the lower and
upper coefficient vectors (the table as printed keeps them in place, which would give an
interval whose ends are exchanged).
"""
from __future__ import annotations

import itertools
from fractions import Fraction

import numpy as np


# ----------------------------------------------------------------------------- descriptions
def shift_two(n=10):
    """B = lambda i: A[i + 2]   (the worked example of Sec. 4.2)."""
    return dict(vars=[("i", n)], n_out=1, inputs=[((n + 2,), [{"i": 1, 1: 2}])])


def conv1d(B, CI, CO, X, DX):
    """Fig. 1 / Fig. 3: out[b, co, x] = Sum(ci, dx: data[b, ci, x + dx] * filters[ci, co, dx])."""
    return dict(vars=[("b", B), ("co", CO), ("x", X), ("ci", CI), ("dx", DX)], n_out=3,
                inputs=[((B, CI, X + DX - 1), [{"b": 1}, {"ci": 1}, {"x": 1, "dx": 1}]),
                        ((CI, CO, DX), [{"ci": 1}, {"co": 1}, {"dx": 1}])])


def matmul(M, N, K):
    return dict(vars=[("m", M), ("n", N), ("k", K)], n_out=2,
                inputs=[((M, K), [{"m": 1}, {"k": 1}]), ((K, N), [{"k": 1}, {"n": 1}])])


def conv2d(batch, c_in, c_out, H, W, KH, KW, stride, pad):
    ho, wo = (H + 2 * pad - KH) // stride + 1, (W + 2 * pad - KW) // stride + 1
    return dict(vars=[("n", batch), ("co", c_out), ("h", ho), ("w", wo), ("ci", c_in), ("kh", KH), ("kw", KW)], n_out=4,
                inputs=[((batch, c_in, H, W), [{"n": 1}, {"ci": 1}, {"h": stride, "kh": 1, 1: -pad}, {"w": stride, "kw": 1, 1: -pad}]),
                        ((c_out, c_in, KH, KW), [{"co": 1}, {"ci": 1}, {"kh": 1}, {"kw": 1}])])


# ----------------------------------------------------------------------------- brute force
def _share(op, splits):
    """Index ranges left to one worker: splits = [(var_name, k, part)], each cutting the current range."""
    rng = {name: (0, ext) for name, ext in op["vars"]}
    for name, k, part in splits:
        lo, hi = rng[name]
        d = hi - lo
        rng[name] = (lo + (part * d) // k, lo + ((part + 1) * d) // k)
    return rng


def touched(op, splits):
    """Boolean masks (one per input, over the global tensor) of the coordinates the loop nest
    reads for the worker's share, plus per input and dimension how many accesses fell outside
    the tensor on the low / high side (those read zeros)."""
    rng = _share(op, splits)
    names = [n for n, _ in op["vars"]]
    masks = [np.zeros(shape, dtype=bool) for shape, _ in op["inputs"]]
    for point in itertools.product(*[range(*rng[n]) for n in names]):
        val = dict(zip(names, point))
        for mask, (shape, exprs) in zip(masks, op["inputs"]):
            coord = [sum(c * (val[v] if v != 1 else 1) for v, c in e.items()) for e in exprs]
            if all(0 <= c < s for c, s in zip(coord, shape)):
                mask[tuple(coord)] = True
    return masks


def bbox(mask):
    idx = np.argwhere(mask)
    return [(int(a), int(b) + 1) for a, b in zip(idx.min(0), idx.max(0))]


def fetch_elements(op, var, k, input_index, part_dim):
    """Communication of one basic strategy for one input (Appendix A.3, first situation): the
    operator is split k ways along `var`, the input tensor is held split k ways along its
    dimension `part_dim`; every worker fetches what it reads but does not hold.  Returns the
    number of elements fetched, summed over the workers, by marking coordinates."""
    shape = op["inputs"][input_index][0]
    total = 0
    for w in range(k):
        need = touched(op, [(var, k, w)])[input_index]
        held = np.zeros(shape, dtype=bool)
        sl = [slice(None)] * len(shape)
        sl[part_dim] = slice((w * shape[part_dim]) // k, ((w + 1) * shape[part_dim]) // k)
        held[tuple(sl)] = True
        total += int((need & ~held).sum())
    return total


# ----------------------------------------------------------------------------- symbolic intervals
class Interval:
    """<l, u, c> over the variables `names`: [sum l_i X_i + c, sum u_i X_i + c]."""

    def __init__(self, names, l=None, u=None, c=0):
        self.names = list(names)
        self.l = {n: Fraction(0) for n in names}
        self.u = {n: Fraction(0) for n in names}
        self.l.update(l or {})
        self.u.update(u or {})
        self.c = Fraction(c)

    @staticmethod
    def variable(names, name, lo=0, hi=1):
        """The index variable `name` ranging over [lo * X, hi * X]; (0, 1) is the whole range,
        (0, 1/2) and (1/2, 1) are the two workers' halves."""
        return Interval(names, {name: Fraction(lo)}, {name: Fraction(hi)})

    def shift(self, k):
        return Interval(self.names, self.l, self.u, self.c + k)

    def scale(self, k):
        k = Fraction(k)
        l = {n: v * k for n, v in self.l.items()}
        u = {n: v * k for n, v in self.u.items()}
        if k < 0:
            l, u = u, l
        return Interval(self.names, l, u, self.c * k)

    def add(self, other):
        if not isinstance(other, Interval):
            return self.shift(other)
        return Interval(self.names, {n: self.l[n] + other.l[n] for n in self.names},
                        {n: self.u[n] + other.u[n] for n in self.names}, self.c + other.c)

    def mul(self, other):
        if isinstance(other, Interval):
            raise ValueError("product of two intervals is not affine")
        return self.scale(other)

    def vector(self):
        return [self.l[n] for n in self.names] + [self.u[n] for n in self.names] + [self.c]

    def concrete(self, upper):
        """Inclusive integer range for concrete upper bounds X (dict name -> X = extent - 1 ...)."""
        lo = sum(self.l[n] * upper[n] for n in self.names) + self.c
        hi = sum(self.u[n] * upper[n] for n in self.names) + self.c
        return lo, hi


def symbolic_regions(op, split_var=None, half=0):
    """Symbolic interval of every input dimension when `split_var` (or nothing) is cut in
    halves and the worker takes half `half`: executes each index expression with the interval
    arithmetic above."""
    names = [n for n, _ in op["vars"]]
    env = {}
    for n in names:
        if n == split_var:
            env[n] = Interval.variable(names, n, *((0, Fraction(1, 2)) if half == 0 else (Fraction(1, 2), 1)))
        else:
            env[n] = Interval.variable(names, n)
    out = []
    for _, exprs in op["inputs"]:
        dims = []
        for e in exprs:
            acc = Interval(names)
            for v, coef in e.items():
                acc = acc.add(Fraction(coef)) if v == 1 else acc.add(env[v].mul(coef))
            dims.append(acc)
        out.append(dims)
    return out
