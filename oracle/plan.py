"""TEST INFRASTRUCTURE (oracle side): communication cost of partition plans and the exhaustive
search for the cheapest one (arXiv 1807.08887 Sec. 5, Appendix A.1 and A.3), by marking
coordinates.  Shares nothing with the HIP library or its host code.

A graph is a list of nodes dict(op=<operator dict of oracle/tdl.py>, inputs=[tensor id per
input], output=<tensor id>, group=<int>).  The output tensor is indexed by the operator's output
variables in order.

Cost of a basic plan for k workers (Appendix A.3): every tensor is held cut k ways along one
dimension, every operator is cut k ways along one variable; worker w
  * fetches every coordinate its share of the operator reads that is not in its slab of the
    input tensor (first situation), and
  * sends away every coordinate its share writes that is not in its slab of the output tensor
    (second situation; with a reduction variable cut, every worker writes the whole output).
Both are counted here on boolean masks over the tensors.

Recursion (Sec. 5.2, the paper's figure of a matrix product cut twice), reading used: the graph
of the next step is that of worker group 0 -- every operator keeps its loop nest with the cut
variable restricted to group 0's share, and each of its input tensors becomes the bounding box
of what that share reads (own part and fetched "extra input" together), re-based to start at 0.
Step i's cost is counted once per group: delta_i = (k_1 * ... * k_{i-1}) * cost(p_i).
"""
from __future__ import annotations

import itertools

import numpy as np

from . import tdl


def _slab(shape, dim, k, w):
    held = np.zeros(shape, dtype=bool)
    sl = [slice(None)] * len(shape)
    sl[dim] = slice((w * shape[dim]) // k, ((w + 1) * shape[dim]) // k)
    held[tuple(sl)] = True
    return held


def written(op, splits):
    """Mask over the output tensor of the coordinates one worker's share of the loop nest writes."""
    rng = tdl._share(op, splits)
    names = [n for n, _ in op["vars"]][:op["n_out"]]
    shape = [e for _, e in op["vars"]][:op["n_out"]]
    mask = np.zeros(shape, dtype=bool)
    mask[tuple(slice(*rng[n]) for n in names)] = True
    return mask


def strategy_cost(op, var, k, in_dims, out_dim):
    """Elements moved when `op` is cut k ways along variable `var` (a name), its inputs are held
    cut along in_dims[i] and its output along out_dim."""
    total = 0
    for w in range(k):
        need = tdl.touched(op, [(var, k, w)])
        for mask, d in zip(need, in_dims):
            total += int((mask & ~_slab(mask.shape, d, k, w)).sum())
        out = written(op, [(var, k, w)])
        total += int((out & ~_slab(out.shape, out_dim, k, w)).sum())
    return total


def _node_cost(node, var, k, tensor_dim):
    return strategy_cost(node["op"], var, k, [tensor_dim[t] for t in node["inputs"]], tensor_dim[node["output"]])


def basic_cost(graph, k, tensor_dim, op_var):
    """Cost of a complete basic plan; op_var[o] is a variable position."""
    return sum(_node_cost(n, n["op"]["vars"][v][0], k, tensor_dim) for n, v in zip(graph, op_var))


def tensor_shapes(graph):
    """Per tensor id: the list of shapes the nodes see (one entry per use)."""
    shapes = {}
    for n in graph:
        for t, (shape, _) in zip(n["inputs"], n["op"]["inputs"]):
            shapes.setdefault(t, []).append(tuple(shape))
        out = tuple(e for _, e in n["op"]["vars"][:n["op"]["n_out"]])
        shapes.setdefault(n["output"], []).append(out)
    return shapes


def candidates(graph, k):
    """Per tensor the dimensions of extent >= k in every view; per node the variables of extent >= k."""
    shapes = tensor_shapes(graph)
    dims = {t: [d for d in range(len(v[0])) if all(s[d] >= k for s in v)] for t, v in shapes.items()}
    vars_ = [[i for i, (_, e) in enumerate(n["op"]["vars"]) if e >= k] for n in graph]
    return dims, vars_


def basic_brute(graph, k, separable=True):
    """Cheapest basic plan by enumeration.  Every assignment of tensor dimensions is visited;
    with separable=False every assignment of operator variables as well (the cost is a sum over
    operators, so given the tensors each operator may as well take its own cheapest variable --
    the two modes must agree).  -> (cost, number of tensor-dimension assignments visited)."""
    dims, vars_ = candidates(graph, k)
    ids = sorted(dims)
    table = {}

    def cost(o, v, td):
        node = graph[o]
        key = (o, v, tuple(td[t] for t in node["inputs"]), td[node["output"]])
        if key not in table:
            table[key] = _node_cost(node, node["op"]["vars"][v][0], k, td)
        return table[key]

    best, visited = None, 0
    for choice in itertools.product(*[dims[t] for t in ids]):
        td = dict(zip(ids, choice))
        visited += 1
        if separable:
            c = sum(min(cost(o, v, td) for v in vars_[o]) for o in range(len(graph)))
        else:
            c = min(sum(cost(o, v, td) for o, v in enumerate(vs)) for vs in itertools.product(*vars_))
        best = c if best is None or c < best else best
    return best, visited


def reduce_graph(graph, k, op_var):
    """Graph of worker group 0 after every node was cut k ways along op_var[o] (a position)."""
    out = []
    for node, v in zip(graph, op_var):
        op = node["op"]
        name = op["vars"][v][0]
        masks = tdl.touched(op, [(name, k, 0)])
        new_vars = [(n, (e // k if n == name else e)) for n, e in op["vars"]]
        new_inputs = []
        for mask, (shape, exprs) in zip(masks, op["inputs"]):
            box = tdl.bbox(mask)
            new_exprs = []
            for (lo, hi), e in zip(box, exprs):
                e = dict(e)
                e[1] = e.get(1, 0) - lo
                new_exprs.append(e)
            new_inputs.append((tuple(hi - lo for lo, hi in box), new_exprs))
        out.append(dict(node, op=dict(vars=new_vars, n_out=op["n_out"], inputs=new_inputs)))
    return out


def sequence_cost(graph, ks, tensor_dims, op_vars):
    """Per-step costs delta_i of a sequence of basic plans, and their sum."""
    deltas, groups = [], 1
    for k, td, ov in zip(ks, tensor_dims, op_vars):
        deltas.append(groups * basic_cost(graph, k, td, ov))
        groups *= k
        graph = reduce_graph(graph, k, ov)
    return deltas, sum(deltas)


# ----------------------------------------------------------------------------- example graphs
def mlp_graph(batch, widths, backward=True):
    """Fig. 5: layer l computes X_l = X_{l-1} . W_l; with `backward`, dX_{l-1} = dX_l . W_l^T and
    dW_l = X_{l-1}^T . dX_l join the forward operator's group.  Tensor ids: X_l -> l, W_l ->
    L + l (l >= 1), dX_l -> 2L + 1 + l, dW_l -> 3L + 1 + l.  -> (graph, number of tensors)."""
    L = len(widths) - 1
    X, W = (lambda l: l), (lambda l: L + l)
    dX, dW = (lambda l: 2 * L + 1 + l), (lambda l: 3 * L + 1 + l)
    g = []
    for l in range(1, L + 1):
        a, b = widths[l - 1], widths[l]
        g.append(dict(op=tdl.matmul(batch, b, a), inputs=[X(l - 1), W(l)], output=X(l), group=l))
        if backward:
            # dX_{l-1}[m, j] = Sum(n: dX_l[m, n] * W_l[j, n])
            g.append(dict(op=dict(vars=[("m", batch), ("j", a), ("n", b)], n_out=2,
                                  inputs=[((batch, b), [{"m": 1}, {"n": 1}]), ((a, b), [{"j": 1}, {"n": 1}])]),
                          inputs=[dX(l), W(l)], output=dX(l - 1), group=l))
            # dW_l[j, n] = Sum(m: X_{l-1}[m, j] * dX_l[m, n])
            g.append(dict(op=dict(vars=[("j", a), ("n", b), ("m", batch)], n_out=2,
                                  inputs=[((batch, a), [{"m": 1}, {"j": 1}]), ((batch, b), [{"m": 1}, {"n": 1}])]),
                          inputs=[X(l - 1), dX(l)], output=dW(l), group=l))
    return g, (4 * L + 2 if backward else 2 * L + 1)
