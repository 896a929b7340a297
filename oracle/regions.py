"""TEST INFRASTRUCTURE (oracle side): shard ranges, shard regions and region fetch, written
out with Python integers and numpy slicing.  Independent of the HIP library: shares no code
with it and never imports it.

Follows arXiv 1807.08887:
  * Sec. 4.2: a partition strategy = the input regions each worker needs; Case-1 splits an
    output dimension (outputs are concatenated), Case-2 splits a reduction dimension
    (outputs are summed).  Regions follow from propagating the worker's index ranges
    through the operator's index expressions -- the concrete-range form of the paper's
    interval analysis (its worked example: B[i] = A[i+2], i in [0,9] split in halves).
  * Sec. 5.2 / Appendix A.1: a plan is a sequence of basic steps, each splitting one
    dimension among k_i parts of the range left by the previous steps.
  * Sec. 6: the fetch assembles a worker's input region from the blocks that hold it.

Ranges are half-open (lo, hi) pairs in global coordinates; the paper's inclusive [a,b] is
(a, b+1).

Readings where the paper is silent (also listed in the design notes):
  * uneven extents: part s of k covers [floor(s*D/k), floor((s+1)*D/k));
  * zero padding (absent from the paper's "valid" conv1d): coordinates of the needed window
    that lie outside the global input are zeros, reported as pad_lo / pad_hi, and the input
    box is the window clipped to the tensor.
"""
from __future__ import annotations

import numpy as np

# iteration dimensions of each operator: (output dims, reduction dims)
ITER_DIMS = {
    "matmul": (("M", "N"), ("K",)),
    "conv2d": (("N", "CO", "H", "W"), ("CI",)),
    "conv2d_wgrad": (("CO", "CI"), ("N",)),
    "conv2d_dgrad": (("N", "CI", "H", "W"), ("CO",)),     # H, W: rows / columns of the forward INPUT
    "lstm_cell": (("B", "H"), ()),                          # element-wise over (batch, hidden unit)
    "conv1d": (("B", "CO", "X"), ("CI",)),                  # Fig. 1: data [B, CI, X + DX - 1], filters [CI, CO, DX]
}


def shard_range(extent: int, k: int, shard: int):
    """Part `shard` of an even k-way split of [0, extent)."""
    if extent < 0 or k < 1 or not (0 <= shard < k) or k > extent:
        raise ValueError("invalid split")
    return (shard * extent) // k, ((shard + 1) * extent) // k


def conv_out_size(size: int, ksize: int, stride: int, pad: int) -> int:
    return (size + 2 * pad - ksize) // stride + 1


def iteration_extents(op: dict) -> dict:
    kind = op["kind"]
    if kind == "matmul":
        return {"M": op["M"], "N": op["N"], "K": op["K"]}
    if kind == "lstm_cell":
        return {"B": op["batch"], "H": op["hidden"]}
    if kind == "conv1d":
        return {"B": op["batch"], "CO": op["c_out"], "X": op["W"] - op["KW"] + 1, "CI": op["c_in"]}
    ho = conv_out_size(op["H"], op["KH"], op["stride"], op["pad"])
    wo = conv_out_size(op["W"], op["KW"], op["stride"], op["pad"])
    if kind == "conv2d":
        return {"N": op["batch"], "CO": op["c_out"], "H": ho, "W": wo, "CI": op["c_in"]}
    if kind == "conv2d_wgrad":
        return {"CO": op["c_out"], "CI": op["c_in"], "N": op["batch"]}
    if kind == "conv2d_dgrad":
        return {"N": op["batch"], "CI": op["c_in"], "H": op["H"], "W": op["W"], "CO": op["c_out"]}
    raise ValueError(kind)


def apply_splits(op: dict, splits):
    """Index range of every iteration dimension left to one worker after the plan `splits`
    = [(dim_name, k, shard), ...]; each step cuts the current range of its dimension."""
    ext = iteration_extents(op)
    rng = {d: (0, e) for d, e in ext.items()}
    for dim, k, shard in splits:
        if dim not in rng:
            raise ValueError(f"dimension {dim} cannot be split for {op['kind']}")
        lo, hi = rng[dim]
        a, b = shard_range(hi - lo, k, shard)
        rng[dim] = (lo + a, lo + b)
    return rng


def worker_splits(dims_per_step, ks, worker: int):
    """Split list of worker `worker` under a recursive plan (Appendix A.1: a plan is the sequence
    of basic plans; Sec. 5.2: step i cuts every worker group of step i-1 into k_i groups).  The
    k_1 * ... * k_m workers are numbered group by group: the step-1 group is the slowest-varying
    part of the worker number.  dims_per_step[i] is the dimension the operator is cut along at
    step i.  -> [(dim, k_i, which of the k_i parts), ...]."""
    group_size = 1
    for k in ks:
        group_size *= k
    if not 0 <= worker < group_size:
        raise ValueError("worker outside the plan's worker count")
    out = []
    for dim, k in zip(dims_per_step, ks):
        group_size //= k                      # workers in one group once this step has cut
        out.append((dim, k, worker // group_size))
        worker %= group_size
    return out


def _window(out_lo, out_hi, ksize, stride, pad, size):
    """Input coordinates touched by outputs [out_lo,out_hi) through index o*stride + d - pad,
    d in [0,ksize): the widened ("halo") range, its clipped part and the zero rows cut off."""
    need_lo = out_lo * stride - pad
    need_hi = (out_hi - 1) * stride + (ksize - 1) - pad + 1
    lo, hi = max(need_lo, 0), min(need_hi, size)
    return (lo, hi), lo - need_lo, need_hi - hi


def _window_back(in_lo, in_hi, ksize, stride, pad, out_size):
    """Output coordinates o whose window o*stride + d - pad, d in [0,ksize), reaches an input
    coordinate in [in_lo,in_hi): the range of dy a data-gradient shard reads.  Same return
    convention as _window; the cut-off counts are the window positions that fall outside dy."""
    need_lo = -((-(in_lo + pad - (ksize - 1))) // stride)          # ceil
    need_hi = (in_hi - 1 + pad) // stride + 1
    lo, hi = max(need_lo, 0), min(need_hi, out_size)
    return (lo, hi), lo - need_lo, need_hi - hi


def op_regions(op: dict, splits):
    """Regions of one shard: dict(out_box, in_boxes=[first, second], pad_lo, pad_hi, is_partial)."""
    kind = op["kind"]
    r = apply_splits(op, splits)
    _, red_dims = ITER_DIMS[kind]
    is_partial = any(dim in red_dims and k > 1 for dim, k, _ in splits)
    pad_lo, pad_hi = [0, 0], [0, 0]
    if kind == "matmul":
        out_box = [r["M"], r["N"]]
        in_boxes = [[r["M"], r["K"]], [r["K"], r["N"]]]
    elif kind == "conv2d":
        hbox, pad_lo[0], pad_hi[0] = _window(*r["H"], op["KH"], op["stride"], op["pad"], op["H"])
        wbox, pad_lo[1], pad_hi[1] = _window(*r["W"], op["KW"], op["stride"], op["pad"], op["W"])
        out_box = [r["N"], r["CO"], r["H"], r["W"]]
        in_boxes = [[r["N"], r["CI"], hbox, wbox],
                    [r["CO"], r["CI"], (0, op["KH"]), (0, op["KW"])]]
    elif kind == "conv2d_wgrad":
        ho = conv_out_size(op["H"], op["KH"], op["stride"], op["pad"])
        wo = conv_out_size(op["W"], op["KW"], op["stride"], op["pad"])
        hbox, pad_lo[0], pad_hi[0] = _window(0, ho, op["KH"], op["stride"], op["pad"], op["H"])
        wbox, pad_lo[1], pad_hi[1] = _window(0, wo, op["KW"], op["stride"], op["pad"], op["W"])
        out_box = [r["CO"], r["CI"], (0, op["KH"]), (0, op["KW"])]
        in_boxes = [[r["N"], r["CI"], hbox, wbox],
                    [r["N"], r["CO"], (0, ho), (0, wo)]]
    elif kind == "conv1d":        # data[b, ci, x + dx]: the x range widened by the window; the data tensor is that much longer
        x0, x1 = r["X"]
        out_box = [r["B"], r["CO"], r["X"]]
        in_boxes = [[r["B"], r["CI"], (x0, x1 + op["KW"] - 1)], [r["CI"], r["CO"], (0, op["KW"])]]
    elif kind == "lstm_cell":     # element-wise: every input is read exactly where the output is written
        out_box = [r["B"], r["H"]]
        in_boxes = [[r["B"], r["H"], (0, 4)], [r["B"], r["H"]]]
    elif kind == "conv2d_dgrad":
        ho = conv_out_size(op["H"], op["KH"], op["stride"], op["pad"])
        wo = conv_out_size(op["W"], op["KW"], op["stride"], op["pad"])
        hbox, pad_lo[0], pad_hi[0] = _window_back(*r["H"], op["KH"], op["stride"], op["pad"], ho)
        wbox, pad_lo[1], pad_hi[1] = _window_back(*r["W"], op["KW"], op["stride"], op["pad"], wo)
        out_box = [r["N"], r["CI"], r["H"], r["W"]]
        in_boxes = [[r["N"], r["CO"], hbox, wbox],
                    [r["CO"], r["CI"], (0, op["KH"]), (0, op["KW"])]]
    else:
        raise ValueError(kind)
    return dict(out_box=out_box, in_boxes=in_boxes, pad_lo=pad_lo, pad_hi=pad_hi,
                is_partial=is_partial, ranges=r)


def box_slices(box, origin=None):
    """numpy slices selecting global box `box` from an array whose element [0,..] sits at
    global coordinate `origin` (default: the array is the whole tensor)."""
    origin = origin or [0] * len(box)
    return tuple(slice(lo - o, hi - o) for (lo, hi), o in zip(box, origin))


def fetch(dst_box, sources):
    """Region fetch (Sec. 6): assemble global box `dst_box` from `sources` =
    [(array, box_of_that_array), ...].  Every coordinate of dst_box must be held by exactly
    one source.  Returns a dense float32 array of the box's shape."""
    shape = [hi - lo for lo, hi in dst_box]
    out = np.zeros(shape, dtype=np.float32)
    claimed = np.zeros(shape, dtype=np.int32)
    for arr, box in sources:
        inter = [(max(lo, blo), min(hi, bhi)) for (lo, hi), (blo, bhi) in zip(dst_box, box)]
        if any(hi <= lo for lo, hi in inter):
            continue
        dsl = box_slices(inter, [lo for lo, _ in dst_box])
        out[dsl] = arr[box_slices(inter, [lo for lo, _ in box])]
        claimed[dsl] += 1
    if (claimed == 0).any():
        raise ValueError("uncovered")
    if (claimed > 1).any():
        raise ValueError("overlap")
    return out
