"""Pins for the CPU oracle: it is checked against what the paper prints, against closed
forms and invariants, against independent library routines (numpy matmul, torch conv2d and
autograd in fp64) and against brute force on tiny shapes.  No GPU, no HIP library."""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import tofu_synth as synth
from oracle import regions as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


# ------------------------------------------------------------------ split ranges
def test_shift_two_example_from_paper():
    """Sec. 4.2 worked example: halves of i in [0,9] need A over [2,6] and [7,11]."""
    rows = [[int(v) for v in r] for r in _rows("shift_two.txt")]
    extent = rows[-1][1] + 1
    for shard, (olo, ohi, ilo, ihi) in enumerate(rows):
        lo, hi = R.shard_range(extent, 2, shard)
        assert (lo, hi - 1) == (olo, ohi)
        # B[i] = A[i+2] is a window of size 1 shifted by +2 (pad = -2); A has extent+2 elements
        (a, b), cut_lo, cut_hi = R._window(lo, hi, 1, 1, -2, extent + 2)
        assert (a, b - 1) == (ilo, ihi) and cut_lo == 0 and cut_hi == 0


def test_shard_range_brute_force():
    for D in range(1, 65):
        for k in range(1, min(D, 8) + 1):
            parts = [R.shard_range(D, k, s) for s in range(k)]
            assert parts[0][0] == 0 and parts[-1][1] == D
            sizes = [hi - lo for lo, hi in parts]
            assert all(parts[i][1] == parts[i + 1][0] for i in range(k - 1))  # ordered, disjoint, no holes
            assert min(sizes) >= 1 and max(sizes) - min(sizes) <= 1
            assert sorted(sizes) == sorted([D // k + (1 if i < D % k else 0) for i in range(k)])


@pytest.mark.parametrize("bad", [(-1, 1, 0), (4, 0, 0), (4, 2, 2), (4, 2, -1), (3, 4, 0)])
def test_shard_range_rejects(bad):
    with pytest.raises(ValueError):
        R.shard_range(*bad)


def test_recursive_steps_make_grids():
    """Sec. 5.2: row split then column split = 2x2 grid; row then row = four row strips."""
    op = dict(kind="matmul", M=8, N=12, K=5)
    seen = set()
    for a, b in itertools.product(range(2), repeat=2):
        box = R.op_regions(op, [("M", 2, a), ("N", 2, b)])["out_box"]
        assert box == [(4 * a, 4 * a + 4), (6 * b, 6 * b + 6)]
        seen.add(tuple(box))
        strip = R.op_regions(op, [("M", 2, a), ("M", 2, b)])["out_box"]
        assert strip == [(2 * (2 * a + b), 2 * (2 * a + b) + 2), (0, 12)]
        assert strip[0] == R.shard_range(8, 4, 2 * a + b)
    assert len(seen) == 4


def test_after_i_steps_tensors_are_1_over_2_to_i():
    """Appendix A.1: after i two-way steps the sub-tensors have 1/2^i of the elements."""
    op = dict(kind="conv2d", batch=8, c_in=16, c_out=32, H=16, W=16, KH=1, KW=1, stride=1, pad=0)
    full = 8 * 32 * 16 * 16
    for dims in itertools.product(["N", "CO", "H", "W"], repeat=3):
        for i in range(1, 4):
            box = R.op_regions(op, [(d, 2, 1) for d in dims[:i]])["out_box"]
            assert np.prod([hi - lo for lo, hi in box]) * 2 ** i == full


def test_search_space_counts_from_paper():
    """Sec. 5.2: 20 even partitions of a 4-D tensor over 8 workers; 20^6; 4^6; 3*4^6."""
    gold = {k: int(v) for k, v in _rows("search_space_counts.txt")}
    op = dict(kind="conv2d", batch=8, c_in=3, c_out=16, H=32, W=64, KH=1, KW=1, stride=1, pad=0)
    shapes = set()
    for dims in itertools.product(["N", "CO", "H", "W"], repeat=3):
        box = R.op_regions(op, [(d, 2, 0) for d in dims])["out_box"]
        shapes.add(tuple(hi - lo for lo, hi in box))
    assert len(shapes) == gold["ways_4d_8workers"]
    assert gold["ways_4d_8workers"] ** 6 == gold["configs_no_recursion"]
    assert 4 ** 6 == gold["configs_per_step"] and 3 * 4 ** 6 == gold["configs_three_steps"]


# ------------------------------------------------------------------ input regions
def _touch_conv(op, ranges):
    """Naive loop nest over one worker's iteration ranges marking every input coordinate it
    reads (outside-tensor reads are the zero padding and are counted separately)."""
    x = np.zeros((op["batch"], op["c_in"], op["H"], op["W"]), dtype=bool)
    w = np.zeros((op["c_out"], op["c_in"], op["KH"], op["KW"]), dtype=bool)
    s, p = op["stride"], op["pad"]
    for n in range(*ranges["N"]):
        for co in range(*ranges["CO"]):
            for h in range(*ranges["H"]):
                for wo in range(*ranges["W"]):
                    for ci in range(*ranges["CI"]):
                        for kh in range(op["KH"]):
                            for kw in range(op["KW"]):
                                w[co, ci, kh, kw] = True
                                ih, iw = h * s + kh - p, wo * s + kw - p
                                if 0 <= ih < op["H"] and 0 <= iw < op["W"]:
                                    x[n, ci, ih, iw] = True
    return x, w


def _bbox(mask):
    idx = np.argwhere(mask)
    return [(int(a), int(b) + 1) for a, b in zip(idx.min(0), idx.max(0))]


@pytest.mark.parametrize("stride,pad,ksz", [(1, 1, 3), (1, 0, 3), (2, 1, 3), (1, 2, 5), (2, 0, 2)])
def test_conv_regions_match_touched_coordinates(stride, pad, ksz):
    op = dict(kind="conv2d", batch=2, c_in=3, c_out=4, H=9, W=7, KH=ksz, KW=ksz, stride=stride, pad=pad)
    for dim in ["N", "CO", "H", "W", "CI"]:
        ext = R.iteration_extents(op)[dim]
        for k in range(1, min(ext, 3) + 1):
            for s in range(k):
                reg = R.op_regions(op, [(dim, k, s)])
                xm, wm = _touch_conv(op, reg["ranges"])
                assert _bbox(xm) == [tuple(b) for b in reg["in_boxes"][0]]
                assert _bbox(wm) == [tuple(b) for b in reg["in_boxes"][1]]
                assert reg["is_partial"] == (dim == "CI" and k > 1)
                # residual padding = rows of the needed window that are outside the tensor
                (hlo, hhi) = reg["ranges"]["H"]
                assert reg["pad_lo"][0] == max(0, pad - hlo * stride)
                assert reg["pad_hi"][0] == max(0, (hhi - 1) * stride + ksz - 1 - pad - (op["H"] - 1))


def test_conv1d_strategies_from_paper():
    """Fig. 2 / Sec. 4.2: which part of data and filters each worker reads for a split of
    b, ci, co, x.  conv1d is our conv2d with W = KW = 1 and no padding; the paper's filters
    are indexed [ci,co,dx], ours [co,ci,dx,1]."""
    X, DX = 12, 3
    op = dict(kind="conv2d", batch=4, c_in=6, c_out=8, H=X + DX - 1, W=1, KH=DX, KW=1, stride=1, pad=0)
    name = {"b": "N", "ci": "CI", "co": "CO", "x": "H"}
    full_x = [(0, 4), (0, 6), (0, X + DX - 1), (0, 1)]
    full_w = [(0, 8), (0, 6), (0, DX), (0, 1)]
    for split, d_b, d_ci, d_x, f_ci, f_co, f_dx, combine in _rows("conv1d_strategies.txt"):
        regs = [R.op_regions(op, [(name[split], 2, s)]) for s in range(2)]
        assert all(r["is_partial"] == (combine == "sum") for r in regs)
        for col, (dimidx, which) in {"data_b": (0, d_b), "data_ci": (1, d_ci), "data_x": (2, d_x)}.items():
            parts = [r["in_boxes"][0][dimidx] for r in regs]
            lo, hi = full_x[dimidx]
            if which == "all":
                assert parts == [(lo, hi)] * 2, col
            elif which == "half":
                assert parts == [(lo, hi // 2), (hi // 2, hi)], col
            else:  # halo: the output half widened by the filter window (Fig. 1: x + dx)
                assert parts == [(0, X // 2 + DX - 1), (X // 2, X + DX - 1)], col
        for col, (dimidx, which) in {"filters_ci": (1, f_ci), "filters_co": (0, f_co), "filters_dx": (2, f_dx)}.items():
            parts = [r["in_boxes"][1][dimidx] for r in regs]
            lo, hi = full_w[dimidx]
            assert parts == ([(lo, hi)] * 2 if which == "all" else [(lo, hi // 2), (hi // 2, hi)]), col


def test_fetch_cost_fractions():
    """Appendix A.3 (Lemma 1): per worker, fetching an input NOT indexed by the split
    dimension moves half of it (the whole tensor is needed, half is local); an input that is
    indexed by it needs only its own half.  Checked as region volumes for the matmul."""
    op = dict(kind="matmul", M=16, N=24, K=32)
    reg = R.op_regions(op, [("M", 2, 0)])
    vol = lambda box: int(np.prod([hi - lo for lo, hi in box]))
    assert vol(reg["in_boxes"][1]) == 32 * 24          # B not indexed by M: whole tensor needed
    assert vol(reg["in_boxes"][0]) * 2 == 16 * 32      # A indexed by M: half
    reg = R.op_regions(op, [("K", 2, 1)])
    assert vol(reg["in_boxes"][0]) * 2 == 16 * 32 and vol(reg["in_boxes"][1]) * 2 == 32 * 24
    assert reg["is_partial"] and reg["out_box"] == [(0, 16), (0, 24)]


def test_wgrad_and_matmul_regions_brute_force():
    op = dict(kind="conv2d_wgrad", batch=5, c_in=3, c_out=4, H=6, W=5, KH=3, KW=3, stride=1, pad=1)
    for dim in ["CO", "CI", "N"]:
        for s in range(2):
            reg = R.op_regions(op, [(dim, 2, s)])
            r = reg["ranges"]
            assert reg["out_box"] == [r["CO"], r["CI"], (0, 3), (0, 3)]
            assert reg["in_boxes"][0] == [r["N"], r["CI"], (0, 6), (0, 5)]      # x: every row is read
            assert reg["in_boxes"][1] == [r["N"], r["CO"], (0, 6), (0, 5)]      # dy
            assert reg["pad_lo"] == [1, 1] and reg["pad_hi"] == [1, 1]
            assert reg["is_partial"] == (dim == "N")


# ------------------------------------------------------------------ fetch
def test_fetch_of_split_blocks_is_identity():
    t = synth.small_int(7, 0, (4, 6, 9), -50, 50)
    blocks = []
    for s in range(3):
        lo, hi = R.shard_range(9, 3, s)
        blocks.append((t[:, :, lo:hi].copy(), [(0, 4), (0, 6), (lo, hi)]))
    box = [(1, 4), (0, 6), (2, 8)]
    got = R.fetch(box, blocks)
    assert got.dtype == np.float32 and np.array_equal(got, t[1:4, :, 2:8])
    with pytest.raises(ValueError, match="uncovered"):
        R.fetch(box, blocks[:2])
    with pytest.raises(ValueError, match="overlap"):
        R.fetch(box, blocks + [blocks[1]])


# ------------------------------------------------------------------ matmul
def test_matmul_against_numpy_and_closed_forms():
    A = synth.uniform(1, 0, (7, 13), -1, 1)
    B = synth.uniform(1, 1, (13, 5), -1, 1)
    v, s = oracle.matmul_box(A, B)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    assert np.allclose(v, ref, rtol=0, atol=1e-13)
    assert np.allclose(s, np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64), rtol=0, atol=1e-13)
    # identity and all-ones
    assert np.array_equal(oracle.matmul_box(A, np.eye(13, dtype=np.float32))[0], A.astype(np.float64))
    assert np.array_equal(oracle.matmul_box(np.ones((3, 9), np.float32), np.ones((9, 4), np.float32))[0],
                          np.full((3, 4), 9.0))
    # small integers: exact against integer arithmetic
    Ai = synth.small_int(2, 0, (6, 11), -8, 8)
    Bi = synth.small_int(2, 1, (11, 9), -8, 8)
    assert np.array_equal(oracle.matmul_box(Ai, Bi)[0], (Ai.astype(np.int64) @ Bi.astype(np.int64)).astype(np.float64))
    # box / points / reduction range agree with slicing the full result
    vb, _ = oracle.matmul_box(A, B, box=((2, 6), (1, 4)))
    assert np.array_equal(vb, v[2:6, 1:4])
    pts = [(0, 0), (6, 4), (3, 2)]
    assert np.array_equal(oracle.matmul_pts(A, B, pts)[0], np.array([v[p] for p in pts]))
    vk, sk = oracle.matmul_box(A, B, krange=(4, 9))
    assert np.allclose(vk, A[:, 4:9].astype(np.float64) @ B[4:9].astype(np.float64), rtol=0, atol=1e-13)


# ------------------------------------------------------------------ conv2d
@pytest.mark.parametrize("stride,pad,kh,kw", [(1, 1, 3, 3), (1, 0, 3, 3), (2, 1, 3, 3), (1, 2, 5, 3), (2, 0, 2, 4)])
def test_conv2d_against_torch_fp64(stride, pad, kh, kw):
    x = synth.normal(3, 0, (2, 3, 9, 8), 1.0)
    w = synth.normal(3, 1, (4, 3, kh, kw), 0.5)
    v, s = oracle.conv2d_box(x, w, stride=stride, pad=pad)
    ref = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=stride, padding=pad).numpy()
    assert v.shape == ref.shape and np.allclose(v, ref, rtol=0, atol=1e-12)
    refs = F.conv2d(torch.from_numpy(x).double().abs(), torch.from_numpy(w).double().abs(), stride=stride,
                    padding=pad).numpy()
    assert np.allclose(s, refs, rtol=0, atol=1e-12)
    pts = synth.coords(5, 0, 20, v.shape)
    assert np.array_equal(oracle.conv2d_pts(x, w, pts, stride=stride, pad=pad)[0], v[tuple(pts.T)])


def test_conv2d_closed_forms():
    # delta kernel: centre tap 1 where co == ci -> y == x exactly
    x = synth.normal(4, 0, (2, 5, 6, 7), 1.0)
    w = np.zeros((5, 5, 3, 3), np.float32)
    w[np.arange(5), np.arange(5), 1, 1] = 1.0
    assert np.array_equal(oracle.conv2d_box(x, w, pad=1)[0], x.astype(np.float64))
    # a single off-centre tap shifts the image the way cross-correlation (x+dx) does, not convolution
    w2 = np.zeros((1, 1, 3, 3), np.float32); w2[0, 0, 0, 2] = 1.0     # reads x[h-1, w+1]
    img = synth.small_int(4, 1, (1, 1, 5, 5), 0, 9)
    y = oracle.conv2d_box(img, w2, pad=1)[0]
    assert np.array_equal(y[0, 0, 1:, :-1], img[0, 0, :-1, 1:].astype(np.float64)) and not y[0, 0, 0].any()
    # all ones: C_in * (9 interior, 6 edge, 4 corner)
    y = oracle.conv2d_box(np.ones((1, 4, 5, 6), np.float32), np.ones((2, 4, 3, 3), np.float32), pad=1)[0]
    assert (y[:, :, 1:-1, 1:-1] == 36).all() and (y[:, :, 0, 1:-1] == 24).all() and (y[:, :, 1:-1, 0] == 24).all()
    assert y[0, 0, 0, 0] == y[0, 1, -1, -1] == y[0, 0, 0, -1] == 16
    # 1x1 image with 3x3/pad 1 only sees the centre tap: reduces to a matmul
    x1 = synth.normal(4, 2, (6, 5, 1, 1), 1.0)
    w1 = synth.normal(4, 3, (7, 5, 3, 3), 1.0)
    mm = oracle.matmul_box(x1[:, :, 0, 0], np.ascontiguousarray(w1[:, :, 1, 1].T))[0]
    assert np.array_equal(oracle.conv2d_box(x1, w1, pad=1)[0][:, :, 0, 0], mm)


# ------------------------------------------------------------------ wgrad
@pytest.mark.parametrize("stride,pad,kh,kw", [(1, 1, 3, 3), (1, 0, 3, 3), (2, 1, 3, 3), (1, 1, 2, 3)])
def test_wgrad_against_torch_autograd_fp64(stride, pad, kh, kw):
    x = synth.normal(6, 0, (3, 2, 7, 6), 1.0)
    w = torch.zeros(4, 2, kh, kw, dtype=torch.float64, requires_grad=True)
    y = F.conv2d(torch.from_numpy(x).double(), w, stride=stride, padding=pad)
    dy = synth.normal(6, 1, tuple(y.shape), 1.0)
    (y * torch.from_numpy(dy).double()).sum().backward()
    v, s = oracle.wgrad_box(x, dy, kh, kw, stride=stride, pad=pad)
    assert np.allclose(v, w.grad.numpy(), rtol=0, atol=1e-12)
    # the tolerance scale S = sum |dy * x| is the same gradient of the absolute values (torch, fp64): pinned exactly,
    # so that an inflated S cannot loosen the parity bar unnoticed
    w2 = torch.zeros(4, 2, kh, kw, dtype=torch.float64, requires_grad=True)
    (F.conv2d(torch.from_numpy(x).double().abs(), w2, stride=stride, padding=pad) * torch.from_numpy(dy).double().abs()).sum().backward()
    assert np.allclose(s, w2.grad.numpy(), rtol=0, atol=1e-12)
    pts = synth.coords(6, 2, 10, v.shape)
    assert np.array_equal(oracle.wgrad_pts(x, dy, kh, kw, pts, stride=stride, pad=pad)[0], v[tuple(pts.T)])


def test_wgrad_adjoint_identity_and_closed_form():
    """<dy, conv(x,w)> == <wgrad(x,dy), w> ties the gradient to the forward definition."""
    x = synth.normal(8, 0, (2, 3, 6, 5), 1.0)
    w = synth.normal(8, 1, (4, 3, 3, 3), 1.0)
    dy = synth.normal(8, 2, (2, 4, 6, 5), 1.0)
    lhs = (dy.astype(np.float64) * oracle.conv2d_box(x, w, pad=1)[0]).sum()
    rhs = (oracle.wgrad_box(x, dy, 3, 3, pad=1)[0] * w.astype(np.float64)).sum()
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # all ones, N=2, 4x5 image: centre tap sees H*W, edge taps (H-1)*W or H*(W-1), corners (H-1)(W-1)
    dw = oracle.wgrad_box(np.ones((2, 1, 4, 5), np.float32), np.ones((2, 1, 4, 5), np.float32), 3, 3, pad=1)[0][0, 0]
    assert np.array_equal(dw, 2.0 * np.array([[12, 15, 12], [16, 20, 16], [12, 15, 12]]))


# ------------------------------------------------------------------ dgrad
@pytest.mark.parametrize("stride,pad,kh,kw", [(1, 1, 3, 3), (1, 0, 3, 3), (2, 1, 3, 3), (1, 1, 2, 3), (2, 0, 3, 3)])
def test_dgrad_against_torch_autograd_fp64(stride, pad, kh, kw):
    x = torch.zeros(3, 2, 7, 6, dtype=torch.float64, requires_grad=True)
    w = synth.normal(12, 0, (4, 2, kh, kw), 1.0)
    y = F.conv2d(x, torch.from_numpy(w).double(), stride=stride, padding=pad)
    dy = synth.normal(12, 1, tuple(y.shape), 1.0)
    (y * torch.from_numpy(dy).double()).sum().backward()
    v, s = oracle.dgrad_box(dy, w, 7, 6, stride=stride, pad=pad)
    assert np.allclose(v, x.grad.numpy(), rtol=0, atol=1e-12)
    # S = sum |dy * w| pinned exactly: the same gradient of the absolute values (torch, fp64)
    x2 = torch.zeros(3, 2, 7, 6, dtype=torch.float64, requires_grad=True)
    (F.conv2d(x2, torch.from_numpy(w).double().abs(), stride=stride, padding=pad) * torch.from_numpy(dy).double().abs()).sum().backward()
    assert np.allclose(s, x2.grad.numpy(), rtol=0, atol=1e-12)
    pts = synth.coords(12, 2, 10, v.shape)
    assert np.array_equal(oracle.dgrad_pts(dy, w, 7, 6, pts, stride=stride, pad=pad)[0], v[tuple(pts.T)])
    # a restricted output-channel range is that channel block's contribution
    a = oracle.dgrad_box(dy, w, 7, 6, stride=stride, pad=pad, corange=(0, 1))[0]
    b = oracle.dgrad_box(dy, w, 7, 6, stride=stride, pad=pad, corange=(1, 4))[0]
    assert np.allclose(a + b, v, rtol=0, atol=1e-12)


def test_dgrad_adjoint_identity_and_closed_forms():
    """<dgrad(dy,w), x> == <dy, conv(x,w)> ties the gradient to the forward definition."""
    x = synth.normal(13, 0, (2, 3, 6, 5), 1.0)
    w = synth.normal(13, 1, (4, 3, 3, 3), 1.0)
    dy = synth.normal(13, 2, (2, 4, 6, 5), 1.0)
    lhs = (oracle.dgrad_box(dy, w, 6, 5, pad=1)[0] * x.astype(np.float64)).sum()
    rhs = (dy.astype(np.float64) * oracle.conv2d_box(x, w, pad=1)[0]).sum()
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))
    # all ones, 4x5 image, 3 output channels: every pixel gets one term per tap whose output position exists
    v = oracle.dgrad_box(np.ones((1, 3, 4, 5), np.float32), np.ones((3, 2, 3, 3), np.float32), 4, 5, pad=1)[0]
    want = 3.0 * np.array([[4, 6, 6, 6, 4], [6, 9, 9, 9, 6], [6, 9, 9, 9, 6], [4, 6, 6, 6, 4]])
    assert np.array_equal(v[0, 0], want) and np.array_equal(v[0, 1], want)
    # centre-tap delta filters: dx[ci] = sum_co dy[co] * w[co,ci,1,1]
    wd = np.zeros((2, 2, 3, 3), np.float32)
    wd[0, 1, 1, 1], wd[1, 0, 1, 1] = 2.0, -3.0
    d = synth.small_int(13, 3, (1, 2, 4, 4), -3, 3)
    v = oracle.dgrad_box(d, wd, 4, 4, pad=1)[0]
    assert np.array_equal(v[0, 1], 2.0 * d[0, 0]) and np.array_equal(v[0, 0], -3.0 * d[0, 1])
    # orientation: the forward tap (kh,kw) = (0,2) reads x[h-1, w+1], so dy[h,w] lands on dx[h-1, w+1]
    wo = np.zeros((1, 1, 3, 3), np.float32)
    wo[0, 0, 0, 2] = 1.0
    d = np.zeros((1, 1, 4, 4), np.float32)
    d[0, 0, 2, 1] = 5.0
    v = oracle.dgrad_box(d, wo, 4, 4, pad=1)[0]
    want = np.zeros((4, 4))
    want[1, 2] = 5.0
    assert np.array_equal(v[0, 0], want)
    # 1x1 image, pad 1: only the centre tap survives and the operator is dy . W[:, :, 1, 1]
    d1 = synth.normal(13, 4, (6, 7, 1, 1), 1.0)
    w1 = synth.normal(13, 5, (7, 5, 3, 3), 1.0)
    mm = oracle.matmul_box(d1[:, :, 0, 0], np.ascontiguousarray(w1[:, :, 1, 1]))[0]
    assert np.array_equal(oracle.dgrad_box(d1, w1, 1, 1, pad=1)[0][:, :, 0, 0], mm)


def _touch_dgrad(op, ranges):
    """Mark every dy / w element the defining loop nest reads for the dx box of `ranges`."""
    s, p = op["stride"], op["pad"]
    ho, wo_ = R.conv_out_size(op["H"], op["KH"], s, p), R.conv_out_size(op["W"], op["KW"], s, p)
    dy = np.zeros((op["batch"], op["c_out"], ho, wo_), dtype=bool)
    w = np.zeros((op["c_out"], op["c_in"], op["KH"], op["KW"]), dtype=bool)
    for n in range(*ranges["N"]):
        for ci in range(*ranges["CI"]):
            for ih in range(*ranges["H"]):
                for iw in range(*ranges["W"]):
                    for co in range(*ranges["CO"]):
                        for h in range(ho):              # every forward output position whose window covers (ih, iw)
                            for ww in range(wo_):
                                kh, kw = ih - h * s + p, iw - ww * s + p
                                if 0 <= kh < op["KH"] and 0 <= kw < op["KW"]:
                                    dy[n, co, h, ww] = True
                                    w[co, ci, kh, kw] = True
    return dy, w


@pytest.mark.parametrize("stride,pad,ksz", [(1, 1, 3), (1, 0, 3), (1, 2, 5)])
def test_dgrad_regions_match_touched_coordinates(stride, pad, ksz):
    op = dict(kind="conv2d_dgrad", batch=2, c_in=3, c_out=4, H=9, W=7, KH=ksz, KW=ksz, stride=stride, pad=pad)
    for dim in ["N", "CI", "H", "W", "CO"]:
        ext = R.iteration_extents(op)[dim]
        for k in range(1, min(ext, 3) + 1):
            for s in range(k):
                reg = R.op_regions(op, [(dim, k, s)])
                dm, wm = _touch_dgrad(op, reg["ranges"])
                assert _bbox(dm) == [tuple(b) for b in reg["in_boxes"][0]], (dim, k, s)
                assert reg["is_partial"] == (dim == "CO" and k > 1)
                if dim not in ("H", "W"):   # spatial shards may not use every tap against a clipped border
                    assert _bbox(wm) == [tuple(b) for b in reg["in_boxes"][1]]
                # residual padding: window positions of the needed dy rows that fall outside dy
                (hlo, hhi) = reg["ranges"]["H"]
                ho = R.conv_out_size(op["H"], ksz, stride, pad)
                assert reg["pad_lo"][0] == max(0, (ksz - 1 - pad) - hlo)
                assert reg["pad_hi"][0] == max(0, hhi - 1 + pad - (ho - 1))


# ------------------------------------------------------------------ reduce
def test_reduce_pins():
    parts = [synth.normal(9, j, (5, 33), 3.0) for j in range(8)]
    v, s = oracle.reduce(parts)
    assert np.allclose(v, np.sum(np.stack(parts).astype(np.float64), axis=0), rtol=0, atol=1e-13)
    assert np.allclose(s, np.sum(np.abs(np.stack(parts)).astype(np.float64), axis=0), rtol=0, atol=1e-13)
    assert np.array_equal(oracle.reduce(parts[:1])[0], parts[0].astype(np.float64))   # k = 1 is a copy
    ints = [synth.small_int(9, 20 + j, (4, 4), -100, 100) for j in range(3)]
    assert np.array_equal(oracle.reduce(ints)[0], (ints[0] + ints[1] + ints[2]).astype(np.float64))


def test_reduce_other_reducers_pins():
    """Max / Min / Prod (the description language's other built-in reducers) against numpy."""
    parts = [synth.normal(9, 40 + j, (7, 19), 2.0) for j in range(5)]
    st = np.stack(parts).astype(np.float64)
    assert np.array_equal(oracle.reduce_op(parts, "max")[0], st.max(axis=0))
    assert np.array_equal(oracle.reduce_op(parts, "min")[0], st.min(axis=0))
    v, s = oracle.reduce_op(parts, "prod")
    assert np.allclose(v, st.prod(axis=0), rtol=1e-14, atol=0) and np.array_equal(s, np.abs(v))
    ints = [synth.small_int(9, 50 + j, (6, 6), -5, 5) for j in range(4)]
    assert np.array_equal(oracle.reduce_op(ints, "prod")[0], (ints[0] * ints[1] * ints[2] * ints[3]).astype(np.float64))
    assert np.array_equal(oracle.reduce_op(parts[:1], "max")[0], parts[0].astype(np.float64))   # k = 1 is a copy
    # a NaN is skipped while another input has a number; all-NaN stays NaN
    a = np.array([np.nan, 1.0, np.nan], np.float32); b = np.array([2.0, np.nan, np.nan], np.float32)
    v = oracle.reduce_op([a, b], "max")[0]
    assert v[0] == 2.0 and v[1] == 1.0 and np.isnan(v[2])
    # Max over a K split is the partition-n-reduce form of a max-reducing operator: max over halves
    x = synth.normal(9, 60, (4, 10), 1.0)
    assert np.array_equal(oracle.reduce_op([x[:, :5].max(axis=1), x[:, 5:].max(axis=1)], "max")[0], x.max(axis=1).astype(np.float64))


# ------------------------------------------------------------------ the partition-n-reduce invariant
def _assemble(op, dim, k, evaluate):
    """Concatenate (Case-1) or sum (Case-2) the k shards produced by evaluate(region)."""
    full_box = R.op_regions(op, [])["out_box"]
    out = np.zeros([hi - lo for lo, hi in full_box])
    for s in range(k):
        reg = R.op_regions(op, [(dim, k, s)])
        part = evaluate(reg)
        sl = R.box_slices(reg["out_box"])
        out[sl] = out[sl] + part if reg["is_partial"] else part
    return out


@pytest.mark.parametrize("k", [2, 3, 4, 8])
def test_pnr_invariant_on_the_oracle(k):
    """Sec. 3.1: O is the concatenation or the element-wise sum of the workers' outputs.
    Small-integer data keeps every fp64 sum exact, so equality is bit-exact."""
    A = synth.small_int(10, 0, (8, 16), -4, 4); B = synth.small_int(10, 1, (16, 9), -4, 4)
    op = dict(kind="matmul", M=8, N=9, K=16)
    full = oracle.matmul_box(A, B)[0]
    for dim in ["M", "N", "K"]:
        got = _assemble(op, dim, k, lambda reg: oracle.matmul_box(A, B, box=reg["out_box"], krange=reg["ranges"]["K"])[0])
        assert np.array_equal(got, full), dim
    x = synth.small_int(10, 2, (8, 8, 9, 8), -3, 3); w = synth.small_int(10, 3, (8, 8, 3, 3), -3, 3)
    op = dict(kind="conv2d", batch=8, c_in=8, c_out=8, H=9, W=8, KH=3, KW=3, stride=1, pad=1)
    full = oracle.conv2d_box(x, w, pad=1)[0]
    for dim in ["N", "CO", "H", "W", "CI"]:
        got = _assemble(op, dim, k, lambda reg: oracle.conv2d_box(x, w, pad=1, box=reg["out_box"],
                                                                  cirange=reg["ranges"]["CI"])[0])
        assert np.array_equal(got, full), dim
    dy = synth.small_int(10, 4, (8, 8, 9, 8), -3, 3)
    op["kind"] = "conv2d_wgrad"
    full = oracle.wgrad_box(x, dy, 3, 3, pad=1)[0]
    for dim in ["CO", "CI", "N"]:
        got = _assemble(op, dim, k, lambda reg: oracle.wgrad_box(x, dy, 3, 3, pad=1, box=reg["out_box"],
                                                                 nrange=reg["ranges"]["N"])[0])
        assert np.array_equal(got, full), dim
    op["kind"] = "conv2d_dgrad"
    full = oracle.dgrad_box(dy, w, 9, 8, pad=1)[0]
    for dim in ["N", "CI", "H", "W", "CO"]:
        got = _assemble(op, dim, k, lambda reg: oracle.dgrad_box(dy, w, 9, 8, pad=1, box=reg["out_box"],
                                                                 corange=reg["ranges"]["CO"])[0])
        assert np.array_equal(got, full), dim


def test_shard_computed_from_its_fetched_region_only():
    """A worker must be able to compute its H-split shard from the fetched (halo-widened)
    region alone, with the residual padding the regions report: run the unpartitioned
    definition on the fetched block, padded by hand, and compare with the full result."""
    x = synth.small_int(11, 0, (2, 3, 10, 6), -3, 3); w = synth.small_int(11, 1, (4, 3, 3, 3), -3, 3)
    op = dict(kind="conv2d", batch=2, c_in=3, c_out=4, H=10, W=6, KH=3, KW=3, stride=1, pad=1)
    full = oracle.conv2d_box(x, w, pad=1)[0]
    own = [(x[:, :, lo:hi].copy(), [(0, 2), (0, 3), (lo, hi), (0, 6)]) for lo, hi in (R.shard_range(10, 2, s) for s in range(2))]
    for s in range(2):
        reg = R.op_regions(op, [("H", 2, s)])
        block = R.fetch(reg["in_boxes"][0], own)
        padded = np.pad(block, ((0, 0), (0, 0), (reg["pad_lo"][0], reg["pad_hi"][0]), (reg["pad_lo"][1], reg["pad_hi"][1])))
        y = oracle.conv2d_box(padded, w, pad=0)[0]
        assert np.array_equal(y, full[R.box_slices(reg["out_box"])])


# ------------------------------------------------------------------ the input generator
def test_synth_is_counter_based_and_plausible():
    a = synth.normal(1, 0, (1000, 100), 2.0)
    assert a.dtype == np.float32 and abs(a.mean()) < 0.02 and abs(a.std() - 2.0) < 0.02
    assert np.array_equal(a, synth.normal(1, 0, (1000, 100), 2.0))
    assert not np.array_equal(a, synth.normal(1, 1, (1000, 100), 2.0))
    u = synth.uniform(1, 2, (100000,), -1 / 128, 1 / 128)
    assert u.min() > -1 / 128 and u.max() < 1 / 128 and abs(u.var() * 3 * 128 * 128 - 1) < 0.02
    i = synth.small_int(1, 3, (10000,), -3, 3)
    assert set(np.unique(i)) == set(range(-3, 4))


def test_synth_random_access_and_device_forms_agree():
    """A tensor too large to draw whole on the host is drawn on the device and, for the oracle,
    at the coordinates it needs: all three forms give the same bits."""
    full = synth.uniform(7, 3, (37, 53), -0.25, 0.5)
    idx = np.array([0, 1, 52, 53, 1000, 37 * 53 - 1])
    assert np.array_equal(synth.uniform_at(7, 3, idx, -0.25, 0.5), full.ravel()[idx])
    t = synth.uniform_torch(7, 3, torch.arange(37 * 53, dtype=torch.int64).reshape(37, 53), -0.25, 0.5)
    assert np.array_equal(t.numpy(), full)
    big = torch.tensor([2 ** 40 + 12345, 2 ** 33], dtype=torch.int64)
    assert np.array_equal(synth.uniform_torch(9, 1, big, -1, 1).numpy(), synth.uniform_at(9, 1, big.numpy(), -1, 1))


def test_lstm_cell_against_torch_fp64_and_closed_forms():
    """The element-wise stage after the gate GEMM, against torch's fp64 formulas and at points
    where the result is known in closed form."""
    g = synth.normal(14, 0, (5, 9, 4), 2.0)
    c = synth.normal(14, 1, (5, 9), 1.0)
    cn, hn, sc = oracle.lstm_cell(g, c)
    tg, tc = torch.from_numpy(g).double(), torch.from_numpy(c).double()
    i, f, gg, o = (tg[..., k] for k in range(4))
    want_c = torch.sigmoid(f) * tc + torch.sigmoid(i) * torch.tanh(gg)
    want_h = torch.sigmoid(o) * torch.tanh(want_c)
    assert np.allclose(cn, want_c.numpy(), rtol=0, atol=1e-14) and np.allclose(hn, want_h.numpy(), rtol=0, atol=1e-14)
    # the tolerance scale of the cell state, |sig(f) c| + |sig(i) tanh(g)|, pinned exactly (torch, fp64)
    want_sc = (torch.sigmoid(f) * tc).abs() + (torch.sigmoid(i) * torch.tanh(gg)).abs()
    assert np.allclose(sc, want_sc.numpy(), rtol=0, atol=1e-14)
    # all pre-activations zero: every sigmoid is 1/2 and tanh(0) = 0
    z = np.zeros((3, 4), np.float32)
    cz, hz, _ = oracle.lstm_cell(z, np.array([2.0, -4.0, 0.0], np.float32))
    assert np.array_equal(cz, [1.0, -2.0, 0.0]) and np.allclose(hz, 0.5 * np.tanh([1.0, -2.0, 0.0]), rtol=0, atol=1e-16)
    # gate order (input, forget, cell, output): a wide-open forget gate alone carries the cell through,
    # a wide-open input gate alone writes tanh(g), a closed output gate silences h
    big = 40.0
    g1 = np.array([[-big, big, 0.3, big]], np.float32)
    c1, h1, _ = oracle.lstm_cell(g1, np.array([0.7], np.float32))
    assert abs(c1[0] - np.float64(np.float32(0.7))) < 1e-15 and abs(h1[0] - np.tanh(np.float64(np.float32(0.7)))) < 1e-15
    g2 = np.array([[big, -big, 0.3, -big]], np.float32)
    c2, h2, _ = oracle.lstm_cell(g2, np.array([0.7], np.float32))
    assert abs(c2[0] - np.tanh(np.float64(np.float32(0.3)))) < 1e-15 and abs(h2[0]) < 1e-15
    # element-wise: any split of batch or hidden units reproduces the whole, bit for bit
    op = dict(kind="lstm_cell", batch=5, hidden=9)
    for dim, k in [("B", 2), ("B", 5), ("H", 3)]:
        out = np.zeros((5, 9))
        for s_ in range(k):
            reg = R.op_regions(op, [(dim, k, s_)])
            assert reg["in_boxes"][0][:2] == reg["out_box"] and reg["in_boxes"][1] == reg["out_box"] and not reg["is_partial"]
            sl = R.box_slices(reg["out_box"])
            out[sl] = oracle.lstm_cell(g[sl], c[sl])[0]
        assert np.array_equal(out, cn)


# ----------------------------------------------------------------------------- conv1d (Fig. 1 / Fig. 3)
def test_conv1d_against_its_loop_nest_the_2d_convolution_and_closed_forms():
    B, CI, CO, X, DX = 2, 3, 4, 7, 3
    data = synth.uniform(120, 0, (B, CI, X + DX - 1), -1, 1)
    filt = synth.uniform(120, 1, (CI, CO, DX), -1, 1)
    val, absum = oracle.conv1d_box(data, filt)
    # the loop nest of Fig. 1, written out
    want = np.zeros((B, CO, X)); wabs = np.zeros((B, CO, X))
    for b in range(B):
        for co in range(CO):
            for x in range(X):
                for ci in range(CI):
                    for dx in range(DX):
                        p = float(data[b, ci, x + dx]) * float(filt[ci, co, dx])
                        want[b, co, x] += p
                        wabs[b, co, x] += abs(p)
    assert np.allclose(val, want, rtol=0, atol=1e-15) and np.allclose(absum, wabs, rtol=0, atol=1e-15)
    # a 2-D convolution with one row, no padding and the filters' first two indices exchanged
    v2, _ = oracle.conv2d_box(data[:, :, None, :], np.ascontiguousarray(filt.transpose(1, 0, 2))[:, :, None, :], pad=0)
    assert np.allclose(val, v2[:, :, 0, :], rtol=0, atol=1e-14)
    # torch's conv1d in fp64
    import torch
    ref = torch.nn.functional.conv1d(torch.from_numpy(data).double(), torch.from_numpy(filt).double().permute(1, 0, 2)).numpy()
    assert np.allclose(val, ref, rtol=0, atol=1e-14)
    # closed forms: all ones -> CI * DX; a one-tap filter shifts the data
    ones = oracle.conv1d_box(np.ones((B, CI, X + DX - 1), np.float32), np.ones((CI, CO, DX), np.float32))[0]
    assert (ones == CI * DX).all()
    shift = np.zeros((CI, CI, DX), np.float32)
    for c in range(CI):
        shift[c, c, 2] = 1.0
    assert np.array_equal(oracle.conv1d_box(data, shift)[0], data[:, :, 2:2 + X].astype(np.float64))
    # the ci range restricts the sum: two halves add up
    a = oracle.conv1d_box(data, filt, cirange=(0, 1))[0] + oracle.conv1d_box(data, filt, cirange=(1, CI))[0]
    assert np.allclose(a, val, rtol=0, atol=1e-15)


def test_conv1d_regions_follow_the_papers_strategies_and_touched_coordinates():
    """The dedicated conv1d regions reproduce the table of strategies (Fig. 2 / Sec. 4.2) and the bounding
    boxes of what the loop nest touches, for every one-step plan."""
    X, DX = 12, 3
    op = dict(kind="conv1d", batch=4, c_in=6, c_out=8, W=X + DX - 1, KW=DX)
    name = {"b": "B", "ci": "CI", "co": "CO", "x": "X"}
    for split, d_b, d_ci, d_x, f_ci, f_co, f_dx, combine in _rows("conv1d_strategies.txt"):
        regs = [R.op_regions(op, [(name[split], 2, s)]) for s in range(2)]
        assert all(r["is_partial"] == (combine == "sum") for r in regs)
        full = [(0, 4), (0, 6), (0, X + DX - 1)]
        for dimidx, which in enumerate((d_b, d_ci, d_x)):
            parts = [r["in_boxes"][0][dimidx] for r in regs]
            lo, hi = full[dimidx]
            want = {"all": [(lo, hi)] * 2, "half": [(lo, hi // 2), (hi // 2, hi)], "halo": [(0, X // 2 + DX - 1), (X // 2, X + DX - 1)]}[which]
            assert parts == want, (split, dimidx)
        fullf = [(0, 6), (0, 8), (0, DX)]
        for dimidx, which in enumerate((f_ci, f_co, f_dx)):
            parts = [r["in_boxes"][1][dimidx] for r in regs]
            lo, hi = fullf[dimidx]
            assert parts == ([(lo, hi)] * 2 if which == "all" else [(lo, hi // 2), (hi // 2, hi)]), (split, dimidx)
    from oracle import tdl as O
    desc = O.conv1d(4, 6, 8, X, DX)
    var = {"B": "b", "CO": "co", "X": "x", "CI": "ci"}
    for dim in var:
        for k in (2, 3, 4):
            for s in range(k):
                reg = R.op_regions(op, [(dim, k, s)])
                masks = O.touched(desc, [(var[dim], k, s)])
                assert [tuple(b) for b in reg["in_boxes"][0]] == O.bbox(masks[0])
                assert [tuple(b) for b in reg["in_boxes"][1]] == O.bbox(masks[1])


@pytest.mark.parametrize("k", [2, 3, 4])
def test_conv1d_pnr_invariant_on_the_oracle(k):
    data = synth.small_int(121, 0, (4, 8, 14), -3, 3)
    filt = synth.small_int(121, 1, (8, 8, 3), -3, 3)
    op = dict(kind="conv1d", batch=4, c_in=8, c_out=8, W=14, KW=3)
    full = oracle.conv1d_box(data, filt)[0]
    for dim in ["B", "CO", "X", "CI"]:
        got = _assemble(op, dim, k, lambda reg: oracle.conv1d_box(data, filt, box=reg["out_box"], cirange=reg["ranges"]["CI"])[0])
        assert np.array_equal(got, full), dim


# ----------------------------------------------------------------------------- workers of a recursive plan
def test_worker_numbering_of_a_recursive_plan():
    """Appendix A.1 / Sec. 5.2: pins of oracle.regions.worker_splits.  (1) Three 2-way steps on one
    dimension give worker w the w-th eighth (the composition rule of readings 3), which fixes the
    digit order; (2) the 2 x 2 grid of Sec. 5.2's figure numbers its quadrants row by row;
    (3) for mixed step sizes over different dimensions the workers' shards tile the iteration
    space exactly (every coordinate marked once)."""
    op = dict(kind="matmul", M=16, N=12, K=24)
    for w in range(8):
        rng = R.apply_splits(op, R.worker_splits(["K", "K", "K"], [2, 2, 2], w))
        assert rng["K"] == R.shard_range(24, 8, w)
    quad = [R.apply_splits(op, R.worker_splits(["M", "N"], [2, 2], w)) for w in range(4)]
    assert [(q["M"], q["N"]) for q in quad] == [((0, 8), (0, 6)), ((0, 8), (6, 12)), ((8, 16), (0, 6)), ((8, 16), (6, 12))]
    for dims, ks in [(["M", "K", "N"], [2, 3, 2]), (["N", "N", "M"], [3, 2, 4]), (["K"], [5])]:
        seen = np.zeros((16, 12, 24), dtype=np.int32)
        total = int(np.prod(ks))
        for w in range(total):
            r = R.apply_splits(op, R.worker_splits(dims, ks, w))
            seen[r["M"][0]:r["M"][1], r["N"][0]:r["N"][1], r["K"][0]:r["K"][1]] += 1
        assert (seen == 1).all()
    with pytest.raises(ValueError):
        R.worker_splits(["M"], [2], 2)
