"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element,
on seeded inputs.  Sizes here are small enough for the oracle to evaluate every element while
still spanning several tiles and ragged tails; the full-size workloads are in
test_gpu_workloads.py.

Bars: indices, regions and copies are bit-exact; fp32 results satisfy
|gpu - oracle| <= 1e-5 * S per element, S = sum |a*b| (for the reduce: sum_j |p_j|); with
small-integer inputs every sum is exact in fp32 and fp64, so equality is bit-exact.
"""
import itertools

import numpy as np
import pytest
import torch

import oracle
import paper_1807_08887_amd as tofu
import tofu_synth as synth
from oracle import regions as R

pytestmark = pytest.mark.gpu
TOL = 1e-5
DEV = "cuda:0"

MM_DIMS = {"M": tofu.MM_DIM_M, "N": tofu.MM_DIM_N, "K": tofu.MM_DIM_K}
CONV_DIMS = {"N": tofu.CONV_DIM_N, "CO": tofu.CONV_DIM_CO, "H": tofu.CONV_DIM_H, "W": tofu.CONV_DIM_W, "CI": tofu.CONV_DIM_CI}
WGRAD_DIMS = {"CO": tofu.WGRAD_DIM_CO, "CI": tofu.WGRAD_DIM_CI, "N": tofu.WGRAD_DIM_N}
DGRAD_DIMS = {"N": tofu.DGRAD_DIM_N, "CI": tofu.DGRAD_DIM_CI, "H": tofu.DGRAD_DIM_H, "W": tofu.DGRAD_DIM_W, "CO": tofu.DGRAD_DIM_CO}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def assert_close(got, val, absum, what=""):
    got = got.astype(np.float64)
    err = np.abs(got - val)
    bound = TOL * absum
    bad = err > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements off, worst ratio {np.max(err / np.maximum(absum, 1e-300)):.3e}"
    assert (got[absum == 0] == 0).all()


def workspace(op, splits):
    n = tofu.workspace_bytes(op, splits)
    return torch.empty(max(n, 16) // 4, dtype=torch.float32, device=DEV) if n else None


# ----------------------------------------------------------------------------- reduce
@pytest.mark.parametrize("k", [1, 2, 3, 8, 16])
@pytest.mark.parametrize("count", [1, 3, 1000, 4097, (1 << 20) + 5])
def test_partition_reduce(k, count):
    parts = [synth.normal(11, j, (count,), 2.0) for j in range(k)]
    d = [dev(p) for p in parts]
    out = torch.empty(count, dtype=torch.float32, device=DEV)
    tofu.partition_reduce(out, d)
    val, absum = oracle.reduce(parts)
    assert_close(out.cpu().numpy(), val, absum, f"reduce k={k} count={count}")
    # fixed left-to-right fp32 order: identical to the same order on the host, bit for bit
    ref = parts[0].copy()
    for p in parts[1:]:
        ref = ref + p
    assert np.array_equal(out.cpu().numpy(), ref)
    # in place: dst == partials[0]
    tofu.partition_reduce(d[0], d)
    assert np.array_equal(d[0].cpu().numpy(), ref)


def test_partition_reduce_edge_cases():
    out = torch.zeros(8, dtype=torch.float32, device=DEV)
    tofu.partition_reduce(out, [out], count=0)                      # empty: no-op
    ints = [synth.small_int(12, j, (1001,), -1000, 1000) for j in range(8)]
    buf = [torch.empty(1004, dtype=torch.float32, device=DEV) for _ in range(8)]
    for b, a in zip(buf, ints):
        b[1:1002] = dev(a)                                          # 4-byte aligned only
    dst = torch.empty(1004, dtype=torch.float32, device=DEV)
    tofu.partition_reduce(dst[1:1002].data_ptr(), [b[1:1002].data_ptr() for b in buf], count=1001)
    assert np.array_equal(dst[1:1002].cpu().numpy().astype(np.float64), oracle.reduce(ints)[0])
    with pytest.raises(tofu.TofuError) as e:
        tofu.partition_reduce(buf[1], buf)                          # dst aliases partials[1]
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError):
        tofu.partition_reduce(dst, buf * 3)                         # k = 24 > 16


# ----------------------------------------------------------------------------- fetch
def _fetch_case(shape, box, cuts_dim, k, dtype_int=True, strided=False):
    t = synth.small_int(21, 0, shape, -99, 99)
    blocks, descs, keep = [], [], []
    for s in range(k):
        lo, hi = R.shard_range(shape[cuts_dim], k, s)
        bbox = [(0, e) for e in shape]
        bbox[cuts_dim] = (lo, hi)
        blk = t[R.box_slices(bbox)]
        blocks.append((blk, bbox))
        if strided:   # block lives inside a larger allocation: non-dense strides
            big = torch.full([e + 3 for e in blk.shape], -7.0, dtype=torch.float32, device=DEV)
            view = big[tuple(slice(1, 1 + e) for e in blk.shape)]
            view.copy_(dev(blk))
        else:
            view = dev(blk)
        keep.append(view)
        descs.append(tofu.tensor(view, [b[0] for b in bbox]))
    want = R.fetch(box, blocks)
    out = torch.full([hi - lo for lo, hi in box], -5.0, dtype=torch.float32, device=DEV)
    tofu.region_fetch(tofu.tensor(out, [lo for lo, _ in box]), descs)
    assert np.array_equal(out.cpu().numpy(), want)


@pytest.mark.parametrize("strided", [False, True])
def test_region_fetch_shapes(strided):
    _fetch_case((40,), [(3, 37)], 0, 3, strided=strided)
    _fetch_case((9, 16), [(2, 9), (4, 12)], 0, 2, strided=strided)                 # 16-byte vectors possible
    _fetch_case((5, 6, 14), [(0, 5), (1, 6), (0, 14)], 1, 3, strided=strided)      # 8-byte vectors
    _fetch_case((4, 6, 9, 7), [(1, 4), (0, 6), (2, 8), (0, 7)], 2, 3, strided=strided)   # scalar runs
    _fetch_case((3, 2, 4, 5, 3, 2), [(0, 3), (0, 2), (1, 4), (0, 5), (1, 3), (0, 2)], 3, 5, strided=strided)


def test_region_fetch_halo_of_h_split():
    """The conv workload's fetch in small: own rows + one halo row of the neighbour (Sec. 4.2)."""
    op = dict(kind="conv2d", batch=6, c_in=20, c_out=4, H=14, W=14, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(22, 0, (6, 20, 14, 14), 1.0)
    own = [(x[:, :, lo:hi].copy(), [(0, 6), (0, 20), (lo, hi), (0, 14)]) for lo, hi in (R.shard_range(14, 2, s) for s in range(2))]
    for s in range(2):
        box = R.op_regions(op, [("H", 2, s)])["in_boxes"][0]
        assert box[2] == ((0, 8) if s == 0 else (6, 14))
        srcs = [dev(b) for b, _ in own]
        out = torch.empty([hi - lo for lo, hi in box], dtype=torch.float32, device=DEV)
        tofu.region_fetch(tofu.tensor(out, [lo for lo, _ in box]), [tofu.tensor(t, [b[0] for b in bb]) for t, (_, bb) in zip(srcs, own)])
        assert np.array_equal(out.cpu().numpy(), R.fetch(box, own))


def test_region_fetch_empty_destination():
    src = torch.zeros(4, 4, dtype=torch.float32, device=DEV)
    out = torch.zeros(0, 4, dtype=torch.float32, device=DEV)
    tofu.region_fetch(tofu.tensor(out, [2, 0]), [tofu.tensor(src)])


# ----------------------------------------------------------------------------- shard runners
def run_matmul(A, B, splits, names=MM_DIMS, a_full=None, b_full=None):
    """Run one matmul shard on full-size device tensors; returns (C device tensor, regions)."""
    M, K = A.shape
    N = B.shape[1]
    op = tofu.matmul_desc(M, N, K)
    sp = [(names[d], k, s) for d, k, s in splits]
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_matmul(op, sp, tofu.tensor(a_full), tofu.tensor(b_full), tofu.tensor(C), workspace(op, sp))
    return C


def assemble(op_dict, dim, k, run):
    full_box = R.op_regions(op_dict, [])["out_box"]
    shape = [hi - lo for lo, hi in full_box]
    total = np.zeros(shape, dtype=np.float32)
    partials = []
    for s in range(k):
        reg = R.op_regions(op_dict, [(dim, k, s)])
        out = run([(dim, k, s)]).cpu().numpy()
        sl = R.box_slices(reg["out_box"])
        inside = np.zeros(shape, dtype=bool)
        inside[sl] = True
        assert not np.isnan(out[inside]).any() and np.isnan(out[~inside]).all(), "shard must write exactly its output box"
        if reg["is_partial"]:
            partials.append(out)
        else:
            total[sl] = out[sl]
    if partials:
        d = [dev(p) for p in partials]
        res = torch.empty_like(d[0])
        tofu.partition_reduce(res, d)
        total = res.cpu().numpy()
    return total


# ----------------------------------------------------------------------------- matmul
def test_tiny_matmul_workload():
    """Workload 1: C[64,96] = A[64,128] B[128,96]; 2-way K split (partials summed) and 2-way N
    split (concatenated) both reproduce the unpartitioned oracle."""
    cfg = synth.CONFIGS["tiny_matmul"]
    A = synth.draw(cfg["a"], cfg["seed"], 0, (cfg["M"], cfg["K"]))
    B = synth.draw(cfg["b"], cfg["seed"], 1, (cfg["K"], cfg["N"]))
    dA, dB = dev(A), dev(B)
    val, absum = oracle.matmul_box(A, B)
    op = dict(kind="matmul", M=cfg["M"], N=cfg["N"], K=cfg["K"])
    for dim in ["K", "N", "M"]:
        got = assemble(op, dim, 2, lambda sp: run_matmul(A, B, sp, a_full=dA, b_full=dB))
        assert_close(got, val, absum, f"tiny matmul split {dim}")
    # a single worker's K partial against the oracle restricted to its K range
    part = run_matmul(A, B, [("K", 2, 1)], a_full=dA, b_full=dB).cpu().numpy()
    pv, ps = oracle.matmul_box(A, B, krange=(64, 128))
    assert_close(part, pv, ps, "tiny matmul K partial")


@pytest.mark.parametrize("M,N,K", [(70, 130, 77), (128, 256, 4096), (1, 1, 1), (33, 65, 1030), (257, 64, 16)])
def test_matmul_shapes_unpartitioned(M, N, K):
    A = synth.uniform(31, 0, (M, K), -1, 1)
    B = synth.uniform(31, 1, (K, N), -1, 1)
    got = run_matmul(A, B, [], a_full=dev(A), b_full=dev(B)).cpu().numpy()
    val, absum = oracle.matmul_box(A, B)
    assert_close(got, val, absum, f"matmul {M}x{N}x{K}")


@pytest.mark.parametrize("k", [2, 3, 4, 8])
def test_matmul_pnr_invariant_bit_exact(k):
    A = synth.small_int(32, 0, (72, 200), -4, 4)
    B = synth.small_int(32, 1, (200, 136), -4, 4)
    dA, dB = dev(A), dev(B)
    want = oracle.matmul_box(A, B)[0]
    op = dict(kind="matmul", M=72, N=136, K=200)
    for dim in ["M", "N", "K"]:
        got = assemble(op, dim, k, lambda sp: run_matmul(A, B, sp, a_full=dA, b_full=dB))
        assert np.array_equal(got.astype(np.float64), want), dim


def test_matmul_recursive_plan_and_blocks():
    """A two-step plan <N/2, K/2> on owned blocks: A and B are passed as the blocks a worker
    holds (extent != whole tensor), C as the worker's own output block."""
    A = synth.small_int(33, 0, (64, 96), -4, 4)
    B = synth.small_int(33, 1, (96, 80), -4, 4)
    op_d = dict(kind="matmul", M=64, N=80, K=96)
    op = tofu.matmul_desc(64, 80, 96)
    want = oracle.matmul_box(A, B)[0]
    total = np.zeros((64, 80))
    for a, b in itertools.product(range(2), repeat=2):
        plan = [("N", 2, a), ("K", 2, b)]
        reg = R.op_regions(op_d, plan)
        (m0, m1), (k0, k1) = reg["in_boxes"][0]
        (_, _), (n0, n1) = reg["in_boxes"][1]
        blkA, blkB = dev(A[m0:m1, k0:k1]), dev(B[k0:k1, n0:n1])
        C = torch.zeros(64, n1 - n0, dtype=torch.float32, device=DEV)
        sp = [(MM_DIMS[d], k, s) for d, k, s in plan]
        tofu.shard_matmul(op, sp, tofu.tensor(blkA, [m0, k0]), tofu.tensor(blkB, [k0, n0]), tofu.tensor(C, [0, n0]), workspace(op, sp))
        total[:, n0:n1] += C.cpu().numpy()
    assert np.array_equal(total, want)


def test_matmul_strided_views():
    A = synth.uniform(34, 0, (64, 300), -1, 1)
    B = synth.uniform(34, 1, (300, 200), -1, 1)
    val, absum = oracle.matmul_box(A, B)
    At = dev(A.T.copy()).t()            # column-major view: unit stride along m
    Bt = dev(B.T.copy()).t()
    op = tofu.matmul_desc(64, 200, 300)
    C = torch.empty(64, 200, dtype=torch.float32, device=DEV)
    tofu.shard_matmul(op, [], tofu.tensor(At), tofu.tensor(Bt), tofu.tensor(C))
    assert_close(C.cpu().numpy(), val, absum, "column-major operands")
    # output written into a column block of a wider row-major buffer
    wide = torch.zeros(64, 512, dtype=torch.float32, device=DEV)
    dA, dB = dev(A), dev(B)              # keep the device buffers alive: descriptors only hold addresses
    tofu.shard_matmul(op, [], tofu.tensor(dA), tofu.tensor(dB), tofu.tensor(wide[:, 100:300]))
    assert_close(wide[:, 100:300].cpu().numpy(), val, absum, "strided output")
    assert (wide[:, :100] == 0).all() and (wide[:, 300:] == 0).all()


@pytest.mark.parametrize("Bt,K,N", [(40, 136, 200), (128, 96, 260), (33, 70, 50)])
def test_matmul_backward_gemms_through_transposed_views(Bt, K, N):
    """The backward GEMMs of Y = X W are the same entry point on transposed views:
    dX = dY W^T (B operand contiguous along k) and dW = X^T dY (A operand contiguous along m),
    each under every split dimension; small integers, so sums are exact and equality is bit-exact.
    Strides that are whole vectors take the vector staging, (33, 70, 50) the guarded one."""
    X = synth.small_int(35, 0, (Bt, K), -3, 3)
    W = synth.small_int(35, 1, (K, N), -3, 3)
    dY = synth.small_int(35, 2, (Bt, N), -3, 3)
    dX_, dW_, ddY = dev(X), dev(W), dev(dY)
    # dX[Bt,K] = dY[Bt,N] . W^T[N,K]
    want = oracle.matmul_box(dY, np.ascontiguousarray(W.T))[0]
    op_d = dict(kind="matmul", M=Bt, N=K, K=N)
    op = tofu.matmul_desc(Bt, K, N)

    def run_dx(sp):
        C = torch.full((Bt, K), float("nan"), dtype=torch.float32, device=DEV)
        spl = [(MM_DIMS[d], k, s) for d, k, s in sp]
        tofu.shard_matmul(op, spl, tofu.tensor(ddY), tofu.tensor(dW_.t()), tofu.tensor(C), workspace(op, spl))
        return C
    for dim, k in itertools.product(["M", "N", "K"], [2, 3]):
        got = assemble(op_d, dim, k, run_dx)
        assert np.array_equal(got.astype(np.float64), want), ("dX", dim, k)
    # dW[K,N] = X^T[K,Bt] . dY[Bt,N]
    want = oracle.matmul_box(np.ascontiguousarray(X.T), dY)[0]
    op_d = dict(kind="matmul", M=K, N=N, K=Bt)
    op2 = tofu.matmul_desc(K, N, Bt)

    def run_dw(sp):
        C = torch.full((K, N), float("nan"), dtype=torch.float32, device=DEV)
        spl = [(MM_DIMS[d], k, s) for d, k, s in sp]
        tofu.shard_matmul(op2, spl, tofu.tensor(dX_.t()), tofu.tensor(ddY), tofu.tensor(C), workspace(op2, spl))
        return C
    for dim, k in itertools.product(["M", "N", "K"], [2, 3]):
        got = assemble(op_d, dim, k, run_dw)
        assert np.array_equal(got.astype(np.float64), want), ("dW", dim, k)


def test_matmul_transposed_views_long_k():
    """Both operands transposed, K long enough for the kernel's own K slices, fp32 data."""
    A = synth.uniform(36, 0, (128, 2080), -1, 1)
    B = synth.uniform(36, 1, (2080, 192), -1, 1)
    val, absum = oracle.matmul_box(A, B)
    dAt, dBt = dev(A.T.copy()), dev(B.T.copy())
    op = tofu.matmul_desc(128, 192, 2080)
    for a_view, b_view, what in [(dAt.t(), dBt.t(), "TT"), (dAt.t(), dev(B), "TN"), (dev(A), dBt.t(), "NT")]:
        C = torch.empty(128, 192, dtype=torch.float32, device=DEV)
        tofu.shard_matmul(op, [], tofu.tensor(a_view), tofu.tensor(b_view), tofu.tensor(C), workspace(op, []))
        assert_close(C.cpu().numpy(), val, absum, what)


# ----------------------------------------------------------------------------- conv2d
def run_conv(opd, splits, dx, dw, x_lo=None):
    op = tofu.conv2d_desc(opd["batch"], opd["c_in"], opd["c_out"], opd["H"], opd["W"], pad=opd["pad"])
    sp = [(CONV_DIMS[d], k, s) for d, k, s in splits]
    ho, wo = opd["H"] + 2 * opd["pad"] - 2, opd["W"] + 2 * opd["pad"] - 2
    y = torch.full((opd["batch"], opd["c_out"], ho, wo), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_conv2d(op, sp, tofu.tensor(dx, x_lo), tofu.tensor(dw), tofu.tensor(y), workspace(op, sp))
    return y


@pytest.mark.parametrize("batch,c_in,c_out,H,W,pad", [(3, 10, 70, 14, 14, 1), (2, 5, 33, 9, 11, 1), (2, 16, 64, 8, 8, 0),
                                                      (1, 3, 5, 1, 1, 1), (2, 9, 40, 30, 28, 1)])
def test_conv2d_shapes_unpartitioned(batch, c_in, c_out, H, W, pad):
    opd = dict(kind="conv2d", batch=batch, c_in=c_in, c_out=c_out, H=H, W=W, KH=3, KW=3, stride=1, pad=pad)
    x = synth.normal(41, 0, (batch, c_in, H, W), 1.0)
    w = synth.normal(41, 1, (c_out, c_in, 3, 3), 0.3)
    got = run_conv(opd, [], dev(x), dev(w)).cpu().numpy()
    val, absum = oracle.conv2d_box(x, w, pad=pad)
    assert_close(got, val, absum, f"conv2d {opd}")


def test_conv2d_wide_rows_and_limits():
    """56-wide rows need the narrower channel step; rows too wide for the staging buffers are
    reported as unsupported instead of being computed some slower way."""
    opd = dict(kind="conv2d", batch=1, c_in=6, c_out=64, H=20, W=56, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(44, 0, (1, 6, 20, 56), 1.0)
    w = synth.normal(44, 1, (64, 6, 3, 3), 0.3)
    got = run_conv(opd, [], dev(x), dev(w)).cpu().numpy()
    val, absum = oracle.conv2d_box(x, w, pad=1)
    assert_close(got, val, absum, "conv2d 20x56")
    wide = dict(opd, W=400)
    with pytest.raises(tofu.TofuError) as e:
        run_conv(wide, [], torch.zeros(1, 6, 20, 400, device=DEV), dev(w))
    assert e.value.status == -6


@pytest.mark.parametrize("k", [2, 3, 4])
def test_conv2d_pnr_invariant_bit_exact(k):
    opd = dict(kind="conv2d", batch=4, c_in=12, c_out=72, H=12, W=10, KH=3, KW=3, stride=1, pad=1)
    x = synth.small_int(42, 0, (4, 12, 12, 10), -3, 3)
    w = synth.small_int(42, 1, (72, 12, 3, 3), -3, 3)
    dx, dw = dev(x), dev(w)
    want = oracle.conv2d_box(x, w, pad=1)[0]
    for dim in ["N", "CO", "H", "W", "CI"]:
        got = assemble(opd, dim, k, lambda sp: run_conv(opd, sp, dx, dw))
        assert np.array_equal(got.astype(np.float64), want), dim


def test_conv2d_on_fetched_halo_region():
    """Plan <CO/2, H/2>: the worker fetches its halo-widened input rows from the two owners'
    blocks, then convolves the fetched buffer (whose extent is the region, not the tensor)."""
    opd = dict(kind="conv2d", batch=5, c_in=16, c_out=64, H=14, W=14, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(43, 0, (5, 16, 14, 14), 1.0)
    w = synth.normal(43, 1, (64, 16, 3, 3), 0.2)
    val, absum = oracle.conv2d_box(x, w, pad=1)
    own = [(x[:, :, lo:hi].copy(), [(0, 5), (0, 16), (lo, hi), (0, 14)]) for lo, hi in (R.shard_range(14, 2, s) for s in range(2))]
    d_own = [dev(b) for b, _ in own]
    dw = dev(w)
    op = tofu.conv2d_desc(5, 16, 64, 14, 14)
    for a, b in itertools.product(range(2), repeat=2):
        plan = [("CO", 2, a), ("H", 2, b)]
        reg = R.op_regions(opd, plan)
        lib = tofu.op_regions(op, [(CONV_DIMS[d], k, s) for d, k, s in plan])
        assert lib["in_boxes"][0] == [tuple(t) for t in reg["in_boxes"][0]] and lib["pad_lo"] == reg["pad_lo"] and lib["pad_hi"] == reg["pad_hi"]
        box = reg["in_boxes"][0]
        region = torch.empty([hi - lo for lo, hi in box], dtype=torch.float32, device=DEV)
        tofu.region_fetch(tofu.tensor(region, [lo for lo, _ in box]), [tofu.tensor(t, [q[0] for q in bb]) for t, (_, bb) in zip(d_own, own)])
        y = run_conv(opd, plan, region, dw, x_lo=[lo for lo, _ in box]).cpu().numpy()
        sl = R.box_slices(reg["out_box"])
        assert_close(y[sl], val[sl], absum[sl], f"conv on fetched region {plan}")
    # a region that misses a needed interior row is an error, never silent zero padding
    short = torch.zeros(5, 16, 7, 14, dtype=torch.float32, device=DEV)
    with pytest.raises(tofu.TofuError) as e:
        run_conv(opd, [("H", 2, 0)], short, dw, x_lo=[0, 0, 0, 0])
    assert e.value.status == -2


def blocks_of(x, cuts, views=False):
    """Cut the global array x into blocks along (N, H, W) at the given cut points; returns
    [(device block, low corner)] in row-major block order (every block spans all channels).
    views: the blocks are strided views of one device copy of x (all with the same strides, close
    together in memory) instead of separately allocated dense copies."""
    out = []
    n_cuts, h_cuts, w_cuts = cuts
    whole = dev(x) if views else None
    for (n0, n1), (h0, h1), (w0, w1) in itertools.product(zip(n_cuts, n_cuts[1:]), zip(h_cuts, h_cuts[1:]), zip(w_cuts, w_cuts[1:])):
        out.append((whole[n0:n1, :, h0:h1, w0:w1] if views else dev(x[n0:n1, :, h0:h1, w0:w1].copy()), [n0, 0, h0, w0]))
    return out


@pytest.mark.parametrize("shape,cuts,views", [
    ((5, 16, 64, 14, 14), ([0, 5], [0, 7, 14], [0, 14]), False),             # the halo case: two row blocks allocated alike
    ((4, 9, 70, 12, 10), ([0, 1, 4], [0, 5, 6, 12], [0, 3, 10]), False),     # blocks cut along N, H and W, one row high, all strides differ
    ((3, 7, 33, 9, 30), ([0, 3], [0, 9], [0, 11, 30]), False),               # ragged channel tail, 128-position tiles
    ((4, 9, 70, 12, 10), ([0, 1, 4], [0, 5, 6, 12], [0, 3, 10]), True),      # the same cuts as views with one channel stride
    ((6, 10, 96, 14, 14), ([0, 2, 6], [0, 7, 14], [0, 14]), True),           # halo blocks of two image groups, one channel stride
])
def test_conv2d_fused_fetch_matches_oracle_and_the_assembled_region(shape, cuts, views):
    """The convolution that reads its region straight from the blocks holding it: against the
    oracle on the global tensor, and bit for bit against fetch-then-convolve, for every shard
    of a <CO/2, H/2> plan and for the unpartitioned operator.  Blocks with differing channel
    strides are read through per-item addresses; blocks that share it (dense blocks of one shape,
    views of one array) through one buffer window."""
    batch, c_in, c_out, H, W = shape
    opd = dict(kind="conv2d", batch=batch, c_in=c_in, c_out=c_out, H=H, W=W, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(47, 0, (batch, c_in, H, W), 1.0)
    w = synth.normal(47, 1, (c_out, c_in, 3, 3), 0.3)
    val, absum = oracle.conv2d_box(x, w, pad=1)
    blocks = blocks_of(x, cuts, views)
    srcs = [tofu.tensor(t, lo) for t, lo in blocks]
    dw = dev(w)
    op = tofu.conv2d_desc(batch, c_in, c_out, H, W)
    plans = [[]] + [[("CO", 2, a), ("H", 2, b)] for a, b in itertools.product(range(2), repeat=2)]
    for plan in plans:
        sp = [(CONV_DIMS[d], k, s) for d, k, s in plan]
        reg = R.op_regions(opd, plan)
        y = torch.full((batch, c_out, H, W), float("nan"), dtype=torch.float32, device=DEV)
        tofu.shard_conv2d_fused(op, sp, srcs, tofu.tensor(dw), tofu.tensor(y), workspace(op, sp))
        sl = R.box_slices(reg["out_box"])
        got = y.cpu().numpy()
        assert_close(got[sl], val[sl], absum[sl], f"fused conv {plan}")
        mask = np.ones(got.shape, bool)
        mask[sl] = False
        assert np.isnan(got[mask]).all(), "wrote outside the shard's output box"
        box = reg["in_boxes"][0]
        region = torch.empty([hi - lo for lo, hi in box], dtype=torch.float32, device=DEV)
        tofu.region_fetch(tofu.tensor(region, [lo for lo, _ in box]), srcs)
        y2 = run_conv(opd, plan, region, dw, x_lo=[lo for lo, _ in box])
        assert torch.equal(y[sl], y2[sl]), f"fused and fetched results differ for {plan}"


def test_conv2d_fused_fetch_error_paths():
    opd = dict(kind="conv2d", batch=2, c_in=8, c_out=64, H=8, W=8, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(48, 0, (2, 8, 8, 8), 1.0)
    dw = dev(synth.normal(48, 1, (64, 8, 3, 3), 0.3))
    op = tofu.conv2d_desc(2, 8, 64, 8, 8)
    y = torch.zeros(2, 64, 8, 8, dtype=torch.float32, device=DEV)
    top, bottom = dev(x[:, :, 0:4].copy()), dev(x[:, :, 4:8].copy())
    call = lambda srcs, sp=(): tofu.shard_conv2d_fused(op, list(sp), srcs, tofu.tensor(dw), tofu.tensor(y), workspace(op, list(sp)))
    with pytest.raises(tofu.TofuError) as e:           # a missing row block is a hole, never zeros
        call([tofu.tensor(top, [0, 0, 0, 0])])
    assert e.value.status == -3
    with pytest.raises(tofu.TofuError) as e:           # the same rows held twice
        call([tofu.tensor(top, [0, 0, 0, 0]), tofu.tensor(bottom, [0, 0, 4, 0]), tofu.tensor(top, [0, 0, 0, 0])])
    assert e.value.status == -4
    lo_c, hi_c = dev(x[:, 0:4].copy()), dev(x[:, 4:8].copy())
    with pytest.raises(tofu.TofuError) as e:           # blocks cut along the channels need the fetch
        call([tofu.tensor(lo_c, [0, 0, 0, 0]), tofu.tensor(hi_c, [0, 4, 0, 0])])
    assert e.value.status == -6
    with pytest.raises(tofu.TofuError) as e:
        call([])
    assert e.value.status == -1
    # a shard that needs only the top rows is served by the top block alone
    call([tofu.tensor(top, [0, 0, 0, 0])], sp=[(CONV_DIMS["H"], 4, 0)])
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------- wgrad
def run_wgrad(opd, splits, dx, ddy):
    op = tofu.wgrad_desc(opd["batch"], opd["c_in"], opd["c_out"], opd["H"], opd["W"], pad=opd["pad"])
    sp = [(WGRAD_DIMS[d], k, s) for d, k, s in splits]
    dw = torch.full((opd["c_out"], opd["c_in"], 3, 3), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_conv2d_wgrad(op, sp, tofu.tensor(dx), tofu.tensor(ddy), tofu.tensor(dw), workspace(op, sp))
    return dw


@pytest.mark.parametrize("batch,c_in,c_out,H,W,pad", [(3, 40, 130, 28, 28, 1), (2, 5, 33, 9, 11, 1), (4, 32, 64, 8, 8, 0),
                                                      (1, 3, 5, 1, 1, 1), (2, 9, 20, 6, 70, 1),
                                                      # widths 16 / 32 / 28 take the unrolled steps, 24 the looped fast one;
                                                      # H = 1 gives workgroups a single step
                                                      (2, 32, 128, 16, 16, 1), (3, 33, 40, 6, 32, 1), (2, 20, 30, 5, 24, 1),
                                                      (1, 8, 8, 1, 16, 1), (5, 64, 256, 2, 28, 1),
                                                      # 14 wide: two rows per step (even heights); 7 wide: four rows per step,
                                                      # heights that leave a short last group; odd height 14 wide takes the guarded path
                                                      (3, 40, 130, 14, 14, 1), (2, 33, 64, 6, 14, 1), (4, 64, 140, 7, 7, 1),
                                                      (2, 20, 30, 5, 7, 1), (3, 32, 128, 1, 7, 1), (2, 16, 32, 9, 14, 1),
                                                      (2, 24, 40, 9, 9, 0), (3, 16, 32, 16, 16, 0),
                                                      # rows wider than 32 columns are cut into chunks: 56 = 2 x 28, 40 = 2 x 20,
                                                      # 36 = 20 + 16 (a short last chunk), 100 = 4 x 28 with a short last chunk
                                                      (2, 16, 40, 5, 56, 1), (1, 8, 32, 3, 40, 1), (2, 9, 20, 4, 36, 1), (1, 5, 16, 2, 100, 1),
                                                      (2, 8, 16, 6, 58, 0)])
def test_wgrad_shapes_unpartitioned(batch, c_in, c_out, H, W, pad):
    opd = dict(kind="conv2d_wgrad", batch=batch, c_in=c_in, c_out=c_out, H=H, W=W, KH=3, KW=3, stride=1, pad=pad)
    ho, wo = H + 2 * pad - 2, W + 2 * pad - 2
    x = synth.normal(51, 0, (batch, c_in, H, W), 1.0)
    dy = synth.normal(51, 1, (batch, c_out, ho, wo), 1.0)
    got = run_wgrad(opd, [], dev(x), dev(dy)).cpu().numpy()
    val, absum = oracle.wgrad_box(x, dy, 3, 3, pad=pad)
    assert_close(got, val, absum, f"wgrad {opd}")


@pytest.mark.parametrize("H,W", [(14, 14), (7, 7)])
def test_wgrad_narrow_images_pnr_invariant_bit_exact(H, W):
    """Several output rows per step: every split dimension, small integers, bit-exact."""
    opd = dict(kind="conv2d_wgrad", batch=6, c_in=40, c_out=136, H=H, W=W, KH=3, KW=3, stride=1, pad=1)
    x = synth.small_int(54, 0, (6, 40, H, W), -3, 3)
    dy = synth.small_int(54, 1, (6, 136, H, W), -3, 3)
    dx, ddy = dev(x), dev(dy)
    want = oracle.wgrad_box(x, dy, 3, 3, pad=1)[0]
    for dim, k in itertools.product(["CO", "CI", "N"], [2, 3]):
        got = assemble(opd, dim, k, lambda sp: run_wgrad(opd, sp, dx, ddy))
        assert np.array_equal(got.astype(np.float64), want), (dim, k)


@pytest.mark.parametrize("k", [2, 3, 4])
def test_wgrad_pnr_invariant_bit_exact(k):
    opd = dict(kind="conv2d_wgrad", batch=8, c_in=36, c_out=130, H=12, W=10, KH=3, KW=3, stride=1, pad=1)
    x = synth.small_int(52, 0, (8, 36, 12, 10), -3, 3)
    dy = synth.small_int(52, 1, (8, 130, 12, 10), -3, 3)
    dx, ddy = dev(x), dev(dy)
    want = oracle.wgrad_box(x, dy, 3, 3, pad=1)[0]
    for dim in ["CO", "CI", "N"]:
        got = assemble(opd, dim, k, lambda sp: run_wgrad(opd, sp, dx, ddy))
        assert np.array_equal(got.astype(np.float64), want), dim


def test_wgrad_many_tiles_few_images():
    """960 output tiles x 2 images: the first 512 tiles run one workgroup each and write dw directly,
    the other 448 are balanced over the workgroup slots and summed from workspace slots."""
    co, ci, nb = 640, 6144, 2
    opd = dict(kind="conv2d_wgrad", batch=nb, c_in=ci, c_out=co, H=4, W=4, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(53, 0, (nb, ci, 4, 4), 1.0)
    dy = synth.normal(53, 1, (nb, co, 4, 4), 1.0)
    got = run_wgrad(opd, [], dev(x), dev(dy)).cpu().numpy()
    pts = np.concatenate([synth.coords(53, 2, 20000, got.shape),
                          np.array([[0, 0, 0, 0], [co - 1, ci - 1, 2, 2], [127, 31, 1, 1], [128, 32, 0, 2]])])
    val, absum = oracle.wgrad_pts(x, dy, 3, 3, pts, pad=1)
    assert not np.isnan(got).any()
    assert_close(got[tuple(pts.T)], val, absum, "wgrad 960 tiles x 2 images")


def test_wgrad_whole_waves_then_a_balanced_rest_on_the_two_row_form():
    """640 tiles of a 14 x 14 layer (two output rows per step): one whole wave of 512 tiles, then 128 tiles
    with four workgroups each; sampled outputs of both parts, the seam between them and the corners."""
    co, ci, nb = 1280, 2048, 4
    opd = dict(kind="conv2d_wgrad", batch=nb, c_in=ci, c_out=co, H=14, W=14, KH=3, KW=3, stride=1, pad=1)
    x = synth.normal(54, 0, (nb, ci, 14, 14), 1.0)
    dy = synth.normal(54, 1, (nb, co, 14, 14), 1.0)
    got = run_wgrad(opd, [], dev(x), dev(dy)).cpu().numpy()
    pts = np.concatenate([synth.coords(54, 2, 6000, got.shape),
                          np.array([[0, 0, 0, 0], [co - 1, ci - 1, 2, 2], [1023, 2047, 1, 1], [1024, 0, 0, 2], [1279, 31, 2, 0], [896, 2016, 1, 2]])])   # incl. the last whole and the first balanced tile
    val, absum = oracle.wgrad_pts(x, dy, 3, 3, pts, pad=1)
    assert not np.isnan(got).any()
    assert_close(got[tuple(pts.T)], val, absum, "wgrad 640 tiles, two-row steps")


def test_runs_are_bit_identical():
    """No atomics anywhere: two runs of the same call give the same bits."""
    A = synth.normal(61, 0, (128, 4096), 1.0); B = synth.normal(61, 1, (4096, 256), 1.0)
    dA, dB = dev(A), dev(B)
    c1 = run_matmul(A, B, [], a_full=dA, b_full=dB).cpu().numpy()
    c2 = run_matmul(A, B, [], a_full=dA, b_full=dB).cpu().numpy()
    assert np.array_equal(c1, c2)


# ----------------------------------------------------------------------------- dgrad
def run_dgrad(opd, splits, ddy, dw, dy_lo=None):
    op = tofu.dgrad_desc(opd["batch"], opd["c_in"], opd["c_out"], opd["H"], opd["W"], pad=opd["pad"])
    sp = [(DGRAD_DIMS[d], k, s) for d, k, s in splits]
    dx = torch.full((opd["batch"], opd["c_in"], opd["H"], opd["W"]), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_conv2d_dgrad(op, sp, tofu.tensor(ddy, dy_lo), tofu.tensor(dw), tofu.tensor(dx), workspace(op, sp))
    return dx


@pytest.mark.parametrize("batch,c_in,c_out,H,W", [(3, 70, 10, 14, 14), (2, 33, 5, 9, 11), (1, 5, 3, 1, 1), (2, 40, 9, 30, 28),
                                                  (4, 64, 37, 7, 14)])
def test_dgrad_shapes_unpartitioned(batch, c_in, c_out, H, W):
    opd = dict(kind="conv2d_dgrad", batch=batch, c_in=c_in, c_out=c_out, H=H, W=W, KH=3, KW=3, stride=1, pad=1)
    dy = synth.normal(61, 0, (batch, c_out, H, W), 1.0)
    w = synth.normal(61, 1, (c_out, c_in, 3, 3), 0.3)
    got = run_dgrad(opd, [], dev(dy), dev(w)).cpu().numpy()
    val, absum = oracle.dgrad_box(dy, w, H, W, pad=1)
    assert_close(got, val, absum, f"dgrad {opd}")


@pytest.mark.parametrize("k", [2, 3, 4])
def test_dgrad_pnr_invariant_bit_exact(k):
    opd = dict(kind="conv2d_dgrad", batch=4, c_in=72, c_out=12, H=12, W=10, KH=3, KW=3, stride=1, pad=1)
    dy = synth.small_int(62, 0, (4, 12, 12, 10), -3, 3)
    w = synth.small_int(62, 1, (12, 72, 3, 3), -3, 3)
    ddy, dw = dev(dy), dev(w)
    want = oracle.dgrad_box(dy, w, 12, 10, pad=1)[0]
    for dim in ["N", "CI", "H", "W", "CO"]:
        got = assemble(opd, dim, k, lambda sp: run_dgrad(opd, sp, ddy, dw))
        assert np.array_equal(got.astype(np.float64), want), dim


def test_dgrad_on_blocks_and_strided_filters():
    """A <CO/2, H/2> shard from the blocks a worker holds: its half of dy's channels with the
    halo row, and its filter block as a strided view of the whole filter tensor; the partial is
    checked against the oracle restricted to the shard's output channels."""
    opd = dict(kind="conv2d_dgrad", batch=3, c_in=40, c_out=16, H=14, W=14, KH=3, KW=3, stride=1, pad=1)
    dy = synth.normal(63, 0, (3, 16, 14, 14), 1.0)
    w = synth.normal(63, 1, (16, 40, 3, 3), 0.3)
    dw_full = dev(w)
    op = tofu.dgrad_desc(3, 40, 16, 14, 14)
    for a, b in itertools.product(range(2), repeat=2):
        plan = [("CO", 2, a), ("H", 2, b)]
        sp = [(DGRAD_DIMS[d], k, s) for d, k, s in plan]
        reg = R.op_regions(opd, plan)
        lib = tofu.op_regions(op, sp)
        assert lib["in_boxes"][0] == [tuple(t) for t in reg["in_boxes"][0]] and lib["pad_lo"] == reg["pad_lo"]
        box = reg["in_boxes"][0]
        blk = dev(dy[R.box_slices(box)].copy())
        (c0, c1) = reg["ranges"]["CO"]
        dx = torch.full((3, 40, 14, 14), float("nan"), dtype=torch.float32, device=DEV)
        tofu.shard_conv2d_dgrad(op, sp, tofu.tensor(blk, [lo for lo, _ in box]), tofu.tensor(dw_full[c0:c1], [c0, 0, 0, 0]),
                                tofu.tensor(dx), workspace(op, sp))
        val, absum = oracle.dgrad_box(dy, w, 14, 14, pad=1, box=reg["out_box"], corange=(c0, c1))
        sl = R.box_slices(reg["out_box"])
        assert_close(dx.cpu().numpy()[sl], val, absum, f"dgrad {plan}")


# ----------------------------------------------------------------------------- reducers and orders
def _tree_f32(parts, op):
    """fold(l, r) = fold(l, m) op fold(m, r), m = l + ceil((r - l) / 2), in float32 like the kernel."""
    def fold(l, r):
        if r - l == 1:
            return parts[l]
        m = l + (r - l + 1) // 2
        return op(fold(l, m), fold(m, r))
    return fold(0, len(parts))


@pytest.mark.parametrize("k", [1, 2, 3, 5, 8, 16])
def test_reduce_reducers_and_orders(k):
    n = 4 * 50021 + 3                                    # vector body plus a scalar tail
    parts = [synth.normal(81, j, (n,), 1.5) for j in range(k)]
    d = [dev(p) for p in parts]
    out = torch.empty(n, dtype=torch.float32, device=DEV)
    # Max / Min: exact, equal to the oracle bit for bit
    for red, name in [(tofu.REDUCE_MAX, "max"), (tofu.REDUCE_MIN, "min")]:
        tofu.partition_reduce(out, d, reducer=red)
        assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.reduce_op(parts, name)[0]), name
    # Sum in both orders: within tolerance of the oracle, and bit-exact against the same order in float32
    val, absum = oracle.reduce(parts)
    tofu.partition_reduce(out, d, reducer=tofu.REDUCE_SUM, order=tofu.ORDER_LINEAR)
    lin = out.cpu().numpy()
    ref = parts[0].copy()
    for p in parts[1:]:
        ref = ref + p
    assert np.array_equal(lin, ref)
    plain = torch.empty_like(out)
    tofu.partition_reduce(plain, d)
    assert torch.equal(plain, out)                       # (SUM, LINEAR) is the plain entry point
    tofu.partition_reduce(out, d, reducer=tofu.REDUCE_SUM, order=tofu.ORDER_TREE)
    tree = out.cpu().numpy()
    assert np.array_equal(tree, _tree_f32(parts, lambda a, b: a + b))
    assert_close(tree, val, absum, "tree sum")
    # Prod: |gpu - oracle| <= 1e-5 |prod| (k - 1 roundings of 2^-24 each)
    small = [synth.uniform(82, j, (n,), 0.5, 1.5) for j in range(k)]
    ds = [dev(p) for p in small]
    pv, ps = oracle.reduce_op(small, "prod")
    for order in (tofu.ORDER_LINEAR, tofu.ORDER_TREE):
        tofu.partition_reduce(out, ds, reducer=tofu.REDUCE_PROD, order=order)
        assert_close(out.cpu().numpy(), pv, ps, f"prod order {order}")
    tofu.partition_reduce(out, ds, reducer=tofu.REDUCE_PROD, order=tofu.ORDER_TREE)
    assert np.array_equal(out.cpu().numpy(), _tree_f32(small, lambda a, b: a * b))


def test_reduce_nan_convention_in_place_and_scatter_share():
    a = np.array([np.nan, 1.0, np.nan, -2.0] * 8, np.float32)
    b = np.array([2.0, np.nan, np.nan, 5.0] * 8, np.float32)
    da, db = dev(a), dev(b)
    tofu.partition_reduce(da, [da, db], reducer=tofu.REDUCE_MAX)       # in place on partials[0]
    got = da.cpu().numpy()
    want = oracle.reduce_op([a, b], "max")[0]
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    # a reduce-scatter share: worker j sums slice j of every partial into slice j of the output
    k, n = 4, 4 * 1000
    parts = [synth.small_int(83, j, (n,), -50, 50) for j in range(k)]
    d = [dev(p) for p in parts]
    out = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    for j in range(k):
        lo, hi = R.shard_range(n, k, j)
        tofu.partition_reduce(out[lo:hi], [p[lo:hi] for p in d], reducer=tofu.REDUCE_SUM, order=tofu.ORDER_TREE)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), oracle.reduce(parts)[0])


# ----------------------------------------------------------------------------- lstm cell
@pytest.mark.parametrize("B,H", [(128, 1024), (5, 33), (1, 1), (64, 250)])
def test_lstm_cell_against_oracle_and_splits(B, H):
    """Element-wise stage after the gate GEMM: within 1e-5 of the fp64 oracle (c against
    |sig(f) c| + |sig(i) tanh(g)|, h against 1), and every split of batch or hidden units writes
    exactly the bits of the unsplit call."""
    g = synth.normal(91, 0, (B, H, 4), 3.0)
    g[0, 0] = [-100.0, 100.0, 50.0, 100.0]          # saturated gates stay finite
    c = synth.normal(91, 1, (B, H), 1.0)
    cn, hn, sc = oracle.lstm_cell(g, c)
    dg, dc = dev(g), dev(c)
    op = tofu.lstm_cell_desc(B, H)
    out_c = torch.full((B, H), float("nan"), dtype=torch.float32, device=DEV)
    out_h = torch.full((B, H), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_lstm_cell(op, [], tofu.tensor(dg), tofu.tensor(dc), tofu.tensor(out_c), tofu.tensor(out_h))
    assert_close(out_c.cpu().numpy(), cn, sc, "lstm c")
    assert_close(out_h.cpu().numpy(), hn, np.ones_like(hn), "lstm h")
    for dim, k in [(tofu.LSTM_DIM_B, 2), (tofu.LSTM_DIM_H, 3), (tofu.LSTM_DIM_H, 8)]:
        if (B if dim == tofu.LSTM_DIM_B else H) < k:
            continue
        pc = torch.full((B, H), float("nan"), dtype=torch.float32, device=DEV)
        ph = torch.full((B, H), float("nan"), dtype=torch.float32, device=DEV)
        for s in range(k):
            tofu.shard_lstm_cell(op, [(dim, k, s)], tofu.tensor(dg), tofu.tensor(dc), tofu.tensor(pc), tofu.tensor(ph))
        assert torch.equal(pc, out_c) and torch.equal(ph, out_h)


def test_lstm_cell_on_a_gate_gemm_shard_in_place():
    """The N-split worker's view: its block of gate columns (hidden units [h0,h1), four gates each)
    as produced by its GEMM shard, its block of the cell state updated in place."""
    B, H, k, s = 16, 64, 4, 2
    h0, h1 = R.shard_range(H, k, s)
    g = synth.normal(92, 0, (B, H, 4), 2.0)
    c = synth.normal(92, 1, (B, H), 1.0)
    cn, hn, sc = oracle.lstm_cell(g, c)
    g_blk = dev(g[:, h0:h1].copy())                       # [B, H/k, 4]: the GEMM shard's output columns 4*h0 .. 4*h1
    c_blk = dev(c[:, h0:h1].copy())
    h_full = torch.full((B, H), float("nan"), dtype=torch.float32, device=DEV)
    op = tofu.lstm_cell_desc(B, H)
    sp = [(tofu.LSTM_DIM_H, k, s)]
    tofu.shard_lstm_cell(op, sp, tofu.tensor(g_blk, [0, h0, 0]), tofu.tensor(c_blk, [0, h0]), tofu.tensor(c_blk, [0, h0]), tofu.tensor(h_full))
    assert_close(c_blk.cpu().numpy(), cn[:, h0:h1], sc[:, h0:h1], "in-place c block")
    got_h = h_full.cpu().numpy()
    assert_close(got_h[:, h0:h1], hn[:, h0:h1], np.ones((B, h1 - h0)), "h block")
    assert np.isnan(got_h[:, :h0]).all() and np.isnan(got_h[:, h1:]).all()


# ----------------------------------------------------------------------------- probes
def test_probes_copy_exactly_and_leave_the_sink_alone():
    """The measurement aids of tofu_probe.h: the copy is bit-exact on a ragged vector count,
    the MFMA loop writes nothing."""
    src = dev(synth.normal(77, 0, (4 * 100003,), 1.0))
    dst = torch.zeros_like(src)
    tofu.probe_copy(dst, src)
    assert torch.equal(dst, src)
    sink = torch.full((64,), 3.0, dtype=torch.float32, device=DEV)
    tofu.probe_mfma(sink, 16, 8)
    tofu.probe_read(src, sink)
    torch.cuda.synchronize()
    assert (sink == 3.0).all()
    # the k:1 stream: small integers, so the sum is exact; a ragged count exercises the last chunk
    for k in (1, 2, 4, 8):
        parts = [dev(synth.small_int(78, j, (4 * 70001,), -8, 8)) for j in range(k)]
        out = torch.zeros_like(parts[0])
        tofu.probe_stream(out, parts)
        assert torch.equal(out, torch.stack(parts).sum(0))


# ----------------------------------------------------------------------------- reduce-scatter share, fused accumulation
@pytest.mark.parametrize("count,shares", [(4 * 1000, 4), (10007, 3), (37, 8), (5, 8), ((1 << 20) + 3, 7)])
def test_reduce_scatter_shares_reproduce_the_whole_reduction(count, shares):
    """Every share writes only its range; all shares together equal tofu_partition_reduce_ex bit for bit
    (odd range starts exercise the kernel's scalar head before the aligned vectors)."""
    k = 5
    parts = [synth.normal(91, j, (count,), 1.0) for j in range(k)]
    d = [dev(p) for p in parts]
    for reducer, order, name in [(tofu.REDUCE_SUM, tofu.ORDER_LINEAR, "sum"), (tofu.REDUCE_SUM, tofu.ORDER_TREE, "sum"),
                                 (tofu.REDUCE_MAX, tofu.ORDER_LINEAR, "max")]:
        whole = torch.empty(count, dtype=torch.float32, device=DEV)
        tofu.partition_reduce(whole, d, reducer=reducer, order=order)
        out = torch.full((count,), float("nan"), dtype=torch.float32, device=DEV)
        for s in range(shares):
            before = out.clone()
            tofu.partition_reduce_scatter(out, d, shares, s, reducer=reducer, order=order)
            lo, hi = (s * count) // shares, ((s + 1) * count) // shares
            changed = (out != before) & ~(torch.isnan(out) & torch.isnan(before))
            idx = torch.nonzero(changed).flatten()
            assert idx.numel() == hi - lo and (idx.numel() == 0 or (int(idx.min()) == lo and int(idx.max()) == hi - 1)), (s, lo, hi)
        assert torch.equal(out, whole)
        val, absum = oracle.reduce_op(parts, name)
        if name == "sum":
            assert_close(out.cpu().numpy(), val, absum, "reduce-scatter sum")
        else:
            assert np.array_equal(out.cpu().numpy().astype(np.float64), val)
    # in place on partials[0]: share 1 of 3 only
    d0 = d[0].clone()
    tofu.partition_reduce_scatter(d0, [d0] + d[1:], 3, 1)
    lo, hi = count // 3, (2 * count) // 3
    ref = torch.empty(count, dtype=torch.float32, device=DEV)
    tofu.partition_reduce(ref, d)
    assert torch.equal(d0[lo:hi], ref[lo:hi]) and torch.equal(d0[:lo], d[0][:lo]) and torch.equal(d0[hi:], d[0][hi:])


def test_reduce_pointers_sharing_a_misalignment_take_the_vector_path_and_stay_exact():
    n = 70001
    parts = [synth.normal(92, j, (n + 3,), 2.0) for j in range(3)]
    d = [dev(p) for p in parts]
    for off in (1, 2, 3):
        out = torch.full((n + 3,), float("nan"), dtype=torch.float32, device=DEV)
        tofu.partition_reduce(out[off:off + n], [p[off:off + n] for p in d])
        val, absum = oracle.reduce([p[off:off + n] for p in parts])
        got = out.cpu().numpy()
        assert np.isnan(got[:off]).all() and np.isnan(got[off + n:]).all()
        assert_close(got[off:off + n], val, absum, f"reduce at offset {off}")
        # mixed phases fall back to element work and give the same bits
        out2 = torch.empty(n, dtype=torch.float32, device=DEV)
        tofu.partition_reduce(out2, [p[off:off + n].clone() if j else p[off:off + n] for j, p in enumerate(d)])
        assert torch.equal(out2, out[off:off + n])


def _accumulated(k, first, rest, out):
    """Shard 0 through the plain call, shards 1..k-1 through the accumulate call, all into `out`."""
    first(0, out)
    for s in range(1, k):
        rest(s, out)
    return out


@pytest.mark.parametrize("M,N,K,k", [(72, 136, 200, 4), (128, 256, 8192, 2), (33, 65, 1030, 3)])
def test_matmul_accumulate_equals_partials_then_reduce(M, N, K, k):
    """K-split shards added into one buffer == k partial buffers + left-to-right reduce, bit for bit
    (with and without the kernel's own K slices), and within tolerance of the oracle."""
    A = synth.normal(93, 0, (M, K), 1.0); B = synth.normal(93, 1, (K, N), 1.0)
    dA, dB = dev(A), dev(B)
    op = tofu.matmul_desc(M, N, K)
    tA, tB = tofu.tensor(dA), tofu.tensor(dB)
    parts = []
    for s in range(k):
        sp = [(tofu.MM_DIM_K, k, s)]
        C = torch.empty((M, N), dtype=torch.float32, device=DEV)
        tofu.shard_matmul(op, sp, tA, tB, tofu.tensor(C), workspace(op, sp))
        parts.append(C)
    want = torch.empty_like(parts[0])
    tofu.partition_reduce(want, parts)
    out = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    for s in range(k):
        sp = [(tofu.MM_DIM_K, k, s)]
        (tofu.shard_matmul if s == 0 else tofu.shard_matmul_accumulate)(op, sp, tA, tB, tofu.tensor(out), workspace(op, sp))
    assert torch.equal(out, want)
    val, absum = oracle.matmul_box(A, B)
    assert_close(out.cpu().numpy(), val, absum, "accumulated K split")
    # an output block of a larger, strided buffer: only the box is touched, and it is added to
    big = torch.full((M + 2, N + 5), 3.0, dtype=torch.float32, device=DEV)
    view = big[1:M + 1, 2:N + 2]
    tofu.shard_matmul_accumulate(op, [], tA, tB, tofu.tensor(view), workspace(op, []))
    whole = torch.empty((M, N), dtype=torch.float32, device=DEV)
    tofu.shard_matmul(op, [], tA, tB, tofu.tensor(whole), workspace(op, []))
    assert torch.equal(view, whole + 3.0)
    edge = big.clone(); edge[1:M + 1, 2:N + 2] = 3.0
    assert torch.equal(edge, torch.full_like(big, 3.0))


def test_conv_family_accumulate_equals_partials_then_reduce():
    """The three convolution operators with their reduction index split: accumulate == partials + reduce."""
    batch, c_in, c_out, H, W = 6, 40, 70, 12, 10
    x = synth.normal(94, 0, (batch, c_in, H, W), 1.0)
    w = synth.normal(94, 1, (c_out, c_in, 3, 3), 0.1)
    dy = synth.normal(94, 2, (batch, c_out, H, W), 1.0)
    dx_, dw_, ddy = dev(x), dev(w), dev(dy)
    cases = [
        ("conv2d CI split", tofu.conv2d_desc(batch, c_in, c_out, H, W), tofu.CONV_DIM_CI, 4, (dx_, dw_), (batch, c_out, H, W),
         tofu.shard_conv2d, tofu.shard_conv2d_accumulate, lambda: oracle.conv2d_box(x, w, pad=1)),
        ("wgrad N split", tofu.wgrad_desc(batch, c_in, c_out, H, W), tofu.WGRAD_DIM_N, 3, (dx_, ddy), (c_out, c_in, 3, 3),
         tofu.shard_conv2d_wgrad, tofu.shard_conv2d_wgrad_accumulate, lambda: oracle.wgrad_box(x, dy, 3, 3, pad=1)),
        ("dgrad CO split", tofu.dgrad_desc(batch, c_in, c_out, H, W), tofu.DGRAD_DIM_CO, 5, (ddy, dw_), (batch, c_in, H, W),
         tofu.shard_conv2d_dgrad, tofu.shard_conv2d_dgrad_accumulate, lambda: oracle.dgrad_box(dy, w, H, W, pad=1)),
    ]
    for name, op, dim, k, (a, b), shape, plain, acc, ref in cases:
        ta, tb = tofu.tensor(a), tofu.tensor(b)
        parts = []
        for s in range(k):
            o = torch.empty(shape, dtype=torch.float32, device=DEV)
            plain(op, [(dim, k, s)], ta, tb, tofu.tensor(o), workspace(op, [(dim, k, s)]))
            parts.append(o)
        want = torch.empty_like(parts[0])
        tofu.partition_reduce(want, parts)
        out = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
        for s in range(k):
            (plain if s == 0 else acc)(op, [(dim, k, s)], ta, tb, tofu.tensor(out), workspace(op, [(dim, k, s)]))
        assert torch.equal(out, want), name
        val, absum = ref()
        assert_close(out.cpu().numpy(), val, absum, name)


def test_wgrad_accumulate_through_workspace_segments():
    """A batch-split weight gradient whose tiles are summed from workspace segments adds to dw after the segment sum."""
    co, ci, nb = 256, 96, 8
    opd = dict(batch=nb, c_in=ci, c_out=co, H=14, W=14, pad=1)
    x = synth.normal(95, 0, (nb, ci, 14, 14), 1.0)
    dy = synth.normal(95, 1, (nb, co, 14, 14), 1.0)
    op = tofu.wgrad_desc(nb, ci, co, 14, 14)
    assert tofu.workspace_bytes(op, [(tofu.WGRAD_DIM_N, 2, 0)]) > 0
    d_x, d_dy = dev(x), dev(dy)          # the descriptors hold addresses only: keep the buffers alive
    tx, tdy = tofu.tensor(d_x), tofu.tensor(d_dy)
    parts = []
    for s in range(2):
        o = torch.empty((co, ci, 3, 3), dtype=torch.float32, device=DEV)
        tofu.shard_conv2d_wgrad(op, [(tofu.WGRAD_DIM_N, 2, s)], tx, tdy, tofu.tensor(o), workspace(op, [(tofu.WGRAD_DIM_N, 2, s)]))
        parts.append(o)
    out = parts[0].clone()
    tofu.shard_conv2d_wgrad_accumulate(op, [(tofu.WGRAD_DIM_N, 2, 1)], tx, tdy, tofu.tensor(out), workspace(op, [(tofu.WGRAD_DIM_N, 2, 1)]))
    want = torch.empty_like(out)
    tofu.partition_reduce(want, parts)
    assert torch.equal(out, want)
    val, absum = oracle.wgrad_box(x, dy, 3, 3, pad=1)
    assert_close(out.cpu().numpy(), val, absum, "accumulated wgrad")


# ----------------------------------------------------------------------------- conv1d (the paper's running example)
CONV1D_DIMS = {"B": tofu.CONV1D_DIM_B, "CO": tofu.CONV1D_DIM_CO, "X": tofu.CONV1D_DIM_X, "CI": tofu.CONV1D_DIM_CI}


def run_conv1d(opd, splits, d_data, d_filt, data_lo=None, call=None, out=None):
    op = tofu.conv1d_desc(opd["batch"], opd["c_in"], opd["c_out"], opd["W"])
    sp = [(CONV1D_DIMS[d], k, s) for d, k, s in splits]
    if out is None:
        out = torch.full((opd["batch"], opd["c_out"], opd["W"] - 2), float("nan"), dtype=torch.float32, device=DEV)
    (call or tofu.shard_conv1d)(op, sp, tofu.tensor(d_data, data_lo), tofu.tensor(d_filt), tofu.tensor(out), workspace(op, sp))
    return out


@pytest.mark.parametrize("B,CI,CO,X", [(3, 16, 70, 64), (2, 5, 33, 37), (4, 24, 64, 256), (2, 12, 10, 1024), (1, 4, 3, 1), (2, 8, 130, 2048),
                                       (5, 7, 9, 100)])
def test_conv1d_shapes_unpartitioned(B, CI, CO, X):
    data = synth.uniform(130, 0, (B, CI, X + 2), -1, 1)
    filt = synth.uniform(130, 1, (CI, CO, 3), -1, 1)
    opd = dict(kind="conv1d", batch=B, c_in=CI, c_out=CO, W=X + 2, KW=3)
    got = run_conv1d(opd, [], dev(data), dev(filt)).cpu().numpy()
    val, absum = oracle.conv1d_box(data, filt)
    assert_close(got, val, absum, f"conv1d {B}x{CI}x{CO}x{X}")


@pytest.mark.parametrize("k", [2, 3, 4])
def test_conv1d_pnr_invariant_bit_exact(k):
    B, CI, CO, X = 4, 36, 72, 96
    data = synth.small_int(131, 0, (B, CI, X + 2), -3, 3)
    filt = synth.small_int(131, 1, (CI, CO, 3), -3, 3)
    d_data, d_filt = dev(data), dev(filt)
    opd = dict(kind="conv1d", batch=B, c_in=CI, c_out=CO, W=X + 2, KW=3)
    want = oracle.conv1d_box(data, filt)[0]
    for dim in ["B", "CO", "X", "CI"]:
        got = assemble(opd, dim, k, lambda sp: run_conv1d(opd, sp, d_data, d_filt))
        assert np.array_equal(got.astype(np.float64), want), dim


def test_conv1d_filter_layouts_halo_block_and_accumulate():
    B, CI, CO, X = 3, 40, 64, 128
    data = synth.normal(132, 0, (B, CI, X + 2), 1.0)
    filt = synth.normal(132, 1, (CI, CO, 3), 0.2)
    opd = dict(kind="conv1d", batch=B, c_in=CI, c_out=CO, W=X + 2, KW=3)
    d_data, d_filt = dev(data), dev(filt)
    val, absum = oracle.conv1d_box(data, filt)
    base = run_conv1d(opd, [], d_data, d_filt)
    assert_close(base.cpu().numpy(), val, absum, "conv1d dense [ci][co][dx] filters")
    # the same filters held as [co][ci][dx] and passed as a permuted view are read in place: same bits
    phys = d_filt.permute(1, 0, 2).contiguous()
    view = phys.permute(1, 0, 2)
    assert view.shape == d_filt.shape and view.stride() == (3, 3 * CI, 1)
    assert torch.equal(run_conv1d(opd, [], d_data, view), base)
    # an X shard computed from a block that holds exactly its window-widened range
    sp = [("X", 4, 2)]
    reg = R.op_regions(opd, sp)
    (x0, x1) = reg["in_boxes"][0][2]
    block = d_data[:, :, x0:x1].contiguous()
    got = run_conv1d(opd, sp, block, d_filt, data_lo=[0, 0, x0])
    (o0, o1) = reg["out_box"][2]
    assert torch.equal(got[:, :, o0:o1], base[:, :, o0:o1])
    assert torch.isnan(got[:, :, :o0]).all() and torch.isnan(got[:, :, o1:]).all()
    # CI shards added into one buffer == partial buffers + reduce
    k = 4
    parts = [run_conv1d(opd, [("CI", k, s)], d_data, d_filt) for s in range(k)]
    want = torch.empty_like(parts[0])
    tofu.partition_reduce(want, parts)
    out = torch.full_like(want, float("nan"))
    for s in range(k):
        run_conv1d(opd, [("CI", k, s)], d_data, d_filt, call=tofu.shard_conv1d if s == 0 else tofu.shard_conv1d_accumulate, out=out)
    assert torch.equal(out, want)
    assert_close(out.cpu().numpy(), val, absum, "conv1d accumulated CI split")


def test_conv1d_length_without_a_suitable_divisor_is_reported():
    B, CI, CO, X = 1, 4, 4, 521          # a prime: rows of one column would stage 256 rows per tile
    opd = dict(kind="conv1d", batch=B, c_in=CI, c_out=CO, W=X + 2, KW=3)
    d_data = torch.zeros(B, CI, X + 2, device=DEV); d_filt = torch.zeros(CI, CO, 3, device=DEV)
    with pytest.raises(tofu.TofuError) as e:
        run_conv1d(opd, [], d_data, d_filt)
    assert e.value.status == -6


def test_matmul_reads_an_operand_held_in_row_blocks_without_assembling_it():
    """The paper's example of a matrix product cut twice (Sec. 5.2): a worker that computes rows of C needs
    all of B, which is held as k row blocks (its own and the fetched ones).  One call per block, the later
    ones accumulating, reads every block in place -- no assembled copy of B -- and equals the K-split
    partials reduced left to right bit for bit."""
    M, N, K, k = 96, 200, 512, 4
    A = synth.normal(140, 0, (M, K), 1.0); B = synth.normal(140, 1, (K, N), 1.0)
    dA = dev(A)
    op = tofu.matmul_desc(M, N, K)
    rows = [R.shard_range(K, k, j) for j in range(k)]
    blocks = [dev(B[lo:hi]) for lo, hi in rows]                      # k separate buffers, never concatenated
    m_split = (tofu.MM_DIM_M, 2, 1)                                  # this worker's rows of C
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    for j, (lo, hi) in enumerate(rows):
        sp = [m_split, (tofu.MM_DIM_K, k, j)]
        call = tofu.shard_matmul if j == 0 else tofu.shard_matmul_accumulate
        call(op, sp, tofu.tensor(dA), tofu.tensor(blocks[j], [lo, 0]), tofu.tensor(C), workspace(op, sp))
    got = C.cpu().numpy()
    m0, m1 = R.shard_range(M, 2, 1)
    assert np.isnan(got[:m0]).all() and not np.isnan(got[m0:m1]).any()
    val, absum = oracle.matmul_box(A, B, box=[(m0, m1), (0, N)])
    assert_close(got[m0:m1], val, absum, "matmul over row blocks of B")
    # the same through k partial buffers and the reduce
    dB = dev(B)
    parts = []
    for j in range(k):
        P = torch.zeros((M, N), dtype=torch.float32, device=DEV)
        sp = [m_split, (tofu.MM_DIM_K, k, j)]
        tofu.shard_matmul(op, sp, tofu.tensor(dA), tofu.tensor(dB), tofu.tensor(P), workspace(op, sp))
        parts.append(P)
    want = torch.empty_like(parts[0])
    tofu.partition_reduce(want, parts)
    assert torch.equal(C[m0:m1], want[m0:m1])
    # a block that does not hold the rows of its step is refused, never read as zeros
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_matmul(op, [m_split, (tofu.MM_DIM_K, k, 1)], tofu.tensor(dA), tofu.tensor(blocks[0], [0, 0]), tofu.tensor(C))
    assert e.value.status == -2


# ----------------------------------------------------------------------------- from a searched plan to executed shards
def _nested_box(shape, cuts):
    """Box of a tensor held after the nested cuts [(dim, k, part), ...] (each cuts the range left by the earlier ones)."""
    box = [(0, e) for e in shape]
    for d, k, part in cuts:
        lo, hi = box[d]
        a, b = R.shard_range(hi - lo, k, part)
        box[d] = (lo + a, lo + b)
    return box


@pytest.mark.parametrize("kind", ["matmul", "conv1d"])
def test_searched_plan_drives_fetch_shard_and_reduce(kind):
    """The whole path for four workers: search a recursive plan (2 x 2), hold every tensor cut as the plan says,
    and for each worker fetch its input regions from the owners' blocks, run its shard, then sum the partials of
    workers that share an output box and place the result -- the unpartitioned operator comes out."""
    from paper_1807_08887_amd import plan as L, tdl as T
    ks = [2, 2]
    if kind == "matmul":
        M, N, K = 64, 96, 160
        op = tofu.matmul_desc(M, N, K)
        ins = [synth.small_int(150, 0, (M, K), -3, 3), synth.small_int(150, 1, (K, N), -3, 3)]
        want = oracle.matmul_box(*ins)[0]
        run = tofu.shard_matmul
    else:
        B, CI, CO, X = 4, 24, 64, 64
        op = tofu.conv1d_desc(B, CI, CO, X + 2)
        ins = [synth.small_int(151, 0, (B, CI, X + 2), -3, 3), synth.small_int(151, 1, (CI, CO, 3), -3, 3)]
        want = oracle.conv1d_box(*ins)[0]
        run = tofu.shard_conv1d
    desc = T.from_op(op)
    g = L.graph(3, [(desc, [0, 1], 2, 0)])
    res = L.recursive(g, ks)
    n_workers = ks[0] * ks[1]
    digits = [(w // ks[1], w % ks[1]) for w in range(n_workers)]
    # every worker's block of each input, as separate device buffers
    held = []
    for t in range(2):
        blocks = []
        for w in range(n_workers):
            box = _nested_box(ins[t].shape, [(res["tensor_dim"][s][t], ks[s], digits[w][s]) for s in range(2)])
            blocks.append((box, dev(ins[t][R.box_slices(box)])))
        held.append(blocks)
    out = torch.full(want.shape, float("nan"), dtype=torch.float32, device=DEV)
    partials = {}
    for w in range(n_workers):
        sp = L.worker_splits(res["op_var"], ks, 0, w)
        assert all(v < desc.n_vars - (1 if kind == "conv1d" else 0) for v, _, _ in sp)      # a variable the shard calls can cut
        reg = tofu.op_regions(op, sp)
        fetched = []
        for t in range(2):
            box = reg["in_boxes"][t]
            dst = torch.empty([hi - lo for lo, hi in box], dtype=torch.float32, device=DEV)
            tofu.region_fetch(tofu.tensor(dst, [lo for lo, _ in box]), [tofu.tensor(b, [lo for lo, _ in bx]) for bx, b in held[t]])
            fetched.append(tofu.tensor(dst, [lo for lo, _ in box]))
            fetched.append(dst)                                                          # keep the buffer alive
        part = torch.zeros(want.shape, dtype=torch.float32, device=DEV)
        run(op, sp, fetched[0], fetched[2], tofu.tensor(part), workspace(op, sp))
        partials.setdefault(tuple(map(tuple, reg["out_box"])), []).append(part)
    assert sum(len(v) for v in partials.values()) == n_workers
    for box, parts in partials.items():
        sl = R.box_slices(list(box))
        if len(parts) == 1:
            out[sl] = parts[0][sl]
        else:                      # Case-2 somewhere in the plan: the workers that share this box hold partial sums
            total = torch.empty_like(parts[0])
            tofu.partition_reduce(total, parts)
            out[sl] = total[sl]
    assert np.array_equal(out.cpu().numpy().astype(np.float64), want)
    # what the plan says it costs is what the fetches moved in its first step: elements read from other groups' blocks
    assert res["total"] == sum(res["step_elements"]) and res["step_elements"][0] <= res["step_elements"][1]


def test_searched_plan_for_a_training_layer_forward_and_backward():
    """One fully-connected layer with its two backward products as ONE operator group (Sec. 5.1): the search may
    cut forward and backward tensors differently.  Four workers execute all three products of their shards from
    blocks held as the plan says (the backward products read W and X through transposed views of the fetched
    regions); Y, dX and dW all come out bit-exact."""
    from paper_1807_08887_amd import plan as L, tdl as T
    Bt, D0, D1, ks = 48, 96, 160, [2, 2]
    X = synth.small_int(160, 0, (Bt, D0), -3, 3); W = synth.small_int(160, 1, (D0, D1), -3, 3); dY = synth.small_int(160, 2, (Bt, D1), -3, 3)
    iX, iW, iY, idY, idX, idW = range(6)
    host = {iX: X, iW: W, idY: dY}
    shapes = {iX: (Bt, D0), iW: (D0, D1), iY: (Bt, D1), idY: (Bt, D1), idX: (Bt, D0), idW: (D0, D1)}
    one = lambda v: {v: 1}
    # (description, inputs, output, matmul extents (M, N, K), which inputs are read transposed)
    ops = [
        (T.describe([Bt, D1, D0], 2, [((Bt, D0), [one(0), one(2)]), ((D0, D1), [one(2), one(1)])]), [iX, iW], iY, (Bt, D1, D0), (False, False)),
        (T.describe([Bt, D0, D1], 2, [((Bt, D1), [one(0), one(2)]), ((D0, D1), [one(1), one(2)])]), [idY, iW], idX, (Bt, D0, D1), (False, True)),
        (T.describe([D0, D1, Bt], 2, [((Bt, D0), [one(2), one(0)]), ((Bt, D1), [one(2), one(1)])]), [iX, idY], idW, (D0, D1, Bt), (True, False)),
    ]
    g = L.graph(6, [(d, ins, out, 0) for d, ins, out, _, _ in ops])
    res = L.recursive(g, ks)
    n_workers = ks[0] * ks[1]
    digits = [(w // ks[1], w % ks[1]) for w in range(n_workers)]
    held = {}
    for t, arr in host.items():
        held[t] = []
        for w in range(n_workers):
            box = _nested_box(arr.shape, [(res["tensor_dim"][s][t], ks[s], digits[w][s]) for s in range(2)])
            held[t].append((box, dev(arr[R.box_slices(box)])))
    results = {}
    for o, (desc, ins, out_t, (M, N, K), transposed) in enumerate(ops):
        mm = tofu.matmul_desc(M, N, K)
        partials = {}
        for w in range(n_workers):
            sp = L.worker_splits(res["op_var"], ks, o, w)          # variables (0, 1, 2) are the product's (M, N, K)
            need = T.regions(desc, sp)                              # boxes in the tensors' own coordinates
            mreg = tofu.op_regions(mm, sp)
            operands, keep = [], []
            for i, t in enumerate(ins):
                box = need["in_boxes"][i]
                dst = torch.empty([hi - lo for lo, hi in box], dtype=torch.float32, device=DEV)
                tofu.region_fetch(tofu.tensor(dst, [lo for lo, _ in box]), [tofu.tensor(b, [lo for lo, _ in bx]) for bx, b in held[t]])
                keep.append(dst)
                lo = [lo for lo, _ in box]
                operands.append(tofu.tensor(dst.t(), lo[::-1]) if transposed[i] else tofu.tensor(dst, lo))
            # the fetched regions are exactly what the product's shard reads, seen through the views
            for i in range(2):
                want_box = [tuple(b) for b in (need["in_boxes"][i][::-1] if transposed[i] else need["in_boxes"][i])]
                assert [tuple(b) for b in mreg["in_boxes"][i]] == want_box
            part = torch.zeros((M, N), dtype=torch.float32, device=DEV)
            tofu.shard_matmul(mm, sp, operands[0], operands[1], tofu.tensor(part), workspace(mm, sp))
            partials.setdefault(tuple(map(tuple, mreg["out_box"])), []).append(part)
        out = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        for box, parts in partials.items():
            sl = R.box_slices(list(box))
            total = parts[0]
            if len(parts) > 1:
                total = torch.empty_like(parts[0])
                tofu.partition_reduce(total, parts)
            out[sl] = total[sl]
        results[out_t] = out.cpu().numpy().astype(np.float64)
    assert np.array_equal(results[iY], oracle.matmul_box(X, W)[0])
    assert np.array_equal(results[idX], oracle.matmul_box(dY, np.ascontiguousarray(W.T))[0])
    assert np.array_equal(results[idW], oracle.matmul_box(np.ascontiguousarray(X.T), dY)[0])
    assert res["step_elements"][0] <= res["step_elements"][1]
