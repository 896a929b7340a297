"""CPU tests of the C-ABI library's host side: it loads, exports every symbol the header
declares, its integer arithmetic (shard ranges, plans, regions, residual padding) is bit-exact
against the oracle's independent Python definitions, and every host-checked error path
returns its status before anything could be launched.  No compute call is made."""
import ctypes
import itertools
import os
import re

import pytest

import paper_1807_08887_amd as tofu
from oracle import regions as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000        # a non-null "device pointer"; nothing below ever dereferences it


def test_library_exports_every_declared_symbol():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["tofu.h", "tofu_plan.h", "tofu_probe.h", "tofu_tdl.h"]
    names = set()
    for h in headers:
        names |= set(re.findall(r"^(?:int|size_t|const char\*)\s+(tofu_[a-z0-9_]+)\s*\(", open(h).read(), flags=re.M))
    assert {"tofu_region_fetch", "tofu_shard_matmul", "tofu_shard_conv2d", "tofu_shard_conv2d_wgrad",
            "tofu_partition_reduce", "tofu_shard_range", "tofu_op_regions", "tofu_workspace_bytes",
            "tofu_last_error", "tofu_probe_mfma", "tofu_probe_copy", "tofu_shard_conv2d_fused", "tofu_shard_conv2d_dgrad", "tofu_partition_reduce_ex", "tofu_tdl_regions", "tofu_tdl_symbolic", "tofu_tdl_from_op",
            "tofu_tdl_fetch_elements", "tofu_shard_lstm_cell", "tofu_partition_reduce_scatter", "tofu_shard_matmul_accumulate",
            "tofu_shard_conv2d_accumulate", "tofu_shard_conv2d_wgrad_accumulate", "tofu_shard_conv2d_dgrad_accumulate",
            "tofu_plan_strategy_cost", "tofu_plan_cost", "tofu_plan_basic", "tofu_plan_recursive", "tofu_shard_conv1d",
            "tofu_shard_conv1d_accumulate"} <= names
    lib = ctypes.CDLL(tofu.lib_path())
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in include/ but not exported"


def test_shard_range_matches_oracle_exhaustively():
    for D in range(1, 65):
        for k in range(1, min(D, 9) + 1):
            for s in range(k):
                assert tofu.shard_range(D, k, s) == R.shard_range(D, k, s)
    big = (1 << 62) + 12345          # shard * extent overflows 64 bits without a wide multiply
    assert tofu.shard_range(big, 7, 6) == R.shard_range(big, 7, 6)
    for bad in [(-1, 1, 0), (4, 0, 0), (4, 2, 2), (4, 2, -1), (3, 4, 0)]:
        with pytest.raises(tofu.TofuError) as e:
            tofu.shard_range(*bad)
        assert e.value.status == -1


def _desc(op):
    if op["kind"] == "lstm_cell":
        return tofu.lstm_cell_desc(op["batch"], op["hidden"]), {"B": 0, "H": 1}
    if op["kind"] == "matmul":
        return tofu.matmul_desc(op["M"], op["N"], op["K"]), {"M": 0, "N": 1, "K": 2}
    if op["kind"] == "conv1d":
        return tofu.conv1d_desc(op["batch"], op["c_in"], op["c_out"], op["W"], op["KW"]), {"B": 0, "CO": 1, "X": 2, "CI": 3}
    args = (op["batch"], op["c_in"], op["c_out"], op["H"], op["W"], op["KH"], op["KW"], op["stride"], op["pad"])
    if op["kind"] == "conv2d":
        return tofu.conv2d_desc(*args), {"N": 0, "CO": 1, "H": 2, "W": 3, "CI": 4}
    if op["kind"] == "conv2d_dgrad":
        return tofu.dgrad_desc(*args), {"N": 0, "CI": 1, "H": 2, "W": 3, "CO": 4}
    return tofu.wgrad_desc(*args), {"CO": 0, "CI": 1, "N": 2}


def _same(lib, ref):
    assert lib["out_box"] == [tuple(b) for b in ref["out_box"]]
    assert lib["in_boxes"] == [[tuple(b) for b in box] for box in ref["in_boxes"]]
    assert lib["pad_lo"] == ref["pad_lo"] and lib["pad_hi"] == ref["pad_hi"]
    assert lib["is_partial"] == ref["is_partial"]


OPS = [
    dict(kind="matmul", M=13, N=9, K=21),
    dict(kind="conv2d", batch=5, c_in=7, c_out=6, H=11, W=9, KH=3, KW=3, stride=1, pad=1),
    dict(kind="conv2d", batch=4, c_in=4, c_out=4, H=12, W=13, KH=5, KW=3, stride=2, pad=2),
    dict(kind="conv2d", batch=4, c_in=4, c_out=4, H=9, W=9, KH=3, KW=3, stride=1, pad=0),
    dict(kind="conv2d_wgrad", batch=6, c_in=5, c_out=7, H=8, W=10, KH=3, KW=3, stride=1, pad=1),
    dict(kind="conv2d_wgrad", batch=6, c_in=5, c_out=7, H=9, W=10, KH=3, KW=2, stride=2, pad=0),
    dict(kind="conv2d_dgrad", batch=5, c_in=7, c_out=6, H=11, W=9, KH=3, KW=3, stride=1, pad=1),
    dict(kind="conv2d_dgrad", batch=4, c_in=4, c_out=4, H=9, W=9, KH=3, KW=3, stride=1, pad=0),
    dict(kind="conv2d_dgrad", batch=4, c_in=4, c_out=4, H=12, W=13, KH=5, KW=3, stride=2, pad=2),
    dict(kind="lstm_cell", batch=6, hidden=10),
    dict(kind="conv1d", batch=4, c_in=6, c_out=8, W=14, KW=3),
    dict(kind="conv1d", batch=3, c_in=5, c_out=4, W=11, KW=5),
]


@pytest.mark.parametrize("op", OPS, ids=lambda o: f"{o['kind']}-{o.get('stride', 0)}-{o.get('pad', 0)}")
def test_regions_match_oracle_for_one_and_two_step_plans(op):
    desc, dims = _desc(op)
    ext = R.iteration_extents(op)
    _same(tofu.op_regions(desc, []), R.op_regions(op, []))
    steps = [(d, k, s) for d in dims for k in range(1, min(ext[d], 4) + 1) for s in range(k)]
    for st in steps:
        _same(tofu.op_regions(desc, [(dims[st[0]], st[1], st[2])]), R.op_regions(op, [st]))
    for a, b in itertools.product(steps, repeat=2):
        try:
            ref = R.op_regions(op, [a, b])
        except ValueError:
            with pytest.raises(tofu.TofuError):
                tofu.op_regions(desc, [(dims[a[0]], a[1], a[2]), (dims[b[0]], b[1], b[2])])
            continue
        _same(tofu.op_regions(desc, [(dims[a[0]], a[1], a[2]), (dims[b[0]], b[1], b[2])]), ref)


def test_workload_regions():
    """The five workloads' ranges: 128->64, 96->48; 32768->4096, 16384->2048, 2560->320, 128->16; 14->7 with halo."""
    mm = tofu.matmul_desc(128, 32768, 16384)
    assert tofu.op_regions(mm, [(tofu.MM_DIM_N, 8, 3)])["in_boxes"][1] == [(0, 16384), (12288, 16384)]
    r = tofu.op_regions(mm, [(tofu.MM_DIM_K, 8, 3)])
    assert r["in_boxes"] == [[(0, 128), (6144, 8192)], [(6144, 8192), (0, 32768)]] and r["is_partial"]
    cv = tofu.conv2d_desc(128, 2560, 2560, 14, 14)
    r0 = tofu.op_regions(cv, [(tofu.CONV_DIM_CO, 8, 3), (tofu.CONV_DIM_H, 2, 0)])
    r1 = tofu.op_regions(cv, [(tofu.CONV_DIM_CO, 8, 3), (tofu.CONV_DIM_H, 2, 1)])
    assert r0["in_boxes"][0][2] == (0, 8) and (r0["pad_lo"][0], r0["pad_hi"][0]) == (1, 0)
    assert r1["in_boxes"][0][2] == (6, 14) and (r1["pad_lo"][0], r1["pad_hi"][0]) == (0, 1)
    assert r0["out_box"] == [(0, 128), (960, 1280), (0, 7), (0, 14)]
    wg = tofu.wgrad_desc(128, 1280, 1280, 28, 28)
    r = tofu.op_regions(wg, [(tofu.WGRAD_DIM_N, 8, 3)])
    assert r["is_partial"] and r["out_box"] == [(0, 1280), (0, 1280), (0, 3), (0, 3)] and r["in_boxes"][0][0] == (48, 64)
    # three 2-way steps on one dimension equal one 8-way step when 8 divides the extent
    for s in range(8):
        plan = [(tofu.MM_DIM_N, 2, (s >> 2) & 1), (tofu.MM_DIM_N, 2, (s >> 1) & 1), (tofu.MM_DIM_N, 2, s & 1)]
        assert tofu.op_regions(mm, plan)["out_box"] == tofu.op_regions(mm, [(tofu.MM_DIM_N, 8, s)])["out_box"]


def _t(box, data=FAKE, stride=None):
    t = tofu.Tensor()
    t.data = data
    t.extent = tofu.Region.from_box(box)
    for i, s in enumerate(stride or []):
        t.stride[i] = s
    return t


def test_fetch_error_paths_are_checked_on_the_host():
    dst = _t([(0, 4), (0, 8)])
    left, right = _t([(0, 4), (0, 4)], FAKE + (1 << 20)), _t([(0, 4), (4, 8)], FAKE + (2 << 20))
    with pytest.raises(tofu.TofuError) as e:
        tofu.region_fetch(dst, [left], stream=0)
    assert e.value.status == -3 and "16 of the 32" in str(e.value)               # UNCOVERED
    with pytest.raises(tofu.TofuError) as e:
        tofu.region_fetch(dst, [left, right, _t([(2, 4), (3, 5)], FAKE + (3 << 20))], stream=0)
    assert e.value.status == -4                                                   # OVERLAP
    with pytest.raises(tofu.TofuError) as e:
        tofu.region_fetch(dst, [left, _t([(0, 4), (4, 8), (0, 1)], FAKE + (2 << 20))], stream=0)
    assert e.value.status == -1                                                   # ndim mismatch
    with pytest.raises(tofu.TofuError) as e:
        tofu.region_fetch(dst, [left, _t([(0, 4), (4, 8)], FAKE + 16)], stream=0)
    assert e.value.status == -1 and "overlaps" in str(e.value)                    # dst aliases a source
    with pytest.raises(tofu.TofuError) as e:
        tofu.region_fetch(dst, [left] * 17, stream=0)
    assert e.value.status == -1                                                   # too many sources
    with pytest.raises(tofu.TofuError) as e:
        tofu.region_fetch(_t([(0, 4), (0, 8)], data=None), [left, right], stream=0)
    assert e.value.status == -1


def test_shard_call_error_paths_are_checked_on_the_host():
    mm = tofu.matmul_desc(64, 96, 128)
    A, B, C = _t([(0, 64), (0, 128)]), _t([(0, 128), (0, 96)], FAKE + (1 << 20)), _t([(0, 64), (0, 96)], FAKE + (2 << 20))
    with pytest.raises(tofu.TofuError) as e:      # B block lacks the K range this shard reads
        tofu.shard_matmul(mm, [(tofu.MM_DIM_K, 2, 1)], A, _t([(0, 64), (0, 96)], FAKE + (1 << 20)), C, stream=0)
    assert e.value.status == -2 and "B does not hold" in str(e.value)
    with pytest.raises(tofu.TofuError) as e:      # split names a dimension the operator does not have
        tofu.shard_matmul(mm, [(3, 2, 0)], A, B, C, stream=0)
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:      # wrong operator kind for the entry point
        tofu.shard_conv2d(mm, [], A, B, C, stream=0)
    assert e.value.status == -1
    big = tofu.matmul_desc(128, 4096, 16384)      # needs split-K workspace
    assert tofu.workspace_bytes(big, []) > 0
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_matmul(big, [], _t([(0, 128), (0, 16384)]), _t([(0, 16384), (0, 4096)], FAKE + (1 << 30)),
                          _t([(0, 128), (0, 4096)], FAKE + (2 << 30)), stream=0)
    assert e.value.status == -5
    cv = tofu.conv2d_desc(2, 4, 4, 8, 8, KH=5, KW=5, pad=2)
    x, w, y = _t([(0, 2), (0, 4), (0, 8), (0, 8)]), _t([(0, 4), (0, 4), (0, 5), (0, 5)], FAKE + (1 << 20)), _t([(0, 2), (0, 4), (0, 8), (0, 8)], FAKE + (2 << 20))
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv2d(cv, [], x, w, y, stream=0)
    assert e.value.status == -6                   # UNSUPPORTED filter size
    cv = tofu.conv2d_desc(2, 4, 4, 8, 8)
    with pytest.raises(tofu.TofuError) as e:      # halo row 4 missing from a 4-row block
        tofu.shard_conv2d(cv, [(tofu.CONV_DIM_H, 2, 0)], _t([(0, 2), (0, 4), (0, 4), (0, 8)]),
                          _t([(0, 4), (0, 4), (0, 3), (0, 3)], FAKE + (1 << 20)), y, stream=0)
    assert e.value.status == -2
    wg = tofu.wgrad_desc(16, 64, 64, 8, 8)
    assert tofu.workspace_bytes(wg, []) > 0
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv2d_wgrad(wg, [], _t([(0, 16), (0, 64), (0, 8), (0, 8)]), _t([(0, 16), (0, 64), (0, 8), (0, 8)], FAKE + (1 << 20)),
                                _t([(0, 64), (0, 64), (0, 3), (0, 3)], FAKE + (2 << 20)), stream=0)
    assert e.value.status == -5


def test_dgrad_error_paths_are_checked_on_the_host():
    dg = tofu.dgrad_desc(2, 4, 64, 8, 8)
    dy, w = _t([(0, 2), (0, 64), (0, 8), (0, 8)]), _t([(0, 64), (0, 4), (0, 3), (0, 3)], FAKE + (1 << 20))
    dx = _t([(0, 2), (0, 4), (0, 8), (0, 8)], FAKE + (2 << 20))
    # reversed filters (rounded up to 256 bytes) plus the convolution's segment slots
    flip = 64 * 4 * 9 * 4
    assert tofu.workspace_bytes(dg, []) >= flip and tofu.workspace_bytes(dg, []) % 256 == 0
    small = tofu.workspace_bytes(dg, [(tofu.DGRAD_DIM_CO, 4, 1), (tofu.DGRAD_DIM_CI, 2, 0)])
    assert (16 * 2 * 9 * 4 + 255) // 256 * 256 <= small <= tofu.workspace_bytes(dg, [])
    with pytest.raises(tofu.TofuError) as e:      # no workspace for the reversed filters
        tofu.shard_conv2d_dgrad(dg, [], dy, w, dx, stream=0)
    assert e.value.status == -5
    with pytest.raises(tofu.TofuError) as e:      # a forward description handed to the gradient entry point
        tofu.shard_conv2d_dgrad(tofu.conv2d_desc(2, 4, 64, 8, 8), [], dy, w, dx, stream=0)
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:      # halo row 4 of dy missing for the upper half of dx
        tofu.shard_conv2d_dgrad(dg, [(tofu.DGRAD_DIM_H, 2, 0)], _t([(0, 2), (0, 64), (0, 4), (0, 8)]), w, dx, stream=0)
    assert e.value.status == -2
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv2d_dgrad(tofu.dgrad_desc(2, 4, 64, 8, 8, pad=0), [], _t([(0, 2), (0, 64), (0, 6), (0, 6)]), w, dx, stream=0)
    assert e.value.status == -6


def test_lstm_cell_error_paths_are_checked_on_the_host():
    op = tofu.lstm_cell_desc(4, 8)
    g, c = _t([(0, 4), (0, 8), (0, 4)]), _t([(0, 4), (0, 8)], FAKE + (1 << 20))
    cn, hn = _t([(0, 4), (0, 8)], FAKE + (2 << 20)), _t([(0, 4), (0, 8)], FAKE + (3 << 20))
    with pytest.raises(tofu.TofuError) as e:      # the gates of only half the hidden units
        tofu.shard_lstm_cell(op, [], _t([(0, 4), (0, 4), (0, 4)]), c, cn, hn, stream=0)
    assert e.value.status == -2
    with pytest.raises(tofu.TofuError) as e:      # h_new in c_new's buffer
        tofu.shard_lstm_cell(op, [], g, c, cn, cn, stream=0)
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_lstm_cell(tofu.matmul_desc(4, 8, 2), [], g, c, cn, hn, stream=0)
    assert e.value.status == -1
    # aliasing is judged by the bytes the boxes span, not by base pointers: partial overlaps are refused
    for bad in [(g, c, cn, _t([(0, 4), (0, 8)], FAKE + (2 << 20) + 16)),        # h_new starts inside c_new
                (g, c, cn, _t([(0, 4), (0, 8)], FAKE + (1 << 20) + 64)),        # h_new starts inside c_prev
                (g, c, cn, _t([(0, 4), (0, 8)], FAKE + 256)),                   # h_new inside gates
                (g, c, _t([(0, 4), (0, 8)], FAKE + 128), hn),                   # c_new inside gates
                (g, c, _t([(0, 4), (0, 8)], FAKE + (1 << 20) + 4), hn),         # c_new shifted by one element against c_prev
                (g, c, _t([(0, 4), (0, 8)], FAKE + (1 << 20), stride=[16, 1]), hn)]:   # same address as c_prev, other strides
        with pytest.raises(tofu.TofuError) as e:
            tofu.shard_lstm_cell(op, [], *bad, stream=0)
        assert e.value.status == -1 and "overlap" in str(e.value)
    # an invalid plan makes workspace_bytes raise instead of returning a 0 that looks like "none needed"
    with pytest.raises(tofu.TofuError):
        tofu.workspace_bytes(op, [(tofu.LSTM_DIM_H, 16, 1)])
    assert tofu.workspace_bytes(op, [(tofu.LSTM_DIM_H, 2, 1)]) == 0
    r = tofu.op_regions(op, [(tofu.LSTM_DIM_H, 2, 1)])
    assert r["in_boxes"] == [[(0, 4), (4, 8), (0, 4)], [(0, 4), (4, 8)]] and not r["is_partial"]


def test_fused_conv_error_paths_are_checked_on_the_host():
    cv = tofu.conv2d_desc(2, 4, 64, 8, 8)
    w, y = _t([(0, 64), (0, 4), (0, 3), (0, 3)], FAKE + (1 << 20)), _t([(0, 2), (0, 64), (0, 8), (0, 8)], FAKE + (2 << 20))
    top = _t([(0, 2), (0, 4), (0, 4), (0, 8)], FAKE + (3 << 20))
    bottom = _t([(0, 2), (0, 4), (4, 8), (0, 8)], FAKE + (4 << 20))
    cases = [([top], -3),                                                       # rows 4..7 held by nobody
             ([top, bottom, top], -4),                                          # rows 0..3 held twice
             ([_t([(0, 2), (0, 2), (0, 8), (0, 8)], FAKE + (5 << 20)), _t([(0, 2), (2, 4), (0, 8), (0, 8)], FAKE + (6 << 20))], -6),  # cut along channels
             ([], -1),
             ([top] * 17, -1)]
    for srcs, status in cases:
        with pytest.raises(tofu.TofuError) as e:
            tofu.shard_conv2d_fused(cv, [], srcs, w, y, stream=0)
        assert e.value.status == status, (len(srcs), tofu.last_error())
    with pytest.raises(tofu.TofuError) as e:      # the H/2 shard needs halo row 4, which the top block lacks
        tofu.shard_conv2d_fused(cv, [(tofu.CONV_DIM_H, 2, 0)], [top], w, y, stream=0)
    assert e.value.status == -3


def test_reduce_error_paths_are_checked_on_the_host():
    import ctypes as C
    lib = tofu.load()
    ptrs = (C.c_void_p * 17)(*[FAKE + i * 4096 for i in range(17)])
    assert lib.tofu_partition_reduce(C.c_void_p(FAKE + (1 << 20)), ptrs, 0, 16, None) == -1
    assert lib.tofu_partition_reduce(C.c_void_p(FAKE + (1 << 20)), ptrs, 17, 16, None) == -1
    assert lib.tofu_partition_reduce(C.c_void_p(FAKE + (1 << 20)), ptrs, 2, -1, None) == -1
    assert lib.tofu_partition_reduce(C.c_void_p(FAKE + 4096 + 8), ptrs, 2, 16, None) == -1     # overlaps partials[1]
    assert lib.tofu_partition_reduce(None, ptrs, 2, 16, None) == -1
    assert lib.tofu_partition_reduce(None, ptrs, 2, 0, None) == 0                              # empty is a no-op
    assert "k = 17" in tofu.last_error() or tofu.last_error()
    ex = lib.tofu_partition_reduce_ex
    assert ex(C.c_void_p(FAKE + (1 << 20)), ptrs, 2, 16, 4, 0, None) == -1      # unknown reducer
    assert ex(C.c_void_p(FAKE + (1 << 20)), ptrs, 2, 16, 0, 2, None) == -1      # unknown order
    assert ex(C.c_void_p(FAKE + (1 << 20)), ptrs, 17, 16, 1, 0, None) == -1
    assert ex(C.c_void_p(FAKE + 4096 + 8), ptrs, 2, 16, 3, 1, None) == -1       # overlaps partials[1]
    assert ex(None, ptrs, 2, 0, 1, 1, None) == 0
    sc = lib.tofu_partition_reduce_scatter
    sc.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
    dst = C.c_void_p(FAKE + (1 << 20))
    assert sc(dst, ptrs, 2, 16, 0, 0, 0, 0, None) == -1       # no shares
    assert sc(dst, ptrs, 2, 16, 4, 4, 0, 0, None) == -1       # share outside [0, shares)
    assert sc(dst, ptrs, 2, 16, 4, -1, 0, 0, None) == -1
    assert sc(dst, ptrs, 2, 16, 4, 0, 9, 0, None) == -1       # unknown reducer
    assert sc(dst, ptrs, 17, 16, 4, 0, 0, 0, None) == -1
    assert sc(C.c_void_p(FAKE + 4096 + 8), ptrs, 2, 16, 4, 0, 0, 0, None) == -1   # overlap is judged on the full arrays
    assert sc(dst, ptrs, 2, 3, 8, 0, 0, 0, None) == 0         # floor(0*3/8) = floor(1*3/8): an empty share launches nothing
    assert sc(dst, ptrs, 2, 0, 8, 3, 0, 0, None) == 0


def test_accumulate_calls_check_their_arguments_like_the_plain_calls():
    mm = tofu.matmul_desc(64, 96, 128)
    A, B, Cc = _t([(0, 64), (0, 128)]), _t([(0, 128), (0, 96)], FAKE + (1 << 20)), _t([(0, 64), (0, 96)], FAKE + (2 << 20))
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_matmul_accumulate(mm, [(tofu.MM_DIM_K, 2, 1)], A, _t([(0, 64), (0, 96)], FAKE + (1 << 20)), Cc, stream=0)
    assert e.value.status == -2
    for call in (tofu.shard_conv2d_accumulate, tofu.shard_conv2d_wgrad_accumulate, tofu.shard_conv2d_dgrad_accumulate):
        with pytest.raises(tofu.TofuError) as e:  # wrong operator kind for the entry point
            call(mm, [], A, B, Cc, stream=0)
        assert e.value.status == -1
    big = tofu.matmul_desc(128, 4096, 16384)
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_matmul_accumulate(big, [], _t([(0, 128), (0, 16384)]), _t([(0, 16384), (0, 4096)], FAKE + (1 << 30)),
                                     _t([(0, 128), (0, 4096)], FAKE + (2 << 30)), stream=0)
    assert e.value.status == -5
    wg = tofu.wgrad_desc(16, 64, 64, 8, 8)
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv2d_wgrad_accumulate(wg, [], _t([(0, 16), (0, 64), (0, 8), (0, 8)]), _t([(0, 16), (0, 64), (0, 8), (0, 8)], FAKE + (1 << 20)),
                                           _t([(0, 64), (0, 64), (0, 3), (0, 3)], FAKE + (2 << 20)), stream=0)
    assert e.value.status == -5


def test_probe_error_paths_are_checked_on_the_host():
    lib = tofu.load()
    vp = ctypes.c_void_p
    assert lib.tofu_probe_mfma(vp(0), 1, 1, None) == -1
    assert lib.tofu_probe_mfma(vp(FAKE), 0, 1, None) == -1
    assert lib.tofu_probe_mfma(vp(FAKE), 1, 0, None) == -1
    assert lib.tofu_probe_copy(vp(0), vp(FAKE), 16, None) == -1
    assert lib.tofu_probe_copy(vp(FAKE), vp(FAKE + 4096), 24, None) == -1      # not a multiple of 16
    assert lib.tofu_probe_copy(vp(FAKE + 4), vp(FAKE + 4096), 16, None) == -1  # misaligned
    assert lib.tofu_probe_copy(vp(FAKE), vp(FAKE + 4096), 0, None) == 0        # nothing to do, nothing launched
    assert "copy probe" in tofu.last_error() or tofu.last_error() is not None
    assert lib.tofu_probe_read(vp(0), 16, vp(FAKE), None) == -1
    assert lib.tofu_probe_read(vp(FAKE), 24, vp(FAKE), None) == -1
    assert lib.tofu_probe_read(vp(FAKE), 0, vp(FAKE), None) == 0
    srcs = (vp * 8)(*[FAKE + 4096 * (j + 1) for j in range(8)])
    assert lib.tofu_probe_stream(vp(FAKE), srcs, 3, 16, None) == -1             # k must be 1, 2, 4 or 8
    assert lib.tofu_probe_stream(vp(FAKE), srcs, 8, 20, None) == -1
    assert lib.tofu_probe_stream(vp(0), srcs, 8, 16, None) == -1
    assert lib.tofu_probe_stream(vp(FAKE), srcs, 8, 0, None) == 0


def test_size_limits_are_reported_not_overflowed():
    """Extents beyond what the kernels' 32-bit indices cover return UNSUPPORTED before any launch."""
    big = 1 << 30
    mm = tofu.matmul_desc(big, 64, 64)
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_matmul(mm, [], _t([(0, big), (0, 64)]), _t([(0, 64), (0, 64)], FAKE + (1 << 40)), _t([(0, big), (0, 64)], FAKE + (2 << 40)), stream=0)
    assert e.value.status == -6
    cv = tofu.conv2d_desc(1 << 22, 4, 4, 16, 16)              # 2^30 output positions
    x = _t([(0, 1 << 22), (0, 4), (0, 16), (0, 16)])
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv2d(cv, [], x, _t([(0, 4), (0, 4), (0, 3), (0, 3)], FAKE + (1 << 40)), _t([(0, 1 << 22), (0, 4), (0, 16), (0, 16)], FAKE + (2 << 40)), stream=0)
    assert e.value.status == -6
    with pytest.raises(tofu.TofuError) as e:                   # one row of 2^33 floats: more vectors than a launch addresses
        tofu.region_fetch(_t([(0, 1 << 33)]), [_t([(0, 1 << 33)], FAKE + (1 << 42))], stream=0)
    assert e.value.status == -6
    # the integer helpers themselves work at any size
    assert tofu.op_regions(mm, [(tofu.MM_DIM_M, 8, 7)])["out_box"][0] == (7 * big // 8, big)


def test_conv1d_error_paths_and_workspace():
    op = tofu.conv1d_desc(4, 64, 64, 130)
    data, filt, out = _t([(0, 4), (0, 64), (0, 130)]), _t([(0, 64), (0, 64), (0, 3)], FAKE + (1 << 20)), _t([(0, 4), (0, 64), (0, 128)], FAKE + (2 << 20))
    ws = tofu.workspace_bytes(op, [])
    assert ws >= 64 * 64 * 3 * 4                    # room for the re-ordered filters
    with pytest.raises(tofu.TofuError) as e:        # dense [ci][co][dx] filters need that room
        tofu.shard_conv1d(op, [], data, filt, out, stream=0)
    assert e.value.status == -5
    with pytest.raises(tofu.TofuError) as e:        # an X shard needs its range widened by the window
        tofu.shard_conv1d(op, [(tofu.CONV1D_DIM_X, 2, 0)], _t([(0, 4), (0, 64), (0, 64)]), filt, out, stream=0)
    assert e.value.status == -2 and "data does not hold" in str(e.value)
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv1d(tofu.conv1d_desc(4, 64, 64, 130, window=5), [], data, _t([(0, 64), (0, 64), (0, 5)], FAKE + (1 << 20)),
                          _t([(0, 4), (0, 64), (0, 126)], FAKE + (2 << 20)), stream=0)
    assert e.value.status == -6                     # only a window of 3 has a kernel
    with pytest.raises(tofu.TofuError) as e:
        tofu.shard_conv1d(tofu.matmul_desc(4, 4, 4), [], data, filt, out, stream=0)
    assert e.value.status == -1
    with pytest.raises(tofu.TofuError) as e:        # W < KW
        tofu.op_regions(tofu.conv1d_desc(1, 1, 1, 2), [])
    assert e.value.status == -1
    # TDL description of the built-in operator gives the same regions
    from paper_1807_08887_amd import tdl as T
    d = T.from_op(op)
    for sp in ([(tofu.CONV1D_DIM_X, 4, 1)], [(tofu.CONV1D_DIM_CI, 2, 1)], [(tofu.CONV1D_DIM_CO, 8, 5), (tofu.CONV1D_DIM_B, 2, 1)]):
        var = {0: 0, 1: 1, 2: 2, 3: 3}
        a, b = tofu.op_regions(op, sp), T.regions(d, [(var[v], k, s) for v, k, s in sp])
        assert a["out_box"] == b["out_box"] and a["in_boxes"] == b["in_boxes"] and a["is_partial"] == b["is_partial"]
