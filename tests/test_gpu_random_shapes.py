"""Seeded random sweep over small shapes and one- or two-step plans for every shard operator: the
shard's output box against the oracle restricted to the same box and reduction range, and
nothing written outside the box.  Shapes are drawn to cross tile edges in every dimension
(channels around 32 / 64 / 128, widths around 4 / 14 / 28 / 32, ragged batch)."""
import random

import numpy as np
import pytest
import torch

import oracle
import paper_1807_08887_amd as tofu
import tofu_synth as synth
from oracle import regions as R

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def ws(op, sp):
    n = tofu.workspace_bytes(op, sp)
    return torch.empty(max(n, 16) // 4, dtype=torch.float32, device=DEV) if n else None


def close(got, val, absum, what):
    err = np.abs(got.astype(np.float64) - val)
    assert (err <= TOL * absum).all(), f"{what}: worst ratio {np.max(err / np.maximum(absum, 1e-300)):.3e}"
    assert (got[absum == 0] == 0).all(), what


def plan(rng, ext, names):
    """One or two steps over random dimensions, k <= the current extent."""
    cur = dict(ext)
    steps = []
    for _ in range(rng.choice([1, 1, 2])):
        d = rng.choice([n for n in names if cur[n] >= 2] or [None])
        if d is None:
            break
        k = rng.randint(2, min(4, cur[d]))
        s = rng.randrange(k)
        lo, hi = R.shard_range(cur[d], k, s)
        cur[d] = hi - lo
        steps.append((d, k, s))
    return steps


def check_box(out, reg, val, absum, what):
    got = out.cpu().numpy()
    sl = R.box_slices(reg["out_box"])
    inside = np.zeros(got.shape, dtype=bool)
    inside[sl] = True
    assert np.isnan(got[~inside]).all(), what + ": wrote outside its box"
    close(got[sl], val, absum, what)


CH = [1, 3, 31, 32, 33, 63, 64, 65, 80, 96, 127, 129, 160]
SP = [1, 2, 3, 4, 7, 13, 14, 15, 16, 27, 28, 31, 32, 33]


@pytest.mark.parametrize("seed", range(12))
def test_random_conv_family(seed):
    rng = random.Random(1000 + seed)
    for case in range(6):
        batch, c_in, c_out = rng.randint(1, 5), rng.choice(CH), rng.choice(CH)
        H, W, pad = rng.choice(SP), rng.choice(SP), rng.choice([0, 1, 1])
        if H + 2 * pad < 3 or W + 2 * pad < 3:
            continue
        ho, wo = H + 2 * pad - 2, W + 2 * pad - 2
        x = synth.normal(seed * 100 + case, 0, (batch, c_in, H, W), 1.0)
        w = synth.normal(seed * 100 + case, 1, (c_out, c_in, 3, 3), 0.3)
        dy = synth.normal(seed * 100 + case, 2, (batch, c_out, ho, wo), 1.0)
        dx_, dw_, ddy = dev(x), dev(w), dev(dy)
        base = dict(batch=batch, c_in=c_in, c_out=c_out, H=H, W=W, KH=3, KW=3, stride=1, pad=pad)
        tag = f"seed {seed} case {case}: b{batch} ci{c_in} co{c_out} {H}x{W} pad{pad}"
        # forward
        opd = dict(base, kind="conv2d")
        sp = plan(rng, R.iteration_extents(opd), ["N", "CO", "H", "W", "CI"])
        reg = R.op_regions(opd, sp)
        names = {"N": tofu.CONV_DIM_N, "CO": tofu.CONV_DIM_CO, "H": tofu.CONV_DIM_H, "W": tofu.CONV_DIM_W, "CI": tofu.CONV_DIM_CI}
        op = tofu.conv2d_desc(batch, c_in, c_out, H, W, pad=pad)
        lsp = [(names[d], k, s) for d, k, s in sp]
        y = torch.full((batch, c_out, ho, wo), float("nan"), dtype=torch.float32, device=DEV)
        print(tag, "conv2d", sp, flush=True)
        tofu.shard_conv2d(op, lsp, tofu.tensor(dx_), tofu.tensor(dw_), tofu.tensor(y), ws(op, lsp))
        val, absum = oracle.conv2d_box(x, w, pad=pad, box=reg["out_box"], cirange=reg["ranges"]["CI"])
        check_box(y, reg, val, absum, tag + " conv2d " + str(sp))
        # weight gradient
        opd = dict(base, kind="conv2d_wgrad")
        sp = plan(rng, R.iteration_extents(opd), ["CO", "CI", "N"])
        reg = R.op_regions(opd, sp)
        names = {"CO": tofu.WGRAD_DIM_CO, "CI": tofu.WGRAD_DIM_CI, "N": tofu.WGRAD_DIM_N}
        op = tofu.wgrad_desc(batch, c_in, c_out, H, W, pad=pad)
        lsp = [(names[d], k, s) for d, k, s in sp]
        g = torch.full((c_out, c_in, 3, 3), float("nan"), dtype=torch.float32, device=DEV)
        print(tag, "wgrad", sp, flush=True)
        tofu.shard_conv2d_wgrad(op, lsp, tofu.tensor(dx_), tofu.tensor(ddy), tofu.tensor(g), ws(op, lsp))
        val, absum = oracle.wgrad_box(x, dy, 3, 3, pad=pad, box=reg["out_box"], nrange=reg["ranges"]["N"])
        check_box(g, reg, val, absum, tag + " wgrad " + str(sp))
        # data gradient (pad 1 only)
        if pad == 1:
            opd = dict(base, kind="conv2d_dgrad")
            sp = plan(rng, R.iteration_extents(opd), ["N", "CI", "H", "W", "CO"])
            reg = R.op_regions(opd, sp)
            names = {"N": tofu.DGRAD_DIM_N, "CI": tofu.DGRAD_DIM_CI, "H": tofu.DGRAD_DIM_H, "W": tofu.DGRAD_DIM_W, "CO": tofu.DGRAD_DIM_CO}
            op = tofu.dgrad_desc(batch, c_in, c_out, H, W, pad=pad)
            lsp = [(names[d], k, s) for d, k, s in sp]
            gx = torch.full((batch, c_in, H, W), float("nan"), dtype=torch.float32, device=DEV)
            print(tag, "dgrad", sp, flush=True)
            tofu.shard_conv2d_dgrad(op, lsp, tofu.tensor(ddy), tofu.tensor(dw_), tofu.tensor(gx), ws(op, lsp))
            val, absum = oracle.dgrad_box(dy, w, H, W, pad=pad, box=reg["out_box"], corange=reg["ranges"]["CO"])
            check_box(gx, reg, val, absum, tag + " dgrad " + str(sp))


@pytest.mark.parametrize("c_out,batch,hw", [(160, 40, 14), (80, 24, 14), (96, 3, 28), (32, 40, 14), (200, 9, 7)])
def test_conv_output_channels_with_a_short_last_tile_row(c_out, batch, hw):
    """Output channels that end in a tile row of at most 32 (160 = 2 x 64 + 32, 80 = 64 + 16, ...) take the
    32-row kernel for that row -- as whole tiles and, with many positions, as balanced segments; forward on
    the whole box and under a C_out split, and the data gradient (whose tile rows are the input channels)."""
    c_in = 24
    x = synth.normal(700 + c_out, 0, (batch, c_in, hw, hw), 1.0)
    w = synth.normal(700 + c_out, 1, (c_out, c_in, 3, 3), 0.3)
    dx_, dw_ = dev(x), dev(w)
    op = tofu.conv2d_desc(batch, c_in, c_out, hw, hw)
    opd = dict(kind="conv2d", batch=batch, c_in=c_in, c_out=c_out, H=hw, W=hw, KH=3, KW=3, stride=1, pad=1)
    for sp, lsp in [([], []), ([("CO", 2, 1)], [(tofu.CONV_DIM_CO, 2, 1)])]:
        reg = R.op_regions(opd, sp)
        y = torch.full((batch, c_out, hw, hw), float("nan"), dtype=torch.float32, device=DEV)
        tofu.shard_conv2d(op, lsp, tofu.tensor(dx_), tofu.tensor(dw_), tofu.tensor(y), ws(op, lsp))
        val, absum = oracle.conv2d_box(x, w, pad=1, box=reg["out_box"])
        check_box(y, reg, val, absum, f"conv2d co{c_out} {sp}")
    # data gradient of a convolution with c_out INPUT channels: dx has c_out channels, the kernel's tile rows
    dy = synth.normal(700 + c_out, 2, (batch, c_in, hw, hw), 1.0)
    wd = synth.normal(700 + c_out, 3, (c_in, c_out, 3, 3), 0.3)
    opg = tofu.dgrad_desc(batch, c_out, c_in, hw, hw)
    gx = torch.full((batch, c_out, hw, hw), float("nan"), dtype=torch.float32, device=DEV)
    d_dy, d_wd = dev(dy), dev(wd)          # kept alive: a descriptor holds only the address
    tofu.shard_conv2d_dgrad(opg, [], tofu.tensor(d_dy), tofu.tensor(d_wd), tofu.tensor(gx), ws(opg, []))
    val, absum = oracle.dgrad_box(dy, wd, hw, hw, pad=1)
    close(gx.cpu().numpy(), val, absum, f"dgrad ci{c_out}")


@pytest.mark.parametrize("batch,c_in,c_out,slots", [(8, 1024, 320, 14 * 35 + 1 * 22 + 2 * 22), (32, 128, 704, 275 + 1 * 237 + 2 * 237)])
def test_conv_balanced_launch_with_own_pieces_and_tails(batch, c_in, c_out, slots):
    """Mid-size shards whose tiles do not fill the workgroup slots and whose reductions are long enough for the
    balanced launch to use all of its forms, every output checked: 35 tiles x 256 channel steps (14 workgroups of
    their own per tile, one round of whole tails, the last 13 tails shared out step by step) and 275 tiles x 32
    steps (one own workgroup per tile, 237 tail workgroups).  The accumulating form must add exactly the same sum."""
    hw = 14
    x = synth.normal(900 + batch, 0, (batch, c_in, hw, hw), 1.0)
    w = synth.normal(900 + batch, 1, (c_out, c_in, 3, 3), 0.05)
    dx_, dw_ = dev(x), dev(w)
    op = tofu.conv2d_desc(batch, c_in, c_out, hw, hw)
    # own pieces + whole tails + two slots per tail workgroup for its share of the last tails, 64 x 256 floats each
    assert tofu.workspace_bytes(op, []) == slots * 64 * 256 * 4, "the shape is meant to take every form of the balanced launch"
    y = torch.full((batch, c_out, hw, hw), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_conv2d(op, [], tofu.tensor(dx_), tofu.tensor(dw_), tofu.tensor(y), ws(op, []))
    val, absum = oracle.conv2d_box(x, w, pad=1)
    close(y.cpu().numpy(), val, absum, f"conv2d b{batch} ci{c_in} co{c_out}")
    base = torch.full_like(y, 0.5)
    acc = base.clone()
    tofu.shard_conv2d_accumulate(op, [], tofu.tensor(dx_), tofu.tensor(dw_), tofu.tensor(acc), ws(op, []))
    assert torch.equal(acc, base + y), "accumulate differs from add-after"


def test_wgrad_balanced_launch_with_own_pieces_and_tails():
    """40 weight-gradient tiles x 112 row steps on 512 workgroups: 12 own workgroups per tile, 32 tail workgroups
    with one whole tail each and a share of the last eight; every output checked, and the accumulating form."""
    batch, c_in, c_out, hw = 4, 320, 512, 28
    x = synth.normal(950, 0, (batch, c_in, hw, hw), 1.0)
    dy = synth.normal(950, 1, (batch, c_out, hw, hw), 1.0)
    d_x, d_dy = dev(x), dev(dy)
    op = tofu.wgrad_desc(batch, c_in, c_out, hw, hw)
    assert tofu.workspace_bytes(op, []) == (12 * 40 + 1 * 32 + 2 * 32) * 9 * 128 * 32 * 4, "the shape is meant to take every form of the balanced launch"
    g = torch.full((c_out, c_in, 3, 3), float("nan"), dtype=torch.float32, device=DEV)
    tofu.shard_conv2d_wgrad(op, [], tofu.tensor(d_x), tofu.tensor(d_dy), tofu.tensor(g), ws(op, []))
    val, absum = oracle.wgrad_box(x, dy, 3, 3, pad=1)
    close(g.cpu().numpy(), val, absum, "wgrad 40 tiles")
    base = torch.full_like(g, -2.0)
    acc = base.clone()
    tofu.shard_conv2d_wgrad_accumulate(op, [], tofu.tensor(d_x), tofu.tensor(d_dy), tofu.tensor(acc), ws(op, []))
    assert torch.equal(acc, base + g), "accumulate differs from add-after"


@pytest.mark.parametrize("seed", range(8))
def test_random_matmul_and_conv1d(seed):
    rng = random.Random(2000 + seed)
    dims = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 257]
    for case in range(8):
        M, N, K = rng.choice(dims), rng.choice(dims), rng.choice(dims + [1030, 2100])
        A = synth.normal(seed * 100 + case, 3, (M, K), 1.0); B = synth.normal(seed * 100 + case, 4, (K, N), 1.0)
        opd = dict(kind="matmul", M=M, N=N, K=K)
        sp = plan(rng, R.iteration_extents(opd), ["M", "N", "K"])
        reg = R.op_regions(opd, sp)
        names = {"M": tofu.MM_DIM_M, "N": tofu.MM_DIM_N, "K": tofu.MM_DIM_K}
        op = tofu.matmul_desc(M, N, K)
        lsp = [(names[d], k, s) for d, k, s in sp]
        C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        tag = f"seed {seed} case {case}: matmul {M}x{N}x{K} {sp}"
        print(tag, flush=True)
        # a random choice of operand layouts: plain, or a transposed view of a transposed buffer
        dA = dev(A) if rng.random() < 0.5 else dev(np.ascontiguousarray(A.T)).t()
        dB = dev(B) if rng.random() < 0.5 else dev(np.ascontiguousarray(B.T)).t()
        tofu.shard_matmul(op, lsp, tofu.tensor(dA), tofu.tensor(dB), tofu.tensor(C), ws(op, lsp))
        val, absum = oracle.matmul_box(A, B, box=reg["out_box"], krange=reg["ranges"]["K"])
        check_box(C, reg, val, absum, tag)
    for case in range(6):
        Bt, CI, CO = rng.randint(1, 4), rng.choice(CH), rng.choice(CH)
        X = rng.choice([1, 2, 5, 14, 24, 32, 48, 64, 96, 100, 128, 192, 256])
        data = synth.normal(seed * 100 + case, 5, (Bt, CI, X + 2), 1.0); filt = synth.normal(seed * 100 + case, 6, (CI, CO, 3), 0.3)
        opd = dict(kind="conv1d", batch=Bt, c_in=CI, c_out=CO, W=X + 2, KW=3)
        sp = plan(rng, R.iteration_extents(opd), ["B", "CO", "X", "CI"])
        reg = R.op_regions(opd, sp)
        names = {"B": tofu.CONV1D_DIM_B, "CO": tofu.CONV1D_DIM_CO, "X": tofu.CONV1D_DIM_X, "CI": tofu.CONV1D_DIM_CI}
        op = tofu.conv1d_desc(Bt, CI, CO, X + 2)
        lsp = [(names[d], k, s) for d, k, s in sp]
        out = torch.full((Bt, CO, X), float("nan"), dtype=torch.float32, device=DEV)
        tag = f"seed {seed} case {case}: conv1d b{Bt} ci{CI} co{CO} x{X} {sp}"
        print(tag, flush=True)
        d_data, d_filt = dev(data), dev(filt)      # descriptors hold addresses only: keep the buffers alive
        try:
            tofu.shard_conv1d(op, lsp, tofu.tensor(d_data), tofu.tensor(d_filt), tofu.tensor(out), ws(op, lsp))
        except tofu.TofuError as e:
            assert e.status == -6, tag         # a shard length without a usable chunk size is reported, not computed wrongly
            continue
        val, absum = oracle.conv1d_box(data, filt, box=reg["out_box"], cirange=reg["ranges"]["CI"])
        check_box(out, reg, val, absum, tag)
