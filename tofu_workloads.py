"""The timed workloads: one worker's share of each partitioned operator, at full size.

Builds, from the seeded generator, the device buffers of the four large workloads and the
"legs" of one step of the hot path (each leg is one call through the C ABI):

  gemm_nsplit   LSTM gate GEMM, shard 3 of an 8-way split of N:  X[128,16384] . W[:,12288:16384]
  gemm_ksplit   same GEMM, shard 3 of an 8-way split of K -> partial [128,32768]
  reduce_gates  that partial + 7 remote partials -> gates                       (partition-n-reduce)
  conv_cout     3x3 conv 2560->2560 @14x14, batch 128: shard 3 of an 8-way C_out split
  fetch_halo    input region of the <C_out/8, H/2> shard: own 7 rows + 1 halo row  (region fetch)
  conv_cout_h   the <C_out/8, H/2> shard computed from the fetched region
  conv_cout_h_fused  (extra, built only when named) the same shard reading its own block and the neighbour's whole block directly
  lstm_cell_nsplit   (extra) element-wise LSTM cell update on the N-split worker's 1024 hidden units (28 bytes per element)
  dgrad_cout         (extra) backward of conv_cout: partial dx from the worker's C_out/8 block of dy and of the filters
  gemm_dx_nsplit     (extra) backward of the N-split gate GEMM: partial dX = dY_s . W_s^T, W_s read transposed in place
  gemm_dw_nsplit     (extra) backward of the N-split gate GEMM: dW_s = X^T . dY_s, X read transposed in place
  gemm_ksplit_accumulate, wgrad_batch_accumulate  (extra) the two Case-2 shards adding into a resident full-size buffer
                     instead of writing a partial (out = out + shard; the buffer starts at zero)
  conv1d_cout        (extra) the paper's conv1d (Fig. 1) with 2048 channels, 512 outputs per row, batch 64: shard 3 of an 8-way C_out split
  wgrad_batch   3x3 conv weight gradient 1280->1280 @28x28: shard 3 of an 8-way batch split -> partial dW
  reduce_dw     that partial + 7 remote partials -> dW                           (partition-n-reduce)

This module holds no arithmetic of the method (ranges and regions come from the library) and
does not import the oracle; tests and the bench's baseline leg bring the oracle themselves and
use the host copies kept in `Leg.host` to evaluate expected values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List

import numpy as np
import torch

import paper_1807_08887_amd as tofu
import tofu_synth as synth


@dataclass
class Leg:
    name: str
    bound: str                 # "mfma" or "hbm"
    work: float                # algorithmic FLOP (mfma) or bytes (hbm) per launch
    run: Callable[[], None]
    out: torch.Tensor          # device tensor the leg writes (full buffer)
    host: Dict[str, object] = field(default_factory=dict)   # host arrays / parameters for checking
    conventional_flop: float = 0.0                            # dense 9-tap count, for reference
    cold: List[Callable[[], None]] = field(default_factory=list)   # the same call on rotating copies of the operands (streaming legs)


def _conv_valid_taps(h_lo, h_hi, w_lo, w_hi, H, W, pad=1):
    """Number of (position, tap) pairs of a 3x3 stride-1 conv that read inside the input."""
    rows = sum(sum(1 for kh in range(3) if 0 <= h + kh - pad < H) for h in range(h_lo, h_hi))
    cols = sum(sum(1 for kw in range(3) if 0 <= w + kw - pad < W) for w in range(w_lo, w_hi))
    return rows * cols


def _call(fn, *args):
    """Bind the arguments now (the builder reuses local names for several legs)."""
    return lambda: fn(*args)


def _ws(op, splits, dev):
    n = tofu.workspace_bytes(op, splits)
    return torch.empty(n // 4, dtype=torch.float32, device=dev) if n else None


STEP_LEGS = ("gemm_nsplit", "gemm_ksplit", "reduce_gates", "conv_cout", "fetch_halo", "conv_cout_h", "wgrad_batch", "reduce_dw")
# variants and backward operators outside the step, built only when named
EXTRA_LEGS = ("conv_cout_h_fused", "gemm_dx_nsplit", "gemm_dw_nsplit", "dgrad_cout", "lstm_cell_nsplit", "gemm_ksplit_accumulate",
              "wgrad_batch_accumulate", "conv1d_cout")


def _rotations(make_call, operands, copies):
    """The leg's call on `copies` fresh copies of its operand tensors: launched in turn, every launch finds its
    operands evicted from the 256 MB last-level cache by the launches before it."""
    runs, keep = [], []
    for _ in range(copies):
        clone = [[t.clone() for t in o] if isinstance(o, (list, tuple)) else o.clone() for o in operands]
        keep.append(clone)
        runs.append(make_call(*clone))
    return runs, keep


def build(dev: str = "cuda:0", which=None, keep_host: bool = True, cold_copies: bool = False) -> List[Leg]:
    which = set(which) if which else None
    want = lambda *names: which is None or any(n in which for n in names)
    legs: List[Leg] = []
    up = lambda a: torch.from_numpy(a).to(dev)

    # ------------------------------------------------------------------ LSTM gate GEMM
    extra = lambda name: which is not None and name in which
    if want("gemm_nsplit", "gemm_ksplit", "reduce_gates") or extra("gemm_ksplit_accumulate"):
        M, N, K, k = 128, 32768, 16384, 8
        op = tofu.matmul_desc(M, N, K)
    if want("gemm_nsplit"):
        cfg = synth.CONFIGS["lstm_gates_nsplit"]
        s = cfg["shard"]
        splits = [(tofu.MM_DIM_N, k, s)]
        reg = tofu.op_regions(op, splits)
        (n0, n1) = reg["out_box"][1]
        X = synth.draw(cfg["a"], cfg["seed"], 0, (M, K))
        Ws = synth.draw(cfg["b"], cfg["seed"], 1, (K, n1 - n0))          # the worker's own dense block of W
        dX, dW, C = up(X), up(Ws), torch.zeros(M, N, dtype=torch.float32, device=dev)
        ws = _ws(op, splits, dev)
        tA, tB, tC = tofu.tensor(dX), tofu.tensor(dW, [0, n0]), tofu.tensor(C)
        legs.append(Leg("gemm_nsplit", "mfma", 2.0 * M * (n1 - n0) * K,
                        _call(tofu.shard_matmul, op, splits, tA, tB, tC, ws), C,
                        dict(kind="matmul", A=X, B=Ws, box=reg["out_box"], krange=(0, K), b_col0=n0, keep=(dX, dW, ws)) if keep_host else dict(keep=(dX, dW, ws))))
    if which is not None and ("gemm_dx_nsplit" in which or "gemm_dw_nsplit" in which):
        # Backward GEMMs of the N-split worker (forward and backward operators form one group and
        # keep the weights' partition): the worker holds X, its block W_s and its block dY_s.
        M, N, K, k = 128, 32768, 16384, 8
        cfg = synth.CONFIGS["lstm_gates_nsplit"]
        s = cfg["shard"]
        n0, n1 = tofu.shard_range(N, k, s)
        X = synth.draw(cfg["a"], cfg["seed"], 0, (M, K))
        Ws = synth.draw(cfg["b"], cfg["seed"], 1, (K, n1 - n0))
        dYs = synth.normal(cfg["seed"], 2, (M, n1 - n0), 1.0)
        dX, dW, ddY = up(X), up(Ws), up(dYs)
        if "gemm_dx_nsplit" in which:      # dX[M,K] = dY[M,N] . W^T[N,K]; the N split is a reduction split here
            opx = tofu.matmul_desc(M, K, N)
            spx = [(tofu.MM_DIM_K, k, s)]
            part = torch.zeros(M, K, dtype=torch.float32, device=dev)
            wsx = _ws(opx, spx, dev)
            legs.append(Leg("gemm_dx_nsplit", "mfma", 2.0 * M * K * (n1 - n0),
                            _call(tofu.shard_matmul, opx, spx, tofu.tensor(ddY, [0, n0]), tofu.tensor(dW.t(), [n0, 0]), tofu.tensor(part), wsx), part,
                            dict(kind="matmul", A=dYs, B=np.ascontiguousarray(Ws.T), box=[(0, M), (0, K)], krange=(0, n1 - n0), b_col0=0,
                                 keep=(ddY, dW, wsx)) if keep_host else dict(keep=(ddY, dW, wsx))))
        if "gemm_dw_nsplit" in which:      # dW[K,N] = X^T[K,M] . dY[M,N]; the N split stays an output split
            opw = tofu.matmul_desc(K, N, M)
            spw = [(tofu.MM_DIM_N, k, s)]
            gW = torch.zeros(K, n1 - n0, dtype=torch.float32, device=dev)
            wsw_ = _ws(opw, spw, dev)
            legs.append(Leg("gemm_dw_nsplit", "mfma", 2.0 * K * (n1 - n0) * M,
                            _call(tofu.shard_matmul, opw, spw, tofu.tensor(dX.t()), tofu.tensor(ddY, [0, n0]), tofu.tensor(gW, [0, n0]), wsw_), gW,
                            dict(kind="matmul", A=np.ascontiguousarray(X.T), B=dYs, box=[(0, K), (0, n1 - n0)], krange=(0, M), b_col0=0,
                                 keep=(dX, ddY, wsw_)) if keep_host else dict(keep=(dX, ddY, wsw_))))
    if which is not None and "lstm_cell_nsplit" in which:
        # the element-wise stage shares the gate GEMM's N partition: 8192 hidden units, 8 workers
        cfg = synth.CONFIGS["lstm_gates_nsplit"]
        Bt, Hd, k, s = 128, 8192, cfg["k"], cfg["shard"]
        opl = tofu.lstm_cell_desc(Bt, Hd)
        spl = [(tofu.LSTM_DIM_H, k, s)]
        h0, h1 = tofu.shard_range(Hd, k, s)
        g_s = synth.normal(cfg["seed"], 3, (Bt, h1 - h0, 4), 2.0)
        c_s = synth.normal(cfg["seed"], 4, (Bt, h1 - h0), 1.0)
        d_g, d_c = up(g_s), up(c_s)
        c_new = torch.zeros(Bt, h1 - h0, dtype=torch.float32, device=dev)
        h_new = torch.zeros(Bt, h1 - h0, dtype=torch.float32, device=dev)
        legs.append(Leg("lstm_cell_nsplit", "hbm", 28.0 * Bt * (h1 - h0),
                        _call(tofu.shard_lstm_cell, opl, spl, tofu.tensor(d_g, [0, h0, 0]), tofu.tensor(d_c, [0, h0]),
                              tofu.tensor(c_new, [0, h0]), tofu.tensor(h_new, [0, h0])), c_new,
                        dict(kind="lstm", gates=g_s, c=c_s, h_out=h_new, keep=(d_g, d_c, h_new)) if keep_host else dict(keep=(d_g, d_c, h_new))))
    if want("gemm_ksplit", "reduce_gates") or extra("gemm_ksplit_accumulate"):
        cfg = synth.CONFIGS["lstm_gates_ksplit"]
        s = cfg["shard"]
        splits = [(tofu.MM_DIM_K, k, s)]
        reg = tofu.op_regions(op, splits)
        (k0, k1) = reg["in_boxes"][0][1]
        X = synth.draw(cfg["a"], cfg["seed"], 0, (M, K))
        Wr = synth.draw(cfg["b"], cfg["seed"], 1, (k1 - k0, N))           # the worker's own rows of W
        dX, dW = up(X), up(Wr)
        part = torch.zeros(M, N, dtype=torch.float32, device=dev)
        ws = _ws(op, splits, dev)
        tA, tB, tC = tofu.tensor(dX), tofu.tensor(dW, [k0, 0]), tofu.tensor(part)   # X is read strided, in place
        host_k = dict(kind="matmul", A=X, B=Wr, box=reg["out_box"], krange=(k0, k1), b_row0=k0, keep=(dX, dW, ws)) if keep_host else dict(keep=(dX, dW, ws))
        if want("gemm_ksplit", "reduce_gates"):
            legs.append(Leg("gemm_ksplit", "mfma", 2.0 * M * N * (k1 - k0), _call(tofu.shard_matmul, op, splits, tA, tB, tC, ws), part, host_k))
        if extra("gemm_ksplit_accumulate"):
            total = torch.zeros(M, N, dtype=torch.float32, device=dev)
            legs.append(Leg("gemm_ksplit_accumulate", "mfma", 2.0 * M * N * (k1 - k0),
                            _call(tofu.shard_matmul_accumulate, op, splits, tA, tB, tofu.tensor(total), ws), total, host_k))
        if want("reduce_gates"):
            remote = [synth.normal(cfg["seed"], 10 + j, (M, N), cfg["partial_std"]) for j in range(k - 1)]
            d_remote = [up(r) for r in remote]
            gates = torch.zeros(M, N, dtype=torch.float32, device=dev)
            order = d_remote[:s] + [part] + d_remote[s:]                  # worker s's partial sits at position s
            legs.append(Leg("reduce_gates", "hbm", 4.0 * M * N * (k + 1),
                            _call(tofu.partition_reduce, gates, order), gates,
                            dict(kind="reduce", remote=remote, own_index=s, own=part, keep=order) if keep_host else dict(keep=order)))
            if cold_copies:      # 4 x 151 MB
                legs[-1].cold, legs[-1].host["cold_keep"] = _rotations(lambda o, p: _call(tofu.partition_reduce, o, p), [gates, order], 4)

    # ------------------------------------------------------------------ Wide-ResNet conv forward
    if want("conv_cout", "fetch_halo", "conv_cout_h") or extra("conv_cout_h_fused"):
        cfg = synth.CONFIGS["wresnet_conv_fwd"]
        NB, C, H, W, k, s = cfg["batch"], cfg["c_in"], cfg["H"], cfg["W"], cfg["k"], cfg["shard"]
        op = tofu.conv2d_desc(NB, C, C, H, W)
        x = synth.draw(cfg["x"], cfg["seed"], 0, (NB, C, H, W))
        sp_co = [(tofu.CONV_DIM_CO, k, s)]
        reg = tofu.op_regions(op, sp_co)
        (co0, co1) = reg["out_box"][1]
        w_s = synth.draw(cfg["w"], cfg["seed"], 1, (co1 - co0, C, 3, 3))  # the worker's own filters
        dx, dw = up(x), up(w_s)
        tw = tofu.tensor(dw, [co0, 0, 0, 0])
        host_common = dict(kind="conv2d", x=x, w=w_s, co0=co0) if keep_host else {}
    if want("conv_cout"):
        y = torch.zeros(NB, co1 - co0, H, W, dtype=torch.float32, device=dev)
        tx, ty = tofu.tensor(dx), tofu.tensor(y, [0, co0, 0, 0])
        taps = _conv_valid_taps(0, H, 0, W, H, W)
        legs.append(Leg("conv_cout", "mfma", 2.0 * NB * (co1 - co0) * C * taps,
                        _call(tofu.shard_conv2d, op, sp_co, tx, tw, ty, _ws(op, sp_co, dev)), y,
                        dict(host_common, box=reg["out_box"], keep=(dx, dw)), conventional_flop=2.0 * NB * (co1 - co0) * C * 9 * H * W))
    if want("fetch_halo", "conv_cout_h") or extra("conv_cout_h_fused"):
        sp = sp_co + [(tofu.CONV_DIM_H, cfg["k_h"], cfg["shard_h"])]
        reg2 = tofu.op_regions(op, sp)
        box = reg2["in_boxes"][0]                                       # rows [0,8) of the input
        _, h_cut = tofu.shard_range(H, cfg["k_h"], cfg["shard_h"])           # rows [0, h_cut) are this worker's own block
        own = dx[:, :, :h_cut].contiguous()                               # rows this worker owns
        halo = dx[:, :, h_cut:h_cut + 1].contiguous()                     # the halo row as a dense block of its own (a received row)
        region = torch.zeros([hi - lo for lo, hi in box], dtype=torch.float32, device=dev)
        t_region = tofu.tensor(region, [lo for lo, _ in box])
        srcs = [tofu.tensor(own, [0, 0, 0, 0]), tofu.tensor(halo, [0, 0, h_cut, 0])]
        nbytes = 2.0 * 4.0 * region.numel()
        if want("fetch_halo"):
            legs.append(Leg("fetch_halo", "hbm", nbytes, _call(tofu.region_fetch, t_region, srcs), region,
                            dict(kind="fetch", x=x if keep_host else None, box=box, keep=(own, halo))))
            if cold_copies:      # 3 x 294 MB
                lo_box = [lo for lo, _ in box]
                legs[-1].cold, legs[-1].host["cold_keep"] = _rotations(
                    lambda r, o, h: _call(tofu.region_fetch, tofu.tensor(r, lo_box), [tofu.tensor(o, [0, 0, 0, 0]), tofu.tensor(h, [0, 0, h_cut, 0])]),
                    [region, own, halo], 3)
        if want("conv_cout_h"):
            (h0, h1) = reg2["out_box"][2]
            y2 = torch.zeros(NB, co1 - co0, h1 - h0, W, dtype=torch.float32, device=dev)
            ty2 = tofu.tensor(y2, [0, co0, h0, 0])
            taps = _conv_valid_taps(h0, h1, 0, W, H, W)
            if not want("fetch_halo"):
                tofu.region_fetch(t_region, srcs)
            legs.append(Leg("conv_cout_h", "mfma", 2.0 * NB * (co1 - co0) * C * taps,
                            _call(tofu.shard_conv2d, op, sp, t_region, tw, ty2, _ws(op, sp, dev)), y2,
                            dict(host_common, box=reg2["out_box"], keep=(region, dw, own, halo)),
                            conventional_flop=2.0 * NB * (co1 - co0) * C * 9 * (h1 - h0) * W))
        if extra("conv_cout_h_fused"):
            # the fused form needs no copy of the halo row at all: it reads it out of the neighbour's whole block, rows [h_cut, H)
            other = dx[:, :, h_cut:].contiguous()
            srcs = [tofu.tensor(own, [0, 0, 0, 0]), tofu.tensor(other, [0, 0, h_cut, 0])]
            (h0, h1) = reg2["out_box"][2]
            y3 = torch.zeros(NB, co1 - co0, h1 - h0, W, dtype=torch.float32, device=dev)
            taps = _conv_valid_taps(h0, h1, 0, W, H, W)
            legs.append(Leg("conv_cout_h_fused", "mfma", 2.0 * NB * (co1 - co0) * C * taps,
                            _call(tofu.shard_conv2d_fused, op, sp, srcs, tw, tofu.tensor(y3, [0, co0, h0, 0]), _ws(op, sp, dev)), y3,
                            dict(host_common, box=reg2["out_box"], keep=(dw, own, other)),
                            conventional_flop=2.0 * NB * (co1 - co0) * C * 9 * (h1 - h0) * W))

    if extra("dgrad_cout"):
        # Data gradient under the forward C_out split: the worker holds dy[:, co0:co1] and its own
        # filters; C_out is a reduction index of this operator, so dx is a full-size partial.
        cfg = synth.CONFIGS["wresnet_conv_fwd"]
        NB, C, H, W, k, s = cfg["batch"], cfg["c_in"], cfg["H"], cfg["W"], cfg["k"], cfg["shard"]
        opd = tofu.dgrad_desc(NB, C, C, H, W)
        spd = [(tofu.DGRAD_DIM_CO, k, s)]
        regd = tofu.op_regions(opd, spd)
        (co0, co1) = regd["in_boxes"][0][1]
        w_s = synth.draw(cfg["w"], cfg["seed"], 1, (co1 - co0, C, 3, 3))
        dy_s = synth.normal(cfg["seed"], 2, (NB, co1 - co0, H, W), 1.0)
        d_dy, d_w = up(dy_s), up(w_s)
        part_dx = torch.zeros(NB, C, H, W, dtype=torch.float32, device=dev)
        wsd = _ws(opd, spd, dev)
        taps = _conv_valid_taps(0, H, 0, W, H, W)
        legs.append(Leg("dgrad_cout", "mfma", 2.0 * NB * C * (co1 - co0) * taps,
                        _call(tofu.shard_conv2d_dgrad, opd, spd, tofu.tensor(d_dy, [0, co0, 0, 0]), tofu.tensor(d_w, [co0, 0, 0, 0]),
                              tofu.tensor(part_dx), wsd), part_dx,
                        dict(kind="dgrad", dy=dy_s, w=w_s, H=H, W=W, keep=(d_dy, d_w, wsd)) if keep_host else dict(keep=(d_dy, d_w, wsd)),
                        conventional_flop=2.0 * NB * C * (co1 - co0) * 9 * H * W))

    if extra("conv1d_cout"):
        cfg = synth.CONFIGS["conv1d_large"]
        NB, C, L, k, s = cfg["batch"], cfg["c_in"], cfg["W"], cfg["k"], cfg["shard"]
        op1 = tofu.conv1d_desc(NB, C, C, L)
        sp1 = [(tofu.CONV1D_DIM_CO, k, s)]
        reg1 = tofu.op_regions(op1, sp1)
        (co0, co1) = reg1["out_box"][1]
        data = synth.draw(cfg["x"], cfg["seed"], 0, (NB, C, L))
        f_s = synth.draw(cfg["w"], cfg["seed"], 1, (C, co1 - co0, 3))     # the worker's own filters, [ci][co][dx] as in Fig. 1
        d_data, d_f = up(data), up(f_s)
        out1 = torch.zeros(NB, co1 - co0, L - 2, dtype=torch.float32, device=dev)
        ws1 = _ws(op1, sp1, dev)
        legs.append(Leg("conv1d_cout", "mfma", 2.0 * NB * (co1 - co0) * (L - 2) * C * 3,
                        _call(tofu.shard_conv1d, op1, sp1, tofu.tensor(d_data), tofu.tensor(d_f, [0, co0, 0]), tofu.tensor(out1, [0, co0, 0]), ws1), out1,
                        dict(kind="conv1d", data=data, filters=f_s, keep=(d_data, d_f, ws1)) if keep_host else dict(keep=(d_data, d_f, ws1))))

    # ------------------------------------------------------------------ Wide-ResNet conv weight gradient
    if want("wgrad_batch", "reduce_dw") or extra("wgrad_batch_accumulate"):
        cfg = synth.CONFIGS["wresnet_conv_wgrad"]
        NB, C, H, W, k, s = cfg["batch"], cfg["c_in"], cfg["H"], cfg["W"], cfg["k"], cfg["shard"]
        opw = tofu.wgrad_desc(NB, C, C, H, W)
        splits_w = [(tofu.WGRAD_DIM_N, k, s)]
        regw = tofu.op_regions(opw, splits_w)
        (n0, n1) = regw["in_boxes"][0][0]
        xs_ = synth.draw(cfg["x"], cfg["seed"], 0, (n1 - n0, C, H, W))   # the worker's own images
        dys = synth.draw(cfg["dy"], cfg["seed"], 1, (n1 - n0, C, H, W))
        dxs, ddys = up(xs_), up(dys)
        part_w = torch.zeros(C, C, 3, 3, dtype=torch.float32, device=dev)
        wsw = _ws(opw, splits_w, dev)
        txw, tdy, tdw = tofu.tensor(dxs, [n0, 0, 0, 0]), tofu.tensor(ddys, [n0, 0, 0, 0]), tofu.tensor(part_w)
        taps = _conv_valid_taps(0, H, 0, W, H, W)
        host_w = dict(kind="wgrad", x=xs_, dy=dys, n0=n0, keep=(dxs, ddys, wsw)) if keep_host else dict(keep=(dxs, ddys, wsw))
        if want("wgrad_batch", "reduce_dw"):
            legs.append(Leg("wgrad_batch", "mfma", 2.0 * (n1 - n0) * C * C * taps,
                            _call(tofu.shard_conv2d_wgrad, opw, splits_w, txw, tdy, tdw, wsw), part_w, host_w,
                            conventional_flop=2.0 * (n1 - n0) * C * C * 9 * H * W))
        if extra("wgrad_batch_accumulate"):
            total_w = torch.zeros(C, C, 3, 3, dtype=torch.float32, device=dev)
            legs.append(Leg("wgrad_batch_accumulate", "mfma", 2.0 * (n1 - n0) * C * C * taps,
                            _call(tofu.shard_conv2d_wgrad_accumulate, opw, splits_w, txw, tdy, tofu.tensor(total_w), wsw), total_w, host_w,
                            conventional_flop=2.0 * (n1 - n0) * C * C * 9 * H * W))
        if want("reduce_dw"):
            remote = [synth.normal(cfg["seed"], 10 + j, (C, C, 3, 3), cfg["partial_std"]) for j in range(k - 1)]
            d_remote = [up(r) for r in remote]
            dw_full = torch.zeros(C, C, 3, 3, dtype=torch.float32, device=dev)
            order = d_remote[:s] + [part_w] + d_remote[s:]
            legs.append(Leg("reduce_dw", "hbm", 4.0 * C * C * 9 * (k + 1),
                            _call(tofu.partition_reduce, dw_full, order), dw_full,
                            dict(kind="reduce", remote=remote, own_index=s, own=part_w, keep=order) if keep_host else dict(keep=order)))
            if cold_copies:      # 2 x 531 MB
                legs[-1].cold, legs[-1].host["cold_keep"] = _rotations(lambda o, p: _call(tofu.partition_reduce, o, p), [dw_full, order], 2)
    return legs
