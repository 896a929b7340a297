"""The partition-n-reduce invariant at the full workload sizes: ALL k shards go through the GPU
kernels one after another on the one GPU, their outputs are concatenated (Case-1) or summed
with tofu_partition_reduce (Case-2), and the result is compared with the unpartitioned oracle on
the corners of the output plus >= 2^16 seeded output coordinates (arXiv 1807.08887 Sec. 3.1: the
operator's output is the concatenation or the element-wise sum of the workers' outputs).

The 2 GiB LSTM weight matrix is drawn on the device (tofu_synth.uniform_torch) and, for the oracle,
only at the sampled columns (tofu_synth.uniform_at): the generator is counter-based, so both see
the same bits.  The weight gradient runs at the workload's channels and image size with batch 32
(4 images per shard instead of 16) to keep the host-side generation of its inputs short.
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


def _ws(op, sp):
    n = tofu.workspace_bytes(op, sp)
    return torch.empty(max(n, 16) // 4, dtype=torch.float32, device=DEV) if n else None


def _close(got, val, absum, what):
    err = np.abs(got.astype(np.float64) - val)
    ratio = np.max(err / np.maximum(absum, 1e-300))
    assert (err <= TOL * absum).all(), f"{what}: worst |err|/S = {ratio:.3e}"
    print(f"{what}: {val.size} outputs, worst |err|/S = {ratio:.2e}", flush=True)


def test_lstm_gate_gemm_all_shards_n_split_and_k_split():
    cfg = synth.CONFIGS["lstm_gates_nsplit"]
    M, N, K, k, seed = cfg["M"], cfg["N"], cfg["K"], cfg["k"], cfg["seed"]
    lo, hi = cfg["b"][1], cfg["b"][2]
    X = synth.draw(cfg["a"], seed, 0, (M, K))
    dX = torch.from_numpy(X).to(DEV)
    op = tofu.matmul_desc(M, N, K)

    def w_block(k0, k1, n0, n1):     # block [k0,k1) x [n0,n1) of the global W, drawn on the device
        rows = torch.arange(k0, k1, dtype=torch.int64, device=DEV).unsqueeze(1) * N
        cols = torch.arange(n0, n1, dtype=torch.int64, device=DEV).unsqueeze(0)
        return synth.uniform_torch(seed, 1, rows + cols, lo, hi)

    # ---- Case-1: every worker writes its column block of the one output tensor ----
    C = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    for s in range(k):
        sp = [(tofu.MM_DIM_N, k, s)]
        n0, n1 = R.shard_range(N, k, s)
        Ws = w_block(0, K, n0, n1)
        tofu.shard_matmul(op, sp, tofu.tensor(dX), tofu.tensor(Ws, [0, n0]), tofu.tensor(C), _ws(op, sp))
        torch.cuda.synchronize()
        del Ws
    # ---- Case-2: every worker produces a full-size partial from its K block; the partials are summed ----
    parts = []
    for s in range(k):
        sp = [(tofu.MM_DIM_K, k, s)]
        k0, k1 = R.shard_range(K, k, s)
        Wr = w_block(k0, k1, 0, N)
        part = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        tofu.shard_matmul(op, sp, tofu.tensor(dX), tofu.tensor(Wr, [k0, 0]), tofu.tensor(part), _ws(op, sp))
        torch.cuda.synchronize()
        parts.append(part)
        del Wr
    tofu.partition_reduce(parts[0], parts)      # in place
    torch.cuda.synchronize()
    # ---- oracle on 512 whole columns (65536 outputs): the first and last column of every shard's block plus seeded ones ----
    edges = [c for s in range(k) for c in (R.shard_range(N, k, s)[0], R.shard_range(N, k, s)[1] - 1)]
    cols = np.unique(np.concatenate([edges, synth.coords(seed, 7, 600, (N,))[:, 0]]))[:512]
    assert len(cols) == 512
    Wc = synth.uniform_at(seed, 1, np.arange(K, dtype=np.int64)[:, None] * N + cols[None, :], lo, hi)
    val, absum = oracle.matmul_box(X, Wc)
    _close(C[:, cols].cpu().numpy(), val, absum, "gate GEMM, 8 N shards concatenated")
    _close(parts[0][:, cols].cpu().numpy(), val, absum, "gate GEMM, 8 K shards summed")
    assert not torch.isnan(C).any() and not torch.isnan(parts[0]).any()


def test_wresnet_conv_all_shards_cout_and_cout_x_h():
    cfg = synth.CONFIGS["wresnet_conv_fwd"]
    NB, C, H, W, k, seed = cfg["batch"], cfg["c_in"], cfg["H"], cfg["W"], cfg["k"], cfg["seed"]
    opd = dict(kind="conv2d", batch=NB, c_in=C, c_out=C, H=H, W=W, KH=3, KW=3, stride=1, pad=1)
    op = tofu.conv2d_desc(NB, C, C, H, W)
    x = synth.draw(cfg["x"], seed, 0, (NB, C, H, W))
    blocks = [R.shard_range(C, k, s) for s in range(k)]
    w = np.concatenate([synth.draw(cfg["w"], seed, 20 + s, (c1 - c0, C, 3, 3)) for s, (c0, c1) in enumerate(blocks)])
    dx, dw = torch.from_numpy(x).to(DEV), torch.from_numpy(w).to(DEV)
    # ---- plan <C_out/8>: 8 workers, each from the whole input ----
    y = torch.full((NB, C, H, W), float("nan"), dtype=torch.float32, device=DEV)
    for s, (c0, c1) in enumerate(blocks):
        sp = [(tofu.CONV_DIM_CO, k, s)]
        tofu.shard_conv2d(op, sp, tofu.tensor(dx), tofu.tensor(dw[c0:c1], [c0, 0, 0, 0]), tofu.tensor(y), _ws(op, sp))
    # ---- plan <C_out/8, H/2>: 16 workers, each reading its rows and the neighbour's halo row from the two owners' blocks ----
    cut = R.shard_range(H, 2, 0)[1]
    own = [dx[:, :, :cut].contiguous(), dx[:, :, cut:].contiguous()]
    srcs = [tofu.tensor(own[0], [0, 0, 0, 0]), tofu.tensor(own[1], [0, 0, cut, 0])]
    y2 = torch.full((NB, C, H, W), float("nan"), dtype=torch.float32, device=DEV)
    for s, (c0, c1) in enumerate(blocks):
        for t in range(2):
            sp = [(tofu.CONV_DIM_CO, k, s), (tofu.CONV_DIM_H, 2, t)]
            tofu.shard_conv2d_fused(op, sp, srcs, tofu.tensor(dw[c0:c1], [c0, 0, 0, 0]), tofu.tensor(y2), _ws(op, sp))
    torch.cuda.synchronize()
    assert not torch.isnan(y).any() and not torch.isnan(y2).any()
    corners = np.array(list(itertools.product((0, NB - 1), (0, C - 1), (0, H - 1), (0, W - 1))), dtype=np.int64)
    seam = np.array([[n, c, h, w_] for n in (0, NB - 1) for c in (0, 319, 320, C - 1) for h in (cut - 1, cut) for w_ in (0, W - 1)], dtype=np.int64)
    pts = np.concatenate([corners, seam, synth.coords(seed, 8, 1 << 16, (NB, C, H, W))])
    val, absum = oracle.conv2d_pts(x, w, pts, stride=1, pad=1)
    idx = tuple(pts.T)
    _close(y.cpu().numpy()[idx], val, absum, "conv, 8 C_out shards concatenated")
    _close(y2.cpu().numpy()[idx], val, absum, "conv, 16 <C_out, H> shards concatenated")


@pytest.mark.timeout(600)
def test_wresnet_wgrad_all_batch_shards_summed():
    cfg = synth.CONFIGS["wresnet_conv_wgrad"]
    C, H, W, k, seed = cfg["c_in"], cfg["H"], cfg["W"], cfg["k"], cfg["seed"]
    NB = cfg["batch"]                                         # the full batch of 128: 16 images per shard
    op = tofu.wgrad_desc(NB, C, C, H, W)
    # every shard's images are drawn as tensors of their own (ids 40 + s, 60 + s), eight at a time on host threads
    from concurrent.futures import ThreadPoolExecutor
    per = NB // k
    with ThreadPoolExecutor(8) as pool:
        xs = list(pool.map(lambda s: synth.draw(cfg["x"], seed, 40 + s, (per, C, H, W)), range(k)))
        dys = list(pool.map(lambda s: synth.draw(cfg["dy"], seed, 60 + s, (per, C, H, W)), range(k)))
    x, dy = np.concatenate(xs), np.concatenate(dys)
    del xs, dys
    dx, ddy = torch.from_numpy(x).to(DEV), torch.from_numpy(dy).to(DEV)
    parts = []
    for s in range(k):
        sp = [(tofu.WGRAD_DIM_N, k, s)]
        n0, n1 = R.shard_range(NB, k, s)
        g = torch.full((C, C, 3, 3), float("nan"), dtype=torch.float32, device=DEV)
        tofu.shard_conv2d_wgrad(op, sp, tofu.tensor(dx[n0:n1], [n0, 0, 0, 0]), tofu.tensor(ddy[n0:n1], [n0, 0, 0, 0]), tofu.tensor(g), _ws(op, sp))
        parts.append(g)
    tofu.partition_reduce(parts[0], parts)
    torch.cuda.synchronize()
    assert not torch.isnan(parts[0]).any()
    corners = np.array(list(itertools.product((0, C - 1), (0, C - 1), (0, 2), (0, 2))), dtype=np.int64)
    pts = np.concatenate([corners, synth.coords(seed, 9, 1 << 16, (C, C, 3, 3))])
    val, absum = oracle.wgrad_pts(x, dy, 3, 3, pts, stride=1, pad=1)
    _close(parts[0].cpu().numpy()[tuple(pts.T)], val, absum, "wgrad, 8 batch shards summed")
