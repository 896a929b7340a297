"""GPU parity at the full workload sizes, in the launch configuration bench.py times: every
leg of tofu_workloads.build() is run once and checked against the oracle on seeded samples
of output coordinates; the copy is checked in full.  The samples of a contraction are
  * seeded uniform points and the corners of the output box,
  * points on every face of the output box, and
  * one point in every 32 x 32 block of the kernel's matrix view of the output ([m] x [n];
    [c_out] x [positions in n-major order over the box]; [c_out] x [c_in] per filter tap), the
    size of one matrix-core accumulator block: whatever tiles a launch cuts that matrix into,
    every accumulator block of every tile is hit, for the weight gradient at every tap."""
import itertools

import numpy as np
import pytest
import torch

import oracle
import tofu_synth as synth
import tofu_workloads
from oracle import regions as R

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _points(seed, n, shape):
    corners = list(itertools.product(*[(0, e - 1) for e in shape]))
    return np.concatenate([np.array(corners, dtype=np.int64), synth.coords(seed, 0, n, shape)])


def _faces(seed, per_face, shape):
    """Seeded points on each of the 2 * ndim faces of a box of `shape`."""
    out = []
    for d, e in enumerate(shape):
        for side, v in enumerate((0, e - 1)):
            p = synth.coords(seed, 10 + 2 * d + side, per_face, shape)
            p[:, d] = v
            out.append(p)
    return np.concatenate(out)


def _strata(seed, rows, cols, block=32):
    """One seeded (row, col) inside every block x block cell of a rows x cols matrix (ragged last cells included)."""
    br, bc = (rows + block - 1) // block, (cols + block - 1) // block
    off = synth.coords(seed, 30, br * bc, (block, block))
    r = np.minimum(np.repeat(np.arange(br), bc) * block + off[:, 0], rows - 1)
    c = np.minimum(np.tile(np.arange(bc), br) * block + off[:, 1], cols - 1)
    return r, c


def _conv_points(seed, n, shape):
    """Sample coordinates of a [batch, channels, h, w] output: uniform + corners + faces + one per 32 x 32 block of
    the [channels] x [positions] matrix, positions numbered batch-major over the box."""
    nb, ch, bh, bw = shape
    r, c = _strata(seed, ch, nb * bh * bw)
    strat = np.stack([c // (bh * bw), r, (c // bw) % bh, c % bw], axis=1).astype(np.int64)
    return np.concatenate([_points(seed, n, shape), _faces(seed, 48, shape), strat])


def _close(got, val, absum, what):
    err = np.abs(got.astype(np.float64) - val)
    assert (err <= TOL * absum).all(), f"{what}: worst ratio {np.max(err / np.maximum(absum, 1e-300)):.3e}"
    print(f"{what}: {len(val)} samples, worst |err|/S = {np.max(err / np.maximum(absum, 1e-300)):.2e}", flush=True)


def _check_reduce(leg):
    h = leg.host
    out = leg.out.cpu().numpy().ravel()
    own = h["own"].cpu().numpy().ravel()
    idx = np.unique(np.concatenate([[0, out.size - 1], synth.coords(77, 0, 1 << 16, (out.size,))[:, 0]]))
    parts = [r.ravel()[idx] for r in h["remote"]]
    parts.insert(h["own_index"], own[idx])
    val, absum = oracle.reduce(parts)
    _close(out[idx], val, absum, leg.name)
    # left-to-right fp32 order, exactly
    ref = parts[0].copy()
    for p in parts[1:]:
        ref = ref + p
    assert np.array_equal(out[idx], ref)


@pytest.mark.parametrize("group", [("gemm_nsplit",), ("gemm_dx_nsplit", "gemm_dw_nsplit"), ("gemm_ksplit", "reduce_gates"),
                                   ("conv_cout", "fetch_halo", "conv_cout_h", "conv_cout_h_fused"), ("wgrad_batch", "reduce_dw"), ("dgrad_cout",), ("lstm_cell_nsplit",),
                                   ("gemm_ksplit_accumulate",), ("wgrad_batch_accumulate",), ("conv1d_cout",)])
def test_full_size_legs(group):
    print(f"building {group}", flush=True)
    legs = tofu_workloads.build("cuda:0", group)
    assert [l.name for l in legs] == list(group)
    for leg in legs:
        print(f"running {leg.name}", flush=True)
        leg.run()
        torch.cuda.synchronize()
        h = leg.host
        if h["kind"] == "matmul":
            box = h["box"]
            (m0, m1), (n0, n1) = box
            r, c = _strata(71, m1 - m0, n1 - n0)
            pts = np.concatenate([_points(71, 4096, (m1 - m0, n1 - n0)), _faces(71, 64, (m1 - m0, n1 - n0)), np.stack([r, c], axis=1).astype(np.int64)])
            k0, k1 = h["krange"]
            if "b_col0" in h:     # B holds the shard's columns only
                val, absum = oracle.matmul_pts(h["A"], h["B"], pts)
            else:                 # B holds the shard's rows only
                val, absum = oracle.matmul_pts(np.ascontiguousarray(h["A"][:, k0:k1]), h["B"], pts)
            got = leg.out.cpu().numpy()[pts[:, 0] + m0, pts[:, 1] + n0]
            _close(got, val, absum, leg.name)
        elif h["kind"] == "conv2d":
            y = leg.out.cpu().numpy()
            pts = _conv_points(72, 4096, y.shape)
            h0 = h["box"][2][0]
            opts = pts.copy()
            opts[:, 2] += h0      # output row in global coordinates; channels stay local to the shard's filters
            val, absum = oracle.conv2d_pts(h["x"], h["w"], opts, stride=1, pad=1)
            _close(y[tuple(pts.T)], val, absum, leg.name)
            if leg.name == "conv_cout_h_fused":   # reading the blocks directly changes no bit of the result
                fetched = next(l for l in legs if l.name == "conv_cout_h")
                assert torch.equal(leg.out, fetched.out)
        elif h["kind"] == "conv1d":
            y = leg.out.cpu().numpy()
            pts = _points(75, 4096, y.shape)
            # the oracle evaluates a box; sample rows of outputs instead of single points: 8 (b, co) rows, all x
            for b, co, _ in pts[:8]:
                val, absum = oracle.conv1d_box(h["data"][b:b + 1], np.ascontiguousarray(h["filters"][:, co:co + 1]))
                _close(y[b, co], val[0, 0], absum[0, 0], leg.name)
        elif h["kind"] == "lstm":
            cn, hn, sc = oracle.lstm_cell(h["gates"], h["c"])
            _close(leg.out.cpu().numpy().ravel(), cn.ravel(), sc.ravel(), leg.name + " c")
            _close(h["h_out"].cpu().numpy().ravel(), hn.ravel(), np.ones(hn.size), leg.name + " h")
        elif h["kind"] == "dgrad":
            dxp = leg.out.cpu().numpy()
            pts = _conv_points(74, 4096, dxp.shape)
            val, absum = oracle.dgrad_pts(h["dy"], h["w"], h["H"], h["W"], pts, stride=1, pad=1)   # the shard's output channels only
            _close(dxp[tuple(pts.T)], val, absum, leg.name)
        elif h["kind"] == "wgrad":
            dw = leg.out.cpu().numpy()
            # one point per (32 output channels, 32 input channels, tap) block, plus faces, corners and uniform points
            co_n, ci_n = dw.shape[0], dw.shape[1]
            r, c = _strata(73, co_n, ci_n)
            strat = np.concatenate([np.stack([r, c, np.full_like(r, t // 3), np.full_like(r, t % 3)], axis=1) for t in range(9)]).astype(np.int64)
            pts = np.concatenate([_points(73, 2048, dw.shape), _faces(73, 48, dw.shape), strat])
            val, absum = oracle.wgrad_pts(h["x"], h["dy"], 3, 3, pts, stride=1, pad=1)   # the shard's images only
            _close(dw[tuple(pts.T)], val, absum, leg.name)
        elif h["kind"] == "fetch":
            x, box = h["x"], h["box"]
            cut = 7
            want = R.fetch(box, [(x[:, :, :cut], [(0, x.shape[0]), (0, x.shape[1]), (0, cut), (0, x.shape[3])]),
                                 (x[:, :, cut:cut + 1], [(0, x.shape[0]), (0, x.shape[1]), (cut, cut + 1), (0, x.shape[3])])])
            assert np.array_equal(leg.out.cpu().numpy(), want), "fetched region differs from the oracle's"
            print(f"{leg.name}: {want.size} elements bit-exact", flush=True)
        elif h["kind"] == "reduce":
            _check_reduce(leg)
    del legs
    torch.cuda.empty_cache()


def test_step_replays_from_a_hip_graph_bit_identically():
    """Every entry point only enqueues kernels on the caller's stream (no allocation, no
    synchronisation, no memset), so a whole step can be captured once and replayed: three
    replays, with eager work and synchronisations in between, each reproduce the eager outputs
    bit for bit."""
    legs = tofu_workloads.build("cuda:0", ["gemm_ksplit", "reduce_gates", "fetch_halo", "conv_cout_h", "wgrad_batch", "reduce_dw"], keep_host=False)
    for leg in legs:
        leg.run()
    torch.cuda.synchronize()
    eager = [leg.out.clone() for leg in legs]
    for leg in legs:
        leg.out.fill_(float("nan"))
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for leg in legs:          # warm-up on the capture stream
            leg.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        for leg in legs:
            leg.run()
    for replay in range(3):
        for leg in legs:
            leg.out.fill_(float("nan"))          # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for leg, want in zip(legs, eager):
            assert torch.equal(leg.out, want), (leg.name, replay)
    del graph, legs
    torch.cuda.empty_cache()
