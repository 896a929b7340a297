"""GPU parity at the full workload sizes, in the launch configuration bench.py times: every
leg of tofu_workloads.build() is run once and checked against the oracle on seeded samples
of output coordinates (plus the corners of the output box); the copy is checked in full."""
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
            pts = _points(71, 4096, (m1 - m0, n1 - n0))
            k0, k1 = h["krange"]
            if "b_col0" in h:     # B holds the shard's columns only
                val, absum = oracle.matmul_pts(h["A"], h["B"], pts)
            else:                 # B holds the shard's rows only
                val, absum = oracle.matmul_pts(np.ascontiguousarray(h["A"][:, k0:k1]), h["B"], pts)
            got = leg.out.cpu().numpy()[pts[:, 0] + m0, pts[:, 1] + n0]
            _close(got, val, absum, leg.name)
        elif h["kind"] == "conv2d":
            y = leg.out.cpu().numpy()
            pts = _points(72, 4096, y.shape)
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
            pts = _points(74, 4096, dxp.shape)
            val, absum = oracle.dgrad_pts(h["dy"], h["w"], h["H"], h["W"], pts, stride=1, pad=1)   # the shard's output channels only
            _close(dxp[tuple(pts.T)], val, absum, leg.name)
        elif h["kind"] == "wgrad":
            dw = leg.out.cpu().numpy()
            pts = _points(73, 2048, dw.shape)
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
