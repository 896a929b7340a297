"""GPU test of tofu_shard_matmul_noalloc, the shard GEMM for callers that cannot allocate: its K
slices go to the library's built-in device array instead of a caller's workspace.  It runs the
kernels of tofu_shard_matmul, so its output must equal that entry point's bit for bit; the
existing entry point is itself checked against the oracle here at the stated tolerance.  Two
calls in a row share the array, the second with a smaller input.  Collected last on purpose."""
import numpy as np
import pytest
import torch

import oracle
import paper_1807_08887_amd as tofu
import tofu_synth as synth
from paper_1807_08887_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _pair(seed, M, N, K, splits):
    """Run both entry points on the same seeded operands; -> (reference output, no-alloc output, A, B, box)."""
    A, B = synth.uniform(seed, 0, (M, K), -1, 1), synth.uniform(seed, 1, (K, N), -1, 1)
    dA, dB = torch.from_numpy(A).to(DEV), torch.from_numpy(B).to(DEV)
    op = tofu.matmul_desc(M, N, K)
    need = tofu.workspace_bytes(op, splits)
    ws = torch.empty(max(need // 4, 1), dtype=torch.float32, device=DEV) if need else None
    ref = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
    got = torch.full((M, N), -7.0, dtype=torch.float32, device=DEV)
    tofu.shard_matmul(op, splits, tofu.tensor(dA), tofu.tensor(dB), tofu.tensor(ref), ws)
    tofu.shard_matmul_noalloc(op, splits, tofu.tensor(dA), tofu.tensor(dB), tofu.tensor(got))
    torch.cuda.synchronize()
    return ref, got, A, B, tofu.op_regions(op, splits), need


def _check_against_oracle(out, A, B, reg):
    (m0, m1), (n0, n1) = reg["out_box"]
    (k0, k1) = reg["in_boxes"][0][1]
    val, absum = oracle.matmul_box(A[:, k0:k1], B[k0:k1, :])
    got = out.cpu().numpy().astype(np.float64)
    assert (np.abs(got[m0:m1, n0:n1] - val[m0:m1, n0:n1]) <= 1e-5 * absum[m0:m1, n0:n1]).all()
    mask = np.ones(got.shape, dtype=bool)
    mask[m0:m1, n0:n1] = False
    assert (got[mask] == -7.0).all()          # nothing outside the shard's box is written


def test_noalloc_matches_workspace_entry_point_on_two_calls_in_a_row():
    # first call: tall-skinny shard whose K range is cut into slices (uses the scratch array)
    ref, got, A, B, reg, need = _pair(41, 96, 512, 6144, [(tofu.MM_DIM_N, 2, 1)])
    assert need > 0, "the first case must be one that needs the scratch array"
    assert torch.equal(ref, got)
    _check_against_oracle(got, A, B, reg)
    # second call right after it: a smaller shard, ragged against the tiles, slices again
    ref2, got2, A2, B2, reg2, need2 = _pair(42, 50, 200, 2100, [(tofu.MM_DIM_K, 2, 0)])
    assert 0 < need2 < need
    assert torch.equal(ref2, got2)
    _check_against_oracle(got2, A2, B2, reg2)
    # and a shard that needs no slices at all goes through the same entry point
    ref3, got3, A3, B3, reg3, need3 = _pair(43, 300, 700, 96, [(tofu.MM_DIM_M, 3, 2)])
    assert need3 == 0
    assert torch.equal(ref3, got3)
    _check_against_oracle(got3, A3, B3, reg3)


def test_noalloc_rejects_a_shard_beyond_the_scratch_array():
    # look for a tall-skinny shard whose K slices need more than the array (the launch plan decides)
    found = None
    for M, n, K in [(128, 4096, 1 << 15), (256, 4096, 1 << 15), (128, 8192, 1 << 15), (512, 2048, 1 << 15), (384, 4096, 1 << 14)]:
        op = tofu.matmul_desc(M, 8 * n, K)
        if tofu.workspace_bytes(op, [(tofu.MM_DIM_N, 8, 0)]) > binding.STATIC_SCRATCH_BYTES:
            found = (M, n, K, op)
            break
    if found is None:
        pytest.skip("no matmul launch plan needs more K-slice space than the built-in array holds")
    M, n, K, op = found
    A = torch.zeros(M, K, dtype=torch.float32, device=DEV)
    B = torch.zeros(K, n, dtype=torch.float32, device=DEV)
    C = torch.full((M, n), 3.0, dtype=torch.float32, device=DEV)
    with pytest.raises(tofu.TofuError) as err:
        tofu.shard_matmul_noalloc(op, [(tofu.MM_DIM_N, 8, 0)], tofu.tensor(A), tofu.tensor(B), tofu.tensor(C))
    assert err.value.status == -5 and "scratch" in str(err.value)
    torch.cuda.synchronize()
    assert (C == 3.0).all()                   # nothing was launched
