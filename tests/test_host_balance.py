"""Host-side check of the work distribution the convolution and weight-gradient kernels use for
their balanced launches (csrc/tofu_balance.h; a partition-n-reduce inside one worker, Sec. 3.1):
tests/native/balance_check.cpp is compiled with the host compiler and run.  It enumerates tile
counts, step counts and workgroup limits and checks that the segments of all workgroups cover
every (tile, step) exactly once, that every segment owns a distinct slot inside the workspace the
plan asks for, that a tile's slots are summed in the order of their steps, and that no workgroup is
more than 5 % busier than under an even split."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)


def test_balance_plan_covers_every_step_once(tmp_path):
    exe = str(tmp_path / "balance_check")
    src = os.path.join(HERE, "native", "balance_check.cpp")
    inc = os.path.join(ROOT, "paper_1807_08887_amd", "csrc")
    subprocess.run(["g++", "-O1", "-std=c++17", "-I", inc, src, "-o", exe], check=True)
    out = subprocess.run([exe], capture_output=True, text=True)
    print(out.stdout)
    assert out.returncode == 0, out.stdout[-2000:] + out.stderr[-2000:]
    # the shapes the benchmark launches: (tiles, steps) -> all 512 workgroups used
    assert "n=490 steps=640: groups=512" in out.stdout
    assert "n=400 steps=448: groups=512" in out.stdout
