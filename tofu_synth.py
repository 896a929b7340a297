"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests and bench.

This module only draws numbers and lists workload shapes.  It contains none of
the method's arithmetic (no split ranges, no regions, no operators): both the
oracle and the HIP library are handed the arrays made here, so the two sides
always see bit-identical fp32 inputs.

Generator: a counter-based hash.  Element `i` of tensor `tid` under `seed`
depends only on (seed, tid, i), so any block of a tensor can be drawn alone and
the result does not depend on chunking or on the machine.
  u64  = mix(seed, tid, i)              (SplitMix64 finaliser, public-domain constants)
  unif = (top 24 bits + 0.5) / 2^24     in (0,1)
  norm = sqrt(-2 ln u1) cos(2 pi u2)    Box-Muller in fp64, rounded once to fp32

The workloads stand in for the paper's evaluation models (Sec. 7.1): a stacked
LSTM with hidden size 8192 trained at batch 128, and Wide-ResNet bottleneck 3x3
convolutions widened x10 at batch 128.  The paper prints no layer shapes and
trains on no labelled data for its throughput figures, so shapes are derived
from those model descriptions and every value is synthetic.
"""
from __future__ import annotations

import math

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_CHUNK = 1 << 22


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z + np.uint64(0x9E3779B97F4A7C15)) & _M64
    z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _M64
    z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _M64
    return z ^ (z >> np.uint64(31))


def _bits(seed: int, tid: int, stream: int, start: int, count: int) -> np.ndarray:
    """64 hashed bits for elements start..start+count of (seed, tid, stream)."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed * 0x100000001B3 + tid * 2 + stream) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix(idx ^ key[0])


def _unit(bits: np.ndarray) -> np.ndarray:
    return ((bits >> np.uint64(40)).astype(np.float64) + 0.5) * (1.0 / 16777216.0)


def _fill(shape, fn) -> np.ndarray:
    n = int(np.prod(shape, dtype=np.int64)) if len(shape) else 1
    out = np.empty(n, dtype=np.float32)
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        out[s:s + c] = fn(s, c)
    return out.reshape(shape)


def uniform(seed: int, tid: int, shape, lo: float, hi: float) -> np.ndarray:
    """fp32 tensor, elements uniform in (lo, hi)."""
    return _fill(shape, lambda s, c: lo + (hi - lo) * _unit(_bits(seed, tid, 0, s, c)))


def uniform_at(seed: int, tid: int, index: np.ndarray, lo: float, hi: float) -> np.ndarray:
    """The elements of uniform(seed, tid, ...) at the given flat (row-major) indices: the
    generator is counter-based, so a few columns of a tensor too large to draw whole can be
    drawn alone, bit for bit as they would appear in the whole tensor."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([(seed * 0x100000001B3 + tid * 2) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))
        bits = _mix(np.asarray(index).astype(np.uint64) ^ key[0])
    return (lo + (hi - lo) * _unit(bits)).astype(np.float32)


def uniform_torch(seed: int, tid: int, index, lo: float, hi: float):
    """The same elements drawn on the device: `index` is an int64 torch tensor of flat indices
    (any shape); returns a float32 tensor of that shape, bit-identical to uniform_at.  64-bit
    unsigned arithmetic is emulated on int64 (wrapping multiply, masked shifts)."""
    import torch

    def s64(v):                      # the uint64 constant as the int64 with the same bits
        v &= 0xFFFFFFFFFFFFFFFF
        return v - (1 << 64) if v >= (1 << 63) else v

    def shr(z, n):                   # logical shift right
        return (z >> n) & ((1 << (64 - n)) - 1)

    def mix(z):
        z = z + s64(0x9E3779B97F4A7C15)
        z = (z ^ shr(z, 30)) * s64(0xBF58476D1CE4E5B9)
        z = (z ^ shr(z, 27)) * s64(0x94D049BB133111EB)
        return z ^ shr(z, 31)
    with np.errstate(over="ignore"):
        key = int(_mix(np.array([(seed * 0x100000001B3 + tid * 2) & 0xFFFFFFFFFFFFFFFF], dtype=np.uint64))[0])
    bits = mix(index ^ s64(key))
    unit = (shr(bits, 40).to(torch.float64) + 0.5) * (1.0 / 16777216.0)
    return (lo + (hi - lo) * unit).to(torch.float32)


def normal(seed: int, tid: int, shape, std: float = 1.0) -> np.ndarray:
    """fp32 tensor, elements N(0, std^2)."""
    def fn(s, c):
        u1 = _unit(_bits(seed, tid, 0, s, c))
        u2 = _unit(_bits(seed, tid, 1, s, c))
        return std * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
    return _fill(shape, fn)


def small_int(seed: int, tid: int, shape, lo: int, hi: int) -> np.ndarray:
    """fp32 tensor of integers in [lo, hi]; sums of products of these stay exact in fp32
    as long as they are below 2^24, which makes bit-exact comparisons meaningful."""
    span = hi - lo + 1
    return _fill(shape, lambda s, c: lo + ((_bits(seed, tid, 0, s, c) >> np.uint64(33)) % np.uint64(span)).astype(np.float64))


def coords(seed: int, tid: int, count: int, shape) -> np.ndarray:
    """`count` int64 coordinates drawn uniformly from a tensor of `shape` -> [count, ndim]."""
    out = np.empty((count, len(shape)), dtype=np.int64)
    for d, ext in enumerate(shape):
        out[:, d] = (_bits(seed, tid, 2 + d, 0, count) >> np.uint64(11)) % np.uint64(ext)
    return out


# --------------------------------------------------------------------------------------
# The five workloads.  `k` and `shard` give the partition the timed worker belongs to.
# Distributions of the stand-in "remote partials": the natural distribution of an own
# partial (variance = number of summed terms x variance of one product).
# --------------------------------------------------------------------------------------
HE_STD_2560 = math.sqrt(2.0 / (2560 * 9))

CONFIGS = {
    # tiny matmul: K-split (two partials summed) and N-split (concatenated)
    "tiny_matmul": dict(kind="matmul", seed=101, M=64, N=96, K=128, k=2,
                        a=("uniform", -1.0, 1.0), b=("uniform", -1.0, 1.0)),
    # LSTM gate GEMM, input+hidden = 16384, 4 gates x 8192; 8-way split of the output dim N
    "lstm_gates_nsplit": dict(kind="matmul", seed=202, M=128, N=32768, K=16384, k=8, shard=3, split="N",
                              a=("normal", 1.0), b=("uniform", -1.0 / 128.0, 1.0 / 128.0)),
    # same GEMM, 8-way split of the reduction dim K; 7 remote partials ~ N(0, 2048/(3*128^2)) = N(0, 1/24)
    "lstm_gates_ksplit": dict(kind="matmul", seed=303, M=128, N=32768, K=16384, k=8, shard=3, split="K",
                              a=("normal", 1.0), b=("uniform", -1.0 / 128.0, 1.0 / 128.0),
                              partial_std=math.sqrt(1.0 / 24.0)),
    # Wide-ResNet 3x3 conv, 2560 channels at 14x14: 8-way C_out split (+ 2-way H split with halo)
    "wresnet_conv_fwd": dict(kind="conv2d", seed=404, batch=128, c_in=2560, c_out=2560, H=14, W=14,
                             KH=3, KW=3, stride=1, pad=1, k=8, shard=3, k_h=2, shard_h=0,
                             x=("normal", 1.0), w=("normal", HE_STD_2560)),
    # Wide-ResNet 3x3 conv weight gradient, 1280 channels at 28x28: 8-way batch split; partials ~ N(0, 16*784)
    "wresnet_conv_wgrad": dict(kind="conv2d_wgrad", seed=505, batch=128, c_in=1280, c_out=1280, H=28, W=28,
                               KH=3, KW=3, stride=1, pad=1, k=8, shard=3,
                               x=("normal", 1.0), dy=("normal", 1.0), partial_std=math.sqrt(16.0 * 784.0)),
    # the paper's running example at a large size: conv1d, 2048 channels, window 3, 512 outputs per row; 8-way C_out split
    "conv1d_large": dict(kind="conv1d", seed=606, batch=64, c_in=2048, c_out=2048, W=514, KW=3, k=8, shard=3,
                         x=("normal", 1.0), w=("normal", math.sqrt(2.0 / (2048 * 3)))),
}


def draw(spec, seed: int, tid: int, shape) -> np.ndarray:
    """Draw a tensor from a ("uniform", lo, hi) / ("normal", std) / ("int", lo, hi) spec."""
    if spec[0] == "uniform":
        return uniform(seed, tid, shape, spec[1], spec[2])
    if spec[0] == "normal":
        return normal(seed, tid, shape, spec[1])
    if spec[0] == "int":
        return small_int(seed, tid, shape, spec[1], spec[2])
    raise ValueError(f"unknown distribution {spec!r}")
