"""Seeded synthetic inputs for the sliding-window workloads.

This module holds no convolution or pooling arithmetic: it only draws numbers.
Both the GPU tests and the CPU oracle's tests take their inputs from here, so
that the two sides see identical bits.

The paper measures on no public dataset (its section 2 varies only the filter
size), so the workloads are synthetic by construction.  Seeds follow
``BASE_SEED + 1000*workload + tensor_index``.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 231005218


def seed_for(workload: int, tensor_index: int) -> int:
    return BASE_SEED + 1000 * workload + tensor_index


def uniform_f32(shape, seed: int, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.uniform(lo, hi, size=shape).astype(np.float32)


def normal_f32(shape, seed: int, std: float = 1.0) -> np.ndarray:
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def normal_bf16(shape, seed: int, std: float = 1.0) -> np.ndarray:
    """bf16 bit patterns (uint16) of N(0, std^2) draws: the upper half of each fp32 draw's bit pattern (no rounding
    arithmetic lives here: checkers widen the patterns with their own helper)."""
    return (normal_f32(shape, seed, std).view(np.uint32) >> 16).astype(np.uint16)


def normal_f16(shape, seed: int, std: float = 1.0) -> np.ndarray:
    """IEEE half-precision bit patterns (uint16) of N(0, std^2) draws (numpy's cast of each fp32 draw)."""
    return normal_f32(shape, seed, std).astype(np.float16).view(np.uint16)


def uniform_s8(shape, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(-128, 128, size=shape, dtype=np.int8)


def small_ints_f32(shape, seed: int, lo: int = -4, hi: int = 4) -> np.ndarray:
    """Integer-valued floats: every product and partial sum is exact in fp32 and fp64."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=shape).astype(np.float32)


# ---------------------------------------------------------------------------
# The five workloads (shapes, distributions) the measurements are quoted on.
# ---------------------------------------------------------------------------

WORKLOADS = {
    1: dict(name="conv2d 1x1x256x256 fp32, 3x3, valid",
            N=1, C_in=1, C_out=1, H=256, W=256, R=3, S=3, stride=1, pad=0),
    2: dict(name="1-D sliding sums, 64 rows x 65536 fp32: conv1d k=9, avg/max pool window 8",
            rows=64, len=65536, k=9, window=8, stride=1, pad=0),
    3: dict(name="conv2d 32x64x56x56 fp32 -> 64 ch, 3x3, pad 1",
            N=32, C_in=64, C_out=64, H=56, W=56, R=3, S=3, stride=1, pad=1),
    4: dict(name="depthwise conv2d 32x256x56x56 fp32, 3x3 pad 1 and 7x7 pad 3",
            N=32, C=256, H=56, W=56, stride=1),
    5: dict(name="conv2d int8 32x128x28x28 -> 128 ch, 3x3, pad 1, int32 out",
            N=32, C_in=128, C_out=128, H=28, W=28, R=3, S=3, stride=1, pad=1),
}


def workload1():
    c = WORKLOADS[1]
    x = uniform_f32((c["N"], c["C_in"], c["H"], c["W"]), seed_for(1, 0))
    w = uniform_f32((c["C_out"], c["C_in"], c["R"], c["S"]), seed_for(1, 1))
    return x, w


def workload2(rows: int | None = None, length: int | None = None):
    c = WORKLOADS[2]
    rows = c["rows"] if rows is None else rows
    length = c["len"] if length is None else length
    x = normal_f32((rows, length), seed_for(2, 0))
    w = normal_f32((c["k"],), seed_for(2, 1))
    return x, w


def workload3(N: int | None = None):
    c = WORKLOADS[3]
    N = c["N"] if N is None else N
    x = normal_f32((N, c["C_in"], c["H"], c["W"]), seed_for(3, 0))
    std = math.sqrt(2.0 / (c["C_in"] * c["R"] * c["S"]))  # Kaiming-normal, fan-in
    w = normal_f32((c["C_out"], c["C_in"], c["R"], c["S"]), seed_for(3, 1), std)
    return x, w


def workload4(N: int | None = None, C: int | None = None):
    """Returns x, w3 ([C,1,3,3], variance 1/9) and w7 ([C,1,7,7], variance 1/49)."""
    c = WORKLOADS[4]
    N = c["N"] if N is None else N
    C = c["C"] if C is None else C
    x = normal_f32((N, C, c["H"], c["W"]), seed_for(4, 0))
    w3 = normal_f32((C, 1, 3, 3), seed_for(4, 1), 1.0 / 3.0)
    w7 = normal_f32((C, 1, 7, 7), seed_for(4, 2), 1.0 / 7.0)
    return x, w3, w7


def workload5(N: int | None = None):
    c = WORKLOADS[5]
    N = c["N"] if N is None else N
    x = uniform_s8((N, c["C_in"], c["H"], c["W"]), seed_for(5, 0))
    w = uniform_s8((c["C_out"], c["C_in"], c["R"], c["S"]), seed_for(5, 1))
    return x, w
