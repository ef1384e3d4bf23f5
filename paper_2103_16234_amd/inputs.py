"""Seeded synthetic inputs and the layer shapes they are drawn for.

This module is shared by the tests, the benchmark and the smoke check. It only
produces tensors and shape records: it holds none of the convolution's
arithmetic and imports neither the HIP binding nor the CPU oracle.

Every value is a pure function of (seed, element index), so any slice of a
tensor can be regenerated anywhere without state:

    h(seed, i) = splitmix64-finaliser(seed * GOLDEN + i)
    uniform u  = (h >> 40) * 2^-24            in [0, 1), exact in fp32
    normal  z  = Box-Muller in fp64 on the draws with counters 2i and 2i+1

The layer shapes stand in for the stride-1 layers of the evaluation sweep
(Section 4, Table 1: square maps of 7..224, 16..2048 filters, 1x1 / 3x3 / 5x5
filters, "same" padding, fp32); activations are post-ReLU-like U[0,1) and
filters He-like N(0, 2/(C*R*S)), except the small first shape which uses
U[-1,1) for both.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _mix(seed: int, counters: np.ndarray) -> np.ndarray:
    """splitmix64 output function applied to seed*GOLDEN + counter (mod 2^64)."""
    with np.errstate(over="ignore"):
        z = np.uint64(seed) * _GOLDEN + counters.astype(np.uint64)
        z = z + _GOLDEN
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform01(seed: int, n: int, start: int = 0) -> np.ndarray:
    """n fp32 values in [0,1) on the 2^-24 grid, elements start..start+n-1."""
    h = _mix(seed, np.arange(start, start + n, dtype=np.uint64))
    return ((h >> np.uint64(40)).astype(np.float64) * 2.0 ** -24).astype(np.float32)


def uniform_pm1(seed: int, n: int, start: int = 0) -> np.ndarray:
    """n fp32 values in [-1,1) on the 2^-23 grid."""
    return (2.0 * uniform01(seed, n, start).astype(np.float64) - 1.0).astype(np.float32)


def normal(seed: int, n: int, sigma: float, start: int = 0) -> np.ndarray:
    """n fp32 draws of N(0, sigma^2): Box-Muller evaluated in fp64, rounded once."""
    i = np.arange(start, start + n, dtype=np.uint64)
    h1 = _mix(seed, np.uint64(2) * i)
    h2 = _mix(seed, np.uint64(2) * i + np.uint64(1))
    u1 = ((h1 >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
    u2 = (h2 >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return (sigma * z).astype(np.float32)


def small_ints(seed: int, n: int, lo: int, hi: int, start: int = 0) -> np.ndarray:
    """n fp32 values that are integers in [lo, hi]: for exact-arithmetic checks."""
    h = _mix(seed, np.arange(start, start + n, dtype=np.uint64))
    span = np.uint64(hi - lo + 1)
    return ((h >> np.uint64(33)) % span).astype(np.int64).astype(np.float32) + np.float32(lo)


@dataclass(frozen=True)
class ConvShape:
    """One stride-1 forward convolution: x[N,C,H,W] * w[K,C,R,S] -> y[N,K,P,Q]."""

    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    pad_h: int
    pad_w: int
    x_dist: str = "u01"      # "u01" | "upm1" | "int"
    w_dist: str = "he"       # "he"  | "upm1" | "int"
    x_seed: int = 1
    w_seed: int = 2

    @property
    def P(self) -> int:
        return self.H + 2 * self.pad_h - self.R + 1

    @property
    def Q(self) -> int:
        return self.W + 2 * self.pad_w - self.S + 1

    @property
    def dims(self) -> tuple:
        return (self.N, self.C, self.H, self.W, self.K, self.R, self.S, self.pad_h, self.pad_w)

    @property
    def x_shape(self) -> tuple:
        return (self.N, self.C, self.H, self.W)

    @property
    def w_shape(self) -> tuple:
        return (self.K, self.C, self.R, self.S)

    @property
    def y_shape(self) -> tuple:
        return (self.N, self.K, self.P, self.Q)

    @property
    def flops(self) -> int:
        """Effective FLOPs: 2 per multiply-add, padding taps counted."""
        return 2 * self.N * self.K * self.P * self.Q * self.C * self.R * self.S

    @property
    def algorithmic_bytes(self) -> int:
        """Compulsory traffic of a direct convolution: x and w read once, y written once."""
        nx = self.N * self.C * self.H * self.W
        nw = self.K * self.C * self.R * self.S
        ny = self.N * self.K * self.P * self.Q
        return 4 * (nx + nw + ny)

    def with_batch(self, n: int) -> "ConvShape":
        d = dict(self.__dict__)
        d["N"] = n
        d["name"] = f"{self.name}@N{n}"
        return ConvShape(**d)


def _draw(dist: str, seed: int, n: int, fan_in: int) -> np.ndarray:
    if dist == "u01":
        return uniform01(seed, n)
    if dist == "upm1":
        return uniform_pm1(seed, n)
    if dist == "he":
        return normal(seed, n, float(np.sqrt(2.0 / fan_in)))
    if dist == "int":
        return small_ints(seed, n, -3, 3)
    raise ValueError(f"unknown distribution {dist!r}")


def make_inputs(shape: ConvShape):
    """(x, w) as C-contiguous fp32 numpy arrays for a shape record."""
    fan_in = shape.C * shape.R * shape.S
    x = _draw(shape.x_dist, shape.x_seed, int(np.prod(shape.x_shape)), fan_in).reshape(shape.x_shape)
    w = _draw(shape.w_dist, shape.w_seed, int(np.prod(shape.w_shape)), fan_in).reshape(shape.w_shape)
    return np.ascontiguousarray(x), np.ascontiguousarray(w)


# The five benchmark layers; seeds are 1000+i for x and 2000+i for w (i = 1..5).
CONFIGS = (
    ConvShape("cfg1_3x3_c16_14", 1, 16, 14, 14, 16, 3, 3, 1, 1, "upm1", "upm1", 1001, 2001),
    ConvShape("cfg2_1x1_c256_56", 1, 256, 56, 56, 64, 1, 1, 0, 0, "u01", "he", 1002, 2002),
    ConvShape("cfg3_3x3_c64_56", 8, 64, 56, 56, 64, 3, 3, 1, 1, "u01", "he", 1003, 2003),
    ConvShape("cfg4_5x5_c48_28", 1, 48, 28, 28, 128, 5, 5, 2, 2, "u01", "he", 1004, 2004),
    ConvShape("cfg5_3x3_c512_14", 32, 512, 14, 14, 512, 3, 3, 1, 1, "u01", "he", 1005, 2005),
)


def config(i: int) -> ConvShape:
    """Benchmark layer i, 1-based as the layers are numbered in the reports."""
    return CONFIGS[i - 1]


# Second workload: a product grid of synthetic layer shapes inside the ranges of the evaluation sweep (Section 4,
# Table 1: batch 1..256, square maps 7..224, 16..2048 filters, 1x1 / 3x3 / 5x5 filters with "same" padding). It is
# a grid over those ranges, not any network's layer list; channel counts shrink as maps grow, as they do in CNNs.
_SWEEP_BATCHES = (1, 8, 16, 32, 64, 128, 256)
_SWEEP_CHANNELS = {   # map size -> (C, K) pairs, per filter size
    1: {7: ((512, 512), (832, 256), (1024, 2048)), 13: ((256, 384), (384, 384)), 14: ((256, 256), (512, 512), (256, 1024)),
        27: ((64, 256), (96, 256)), 28: ((128, 128), (192, 256), (512, 128)), 56: ((64, 64), (256, 64), (64, 256)),
        112: ((32, 64), (64, 128))},
    3: {7: ((512, 512), (192, 384), (512, 2048)), 13: ((256, 384), (384, 384)), 14: ((256, 256), (512, 512), (512, 1024)),
        27: ((64, 192), (96, 256)), 28: ((128, 128), (128, 256)), 56: ((64, 64), (64, 192)),
        112: ((32, 64), (64, 128)), 224: ((3, 64), (16, 16), (64, 64))},
    5: {7: ((48, 128), (32, 128), (64, 512)), 13: ((32, 96), (48, 128)), 14: ((16, 48), (32, 96)), 27: ((48, 128), (96, 256)),
        28: ((16, 32), (32, 96), (48, 128))},
}


def sweep_shapes(max_elems: int = 1 << 25):
    """The shapes of the sweep workload whose x and y both hold at most max_elems elements."""
    out = []
    for f in (1, 3, 5):
        for hw in sorted(_SWEEP_CHANNELS[f]):
            for (c, k) in _SWEEP_CHANNELS[f][hw]:
                for n in _SWEEP_BATCHES:
                    if n * c * hw * hw > max_elems or n * k * hw * hw > max_elems:
                        continue
                    i = len(out)
                    out.append(ConvShape(f"sweep_{f}x{f}_n{n}_c{c}_{hw}_k{k}", n, c, hw, hw, k, f, f, f // 2, f // 2,
                                         "u01", "he", 3000 + i, 4000 + i))
    return out
