"""Seeded synthetic conv2d workloads (shapes + int8 tensors).

This module only *generates inputs*: it holds none of the method's arithmetic
(no convolution, no packing, no im2col, no cost model).  Both the GPU path and
the CPU checker are fed from here so that they see identical bytes.

Shapes stand in for the DeepBench inference convolutions the paper measures on
(Sec. 5.1): ordinary many-channel 3x3 layers, the 7x7 stride-2 three-channel
stem and the one-channel 20x5 stride-2 speech layer of Table 3.  Values are
seeded noise; the computation is data independent.

Generator: SplitMix64 used counter-based.  Element i of stream `seed` is
    z = seed + (i+1)*0x9E3779B97F4A7C15  (mod 2^64)
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9
    z = (z ^ (z >> 27)) * 0x94D049BB133111EB
    z =  z ^ (z >> 31)
uniform int8  = low byte of z reinterpreted as two's complement;
normal  int8  = clip(rint(sigma * sqrt(-2 ln u1) * cos(2 pi u2)), -128, 127)
                with u1 = ((z_{2i} >> 11) + 1) / 2^53, u2 = (z_{2i+1} >> 11) / 2^53.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def splitmix64(seed: int, count: int, start: int = 0) -> np.ndarray:
    """`count` 64-bit outputs of the SplitMix64 stream `seed`, from index `start`."""
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


def uniform_int8(seed: int, shape) -> np.ndarray:
    """iid uniform over [-128, 127]."""
    n = int(np.prod(shape))
    z = splitmix64(seed, n)
    return (z & np.uint64(0xFF)).astype(np.uint8).view(np.int8).reshape(shape)


def normal_int8(seed: int, shape, sigma: float = 32.0) -> np.ndarray:
    """Rounded N(0, sigma^2), clipped to the int8 range (Box-Muller)."""
    n = int(np.prod(shape))
    z = splitmix64(seed, 2 * n)
    u1 = ((z[0::2] >> np.uint64(11)).astype(np.float64) + 1.0) / 9007199254740992.0
    u2 = (z[1::2] >> np.uint64(11)).astype(np.float64) / 9007199254740992.0
    g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    v = np.clip(np.rint(sigma * g), -128, 127)
    return v.astype(np.int8).reshape(shape)


@dataclass(frozen=True)
class ConvShape:
    """conv2d problem: NCHW int8 input, KCRS int8 weights, NKPQ int32 output."""

    name: str
    N: int
    C: int
    H: int
    W: int
    K: int
    R: int
    S: int
    stride: int
    pad: int
    dist: str = "uniform"  # "uniform" | "normal32"
    seed_in: int = 1
    seed_wt: int = 2

    @property
    def P(self) -> int:
        return (self.H + 2 * self.pad - self.R) // self.stride + 1

    @property
    def Q(self) -> int:
        return (self.W + 2 * self.pad - self.S) // self.stride + 1

    @property
    def M(self) -> int:
        return self.N * self.P * self.Q

    @property
    def Kg(self) -> int:
        return self.C * self.R * self.S

    @property
    def macs(self) -> int:
        return self.M * self.K * self.Kg

    @property
    def ops(self) -> int:
        return 2 * self.macs

    @property
    def io_bytes(self) -> int:
        return (self.N * self.C * self.H * self.W + self.K * self.Kg
                + 4 * self.M * self.K)

    def dims(self):
        return (self.N, self.C, self.H, self.W, self.K, self.R, self.S,
                self.stride, self.pad)

    def scaled(self, N: int) -> "ConvShape":
        """Same layer at another batch size (for steady-state measurements)."""
        from dataclasses import replace
        return replace(self, name=f"{self.name}@N{N}", N=N)

    def make(self):
        """(input NCHW int8, weights KCRS int8) for this shape's seeds."""
        ishape = (self.N, self.C, self.H, self.W)
        wshape = (self.K, self.C, self.R, self.S)
        if self.dist == "normal32":
            return normal_int8(self.seed_in, ishape), normal_int8(self.seed_wt, wshape)
        return uniform_int8(self.seed_in, ishape), uniform_int8(self.seed_wt, wshape)


# The five benchmark configurations (the fourth is a pair of independent convs).
CONFIGS = {
    "C1": ConvShape("C1", 1, 16, 14, 14, 16, 3, 3, 1, 1, "uniform", 1001, 2001),
    "C2": ConvShape("C2", 1, 64, 56, 56, 64, 3, 3, 1, 1, "uniform", 1002, 2002),
    "C3": ConvShape("C3", 4, 3, 224, 224, 64, 7, 7, 2, 3, "uniform", 1003, 2003),
    "C4a": ConvShape("C4a", 8, 256, 14, 14, 512, 3, 3, 1, 1, "uniform", 1004, 2004),
    "C4b": ConvShape("C4b", 8, 512, 14, 14, 128, 1, 1, 1, 0, "uniform", 1014, 2014),
    "C5": ConvShape("C5", 4, 1, 161, 500, 32, 20, 5, 2, 0, "normal32", 1005, 2005),
}

# Shapes printed in the paper's Tables 3 and 5 that fit the (square stride/pad,
# dilation 1) operator; used as extra parity shapes.  The tables write the data
# tensor as (n, dim, dim, c); the first spatial extent is taken as H here, except
# for the speech rows where the 20-tap axis runs along the 161 axis as in C5.
PAPER_SHAPES = [
    ConvShape("T3-speech-n1", 1, 1, 161, 700, 32, 20, 5, 2, 0, "normal32", 3001, 4001),
    ConvShape("T3-480x48", 1, 1, 480, 48, 16, 3, 3, 1, 1, "uniform", 3002, 4002),
    ConvShape("T3-108-s2", 1, 3, 108, 108, 64, 3, 3, 2, 1, "uniform", 3003, 4003),
    ConvShape("T3-224-3x3", 1, 3, 224, 224, 64, 3, 3, 1, 1, "uniform", 3004, 4004),
    ConvShape("T3-stem-n1", 1, 3, 224, 224, 64, 7, 7, 2, 3, "uniform", 3005, 4005),
    ConvShape("T3-151x40-p8", 1, 1, 151, 40, 32, 20, 5, 2, 8, "uniform", 3006, 4006),
    ConvShape("T3-5x5-s2", 1, 1, 161, 700, 64, 5, 5, 2, 1, "uniform", 3007, 4007),
    ConvShape("T5-32x8x8", 1, 32, 8, 8, 64, 3, 3, 1, 1, "uniform", 3008, 4008),
    ConvShape("T5-32x32x32", 1, 32, 32, 32, 64, 3, 3, 1, 1, "uniform", 3009, 4009),
    ConvShape("T5-256x8x8", 1, 256, 8, 8, 256, 3, 3, 1, 1, "uniform", 3010, 4010),
    ConvShape("T5-128x16x16", 1, 128, 16, 16, 256, 3, 3, 1, 1, "uniform", 3011, 4011),
    ConvShape("T5-72x56-1x1", 1, 72, 56, 56, 96, 1, 1, 1, 0, "uniform", 3012, 4012),
    ConvShape("T5-256x7-1x1", 1, 256, 7, 7, 512, 1, 1, 1, 0, "uniform", 3013, 4013),
    ConvShape("T5-8x224-s2", 1, 8, 224, 224, 24, 3, 3, 2, 1, "uniform", 3014, 4014),
    ConvShape("T5-72x56-s2", 1, 72, 56, 56, 96, 3, 3, 2, 1, "uniform", 3015, 4015),
]
