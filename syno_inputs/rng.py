"""Seeded synthetic tensors.

The generator is counter based: draw number i of stream `seed` is the
SplitMix64 output function applied to seed + (i+1)*gamma, so any slice of a
stream can be produced independently and the arrays do not depend on numpy's
own generators.  Normal deviates come from the Box-Muller transform of two
consecutive draws.  A `Stream` hands out consecutive slices, so tensors that
share a seed are drawn one after the other from the same stream.

Nothing here belongs to the operator arithmetic; the arrays produced are the
common inputs of the CPU checker and of the GPU library.
"""
from __future__ import annotations

import numpy as np

_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def _splitmix64(seed: int, start: int, count: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        idx = np.arange(start + 1, start + count + 1, dtype=np.uint64)
        z = np.uint64(seed & 0xFFFFFFFFFFFFFFFF) + idx * _GAMMA
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        z = z ^ (z >> np.uint64(31))
    return z


class Stream:
    def __init__(self, seed: int):
        self.seed = int(seed)
        self.pos = 0

    def _bits(self, count: int) -> np.ndarray:
        z = _splitmix64(self.seed, self.pos, count)
        self.pos += count
        return z

    def uniform01(self, count: int) -> np.ndarray:
        """count doubles, uniform on [0, 1) with 53 random bits."""
        return (self._bits(count) >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)

    def normal(self, shape) -> np.ndarray:
        """N(0,1) as float32, shape `shape`."""
        n = int(np.prod(shape))
        u = self.uniform01(2 * n)
        u1 = 1.0 - u[0::2]          # (0, 1]
        u2 = u[1::2]
        g = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
        return g.astype(np.float32).reshape(shape)

    def uniform_pm(self, a: float, shape) -> np.ndarray:
        """Uniform on [-a, a) as float32."""
        n = int(np.prod(shape))
        u = self.uniform01(n)
        return ((2.0 * u - 1.0) * a).astype(np.float32).reshape(shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns the uint16 patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    with np.errstate(over="ignore"):
        r = (b + bias) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 patterns to float32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
