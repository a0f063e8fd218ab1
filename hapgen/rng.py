"""Counter-based N(0, sigma) generator and bf16 helpers.

Element k of tensor t under seed s is a pure function of (s, t, k): a
splitmix64 finaliser over the packed counter gives two 64-bit words, their top
53 bits give two uniforms, and a Box-Muller transform gives one normal.  The
value does not depend on generation order, chunking or thread count, so any
slice of a tensor can be regenerated on its own.
"""
from __future__ import annotations

import enum
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


class TensorId(enum.IntEnum):
    """Stream ids: one per named tensor so tensors never share counters."""
    X = 1
    W = 2
    DY = 3
    BIAS = 4
    W2 = 5
    BIAS2 = 6
    WQ = 7
    WK = 8
    WV = 9
    WO = 10
    Q = 11
    K = 12
    V = 13
    DO = 14
    GAMMA = 15
    BETA = 16
    SFB_X = 32     # + device index
    SFB_DY = 64    # + device index
    MISC = 128


def _mix(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def _uniform_pair(seed: int, tensor: int, start: int, count: int):
    with np.errstate(over="ignore"):
        k = np.arange(start, start + count, dtype=np.uint64)
        base = np.uint64((seed * 0x100000001B3 + tensor * 0x9E3779B1) & 0xFFFFFFFFFFFFFFFF)
        c = (k * np.uint64(2) + base) * _GOLDEN
        a = _mix(c + _GOLDEN)
        b = _mix(c + _GOLDEN + _GOLDEN)
    inv = 1.0 / float(1 << 53)
    u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * inv      # (0, 1]
    u2 = (b >> np.uint64(11)).astype(np.float64) * inv              # [0, 1)
    return u1, u2


def normal(seed: int, tensor: int, shape, sigma: float = 1.0, dtype=np.float64) -> np.ndarray:
    """N(0, sigma^2) samples of the given shape, element k drawn from counter k."""
    n = int(np.prod(shape)) if len(tuple(shape)) else 1
    out = np.empty(n, dtype=dtype)

    def fill(s):
        c = min(_CHUNK, n - s)
        u1, u2 = _uniform_pair(seed, int(tensor), s, c)
        out[s:s + c] = (np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2) * sigma).astype(dtype)

    starts = range(0, n, _CHUNK)
    if len(starts) > 1:     # chunks are independent (counter-based), so threads only change the wall time
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, starts))
    else:
        for s in starts:
            fill(s)
    return out.reshape(shape)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def from_bf16_bits(bits: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns to float32 exactly."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16(seed: int, tensor: int, shape, sigma: float = 1.0):
    """Samples snapped to the bf16 grid.  Returns (float32 values, uint16 bit patterns)."""
    bits = to_bf16_bits(normal(seed, tensor, shape, sigma, dtype=np.float32))
    return from_bf16_bits(bits), bits
