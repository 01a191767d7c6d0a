"""Seeded synthetic input generators shared by the CPU oracle's tests and the HIP path's tests.

This module holds none of the method's arithmetic: it only produces raw values (floats, integer codes,
+-1 entries, thresholds) from a counter-based generator, so that both sides can be fed identical inputs
without sharing any code that binarizes, packs, multiplies or thresholds.

Generator: element i of stream s under seed z is  mix(key(z, s) + (i + 1) * GAMMA)  where mix is the
64-bit finalizer of the public-domain SplitMix64 generator and key(z, s) = mix(z * GAMMA + s).
It is frozen: changing it changes every stored expectation.
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 160907061
_GAMMA = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_CHUNK = 1 << 22


def _mix(z: np.ndarray) -> np.ndarray:
    z = z.astype(np.uint64, copy=True)
    z ^= z >> np.uint64(30)
    z *= _M1
    z ^= z >> np.uint64(27)
    z *= _M2
    z ^= z >> np.uint64(31)
    return z


def _key(seed: int, stream: int) -> np.uint64:
    with np.errstate(over="ignore"):
        k = np.array([np.uint64(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64) * _GAMMA + np.uint64(stream)
        return _mix(k)[0]


def raw_u64(seed: int, stream: int, n: int, offset: int = 0) -> np.ndarray:
    """n raw 64-bit values, elements offset .. offset+n-1 of the stream."""
    key = _key(seed, stream)
    out = np.empty(n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        for lo in range(0, n, _CHUNK):
            hi = min(n, lo + _CHUNK)
            idx = np.arange(offset + lo + 1, offset + hi + 1, dtype=np.uint64)
            out[lo:hi] = _mix(key + idx * _GAMMA)
    return out


def _count(shape) -> int:
    n = 1
    for d in shape:
        n *= int(d)
    return n


def bernoulli_bits(seed: int, stream: int, shape) -> np.ndarray:
    """i.i.d. fair bits as uint8 in {0,1}; element i is bit (i % 64) of raw value i // 64."""
    n = _count(shape)
    words = raw_u64(seed, stream, (n + 63) // 64)
    bits = np.unpackbits(words.view(np.uint8), bitorder="little")[:n]
    return bits.reshape(shape)


def pm1(seed: int, stream: int, shape) -> np.ndarray:
    """i.i.d. entries in {-1,+1} with probability 1/2 each, as int8 (fair bit 1 -> +1)."""
    b = bernoulli_bits(seed, stream, shape).astype(np.int8)
    return (2 * b - 1).astype(np.int8)


def uniform_int(seed: int, stream: int, shape, lo: int, hi: int, dtype=np.int32) -> np.ndarray:
    """i.i.d. integers uniform on [lo, hi] inclusive (top 32 bits of the raw value scaled to the range)."""
    n = _count(shape)
    span = np.uint64(hi - lo + 1)
    r = raw_u64(seed, stream, n) >> np.uint64(32)
    v = ((r * span) >> np.uint64(32)).astype(np.int64) + lo
    return v.astype(dtype).reshape(shape)


def normal_f32(seed: int, stream: int, shape) -> np.ndarray:
    """i.i.d. N(0,1) by Box-Muller in double precision, rounded to float32."""
    n = _count(shape)
    m = (n + 1) // 2
    r = raw_u64(seed, stream, 2 * m)
    u1 = ((r[:m] >> np.uint64(11)).astype(np.float64) + 1.0) * (1.0 / 9007199254740992.0)  # (0, 1]
    u2 = (r[m:] >> np.uint64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)  # [0, 1)
    rad = np.sqrt(-2.0 * np.log(u1))
    z = np.concatenate([rad * np.cos(2.0 * np.pi * u2), rad * np.sin(2.0 * np.pi * u2)])[:n]
    return z.astype(np.float32).reshape(shape)


def special_floats() -> np.ndarray:
    """The float32 edge values every binarizer has to get right (zeros, denormals, infinities, NaNs)."""
    bits = np.array(
        [
            0x00000000,  # +0.0
            0x80000000,  # -0.0
            0x00000001,  # smallest positive denormal
            0x80000001,  # smallest negative denormal
            0x007FFFFF,  # largest positive denormal
            0x807FFFFF,  # largest negative denormal
            0x00800000,  # +FLT_MIN
            0x80800000,  # -FLT_MIN
            0x7F800000,  # +inf
            0xFF800000,  # -inf
            0x7FC00000,  # quiet NaN, sign clear
            0xFFC00000,  # quiet NaN, sign set
            0x7F800001,  # signalling NaN, sign clear
            0x3F800000,  # +1.0
            0xBF800000,  # -1.0
            0x7F7FFFFF,  # +FLT_MAX
            0xFF7FFFFF,  # -FLT_MAX
        ],
        dtype=np.uint32,
    )
    return bits.view(np.float32)


def with_special_floats(x: np.ndarray, seed: int, stream: int) -> np.ndarray:
    """Copy of float32 array x with the edge values planted at seeded positions (and at both ends)."""
    y = x.copy().reshape(-1)
    sp = special_floats()
    n = y.size
    if n == 0:
        return x.copy()
    pos = (raw_u64(seed, stream, 4 * sp.size) % np.uint64(n)).astype(np.int64)
    for i, p in enumerate(pos):
        y[p] = sp[i % sp.size]
    y[0] = sp[1]
    y[-1] = sp[11]
    return y.reshape(x.shape)
