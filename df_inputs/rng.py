"""Counter-based seeded generator and bf16 bit conversion.

Every tensor is keyed by (seed, name): the Philox key is built from the seed
and a CRC of the name, so a tensor's values do not depend on the order in
which tensors are drawn, and both consumers read identical values.
"""
import zlib

import numpy as np

_MASK64 = (1 << 64) - 1


def _generator(seed, name):
    tag = zlib.crc32(name.encode("utf-8")) | (len(name) << 32)
    return np.random.Generator(np.random.Philox(key=[int(seed) & _MASK64, tag & _MASK64]))


def normal(seed, name, shape, std=1.0, mean=0.0):
    """float32 tensor of N(mean, std^2) values keyed by (seed, name)."""
    g = _generator(seed, name)
    x = g.standard_normal(size=tuple(int(s) for s in shape), dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return x


def to_bf16_bits(x):
    """float32 -> uint16 bfloat16 bit patterns, round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = ((u + bias) >> np.uint32(16)).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r[nan] = np.uint16(0x7FC0)
    return r


def from_bf16_bits(b):
    """uint16 bfloat16 bit patterns -> float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(x):
    """float32 -> float32 holding the nearest bfloat16 value."""
    return from_bf16_bits(to_bf16_bits(x))
