"""Seeded synthetic input generator (host side, numpy).

A counter-based generator: every element of every tensor is a pure function of
(seed, stream, index), so the host and the device (gen.hip, same integer
recipe) produce identical bits without shipping data, and any window of a
64 GB tensor can be regenerated on the host.

This module holds none of the method's arithmetic: it only draws numbers.

Recipe
------
word(seed, stream, index, w) is a 32-bit hash (two rounds of a multiply /
xor-shift finaliser over the 64-bit counter 4*index + w).
* uniform u in [0,1): top 24 bits of word 0 times 2^-24 (exact in fp32).
* normal z: the eight 16-bit halves of words 0..3 are summed as integers
  (Irwin-Hall, n = 8), centred and scaled to unit variance with ONE fp32
  multiply.  Integer sum -> fp32 is exact, so z is bit-reproducible on any
  IEEE machine.  |z| <= 4.9; excess kurtosis -0.15: "N(0,1)" for the
  purposes of shaping inputs, not for statistics.
* value = fl(mean + fl(std * z)) in fp32 (two separately rounded operations).
* bf16 tensors: the fp32 value rounded to nearest-even to 16 bits.
"""
import numpy as np

_M1 = np.uint32(0x7FEB352D)
_M2 = np.uint32(0x846CA68B)
_GOLD = np.uint32(0x9E3779B9)
_SALT = np.uint32(0x68E31DA4)

# 1 / sqrt(8 * (2^32 - 1) / 12): unit-variance scale of the centred sum of
# eight independent uniform integers in [0, 65535].
NORMAL_SCALE = np.float32(1.0 / np.sqrt(8.0 * (2.0**32 - 1.0) / 12.0))
_CENTRE = 8 * 65535 // 2  # 262140, exact (8*65535 is even)


def _mix32(x):
    x = x ^ (x >> np.uint32(16))
    x = x * _M1
    x = x ^ (x >> np.uint32(15))
    x = x * _M2
    x = x ^ (x >> np.uint32(16))
    return x


def _key(seed, stream):
    with np.errstate(over="ignore"):
        k = _mix32(np.array([np.uint32(seed & 0xFFFFFFFF) + _GOLD], dtype=np.uint32))
        k = _mix32(k ^ np.uint32(stream & 0xFFFFFFFF))
    return k[0]


def _words(seed, stream, index, w):
    """32-bit hash word w (0..3) for each 64-bit element index."""
    key = _key(seed, stream)
    ctr = index.astype(np.uint64) * np.uint64(4) + np.uint64(w)
    lo = (ctr & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    hi = (ctr >> np.uint64(32)).astype(np.uint32)
    with np.errstate(over="ignore"):
        h = _mix32(lo + key)
        h = _mix32(h ^ hi ^ _SALT)
    return h


def _index(n, offset):
    return np.arange(offset, offset + n, dtype=np.uint64)


def standard_normal_at(seed, stream, index):
    """fp32 z values for arbitrary element indices (uint64 array)."""
    index = np.asarray(index, dtype=np.uint64)
    acc = np.zeros(index.shape, dtype=np.int64)
    for w in range(4):
        h = _words(seed, stream, index, w)
        acc += (h & np.uint32(0xFFFF)).astype(np.int64)
        acc += (h >> np.uint32(16)).astype(np.int64)
    return (acc - _CENTRE).astype(np.float32) * NORMAL_SCALE


def normal_f32(seed, stream, n, mean=0.0, std=1.0, offset=0):
    """n fp32 values mean + std*z for element indices offset..offset+n-1."""
    z = standard_normal_at(seed, stream, _index(n, offset))
    v = z * np.float32(std)
    v = v + np.float32(mean)
    return v.astype(np.float32)


def normal_f32_at(seed, stream, index, mean=0.0, std=1.0):
    z = standard_normal_at(seed, stream, index)
    v = z * np.float32(std)
    v = v + np.float32(mean)
    return v.astype(np.float32)


def uniform_f32(seed, stream, n, lo=0.0, hi=1.0, offset=0):
    """n fp32 values lo + (hi-lo)*u, u = 24-bit uniform in [0,1)."""
    h = _words(seed, stream, _index(n, offset), 0)
    u = (h >> np.uint32(8)).astype(np.float32) * np.float32(2.0**-24)
    v = u * (np.float32(hi) - np.float32(lo))
    v = v + np.float32(lo)
    return v.astype(np.float32)


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    with np.errstate(over="ignore"):
        r = (b + rnd) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def normal_bf16_bits(seed, stream, n, mean=0.0, std=1.0, offset=0):
    return f32_to_bf16_bits(normal_f32(seed, stream, n, mean, std, offset))
