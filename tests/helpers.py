"""Small independent reference routines used only by the tests (numpy / Python integers)."""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def half_to_fraction(h: int) -> Fraction:
    """Exact value of a finite fp16 bit pattern."""
    sign = -1 if (h & 0x8000) else 1
    e = (h >> 10) & 0x1F
    m = h & 0x3FF
    assert e != 31
    if e == 0:
        return sign * Fraction(m, 1 << 24)
    return sign * Fraction((m | 0x400) << e, 1 << 25) if e < 25 else sign * Fraction((m | 0x400) * (1 << (e - 25)))


def round_fraction_to_half(v: Fraction) -> int:
    """Round an exact rational to fp16, nearest-even, from the definition of the format."""
    sign = 0x8000 if v < 0 else 0
    a = abs(v)
    if a == 0:
        return sign
    # exponent e with 2^e <= a < 2^(e+1), clamped to the subnormal range
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -14)
    ulp = Fraction(2) ** (e - 10)
    q = a / ulp
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    # n in [0, 2048]; compose bits: value = n * 2^(e-10)
    if e == -14 and n < 1024:
        return sign | n  # subnormal
    if n == 2048:
        n = 1024
        e += 1
    if e > 15:
        return sign | 0x7C00
    return sign | ((e + 15) << 10) | (n - 1024)


def stream_bits(block_u8: np.ndarray) -> np.ndarray:
    """512 stream bits of one 64-byte block: 16 little-endian words, most significant bit of each first."""
    words = np.asarray(block_u8, np.uint8).view("<u4")
    return ((words[:, None] >> np.arange(31, -1, -1, dtype=np.uint32)[None, :]) & 1).astype(np.uint8).reshape(-1)


def pack_raw(idx: np.ndarray) -> np.ndarray:
    """Raw-mode payload of 128 indices: value i in stream bits 4i..4i+3, top bit first."""
    idx = np.asarray(idx, np.uint32).reshape(16, 8)
    words = np.zeros(16, np.uint32)
    for j in range(8):
        words |= idx[:, j] << np.uint32(28 - 4 * j)
    return words.astype("<u4").view(np.uint8)


def py_canonical(lens):
    """Canonical codes by the textbook recipe, independently of the oracle."""
    order = sorted(range(len(lens)), key=lambda k: (lens[k], k))
    codes = [0] * len(lens)
    code = 0
    for j, k in enumerate(order):
        if j:
            code = (code + 1) << (lens[k] - lens[order[j - 1]])
        codes[k] = code
    return codes
