"""Oracle of the 8-bit KV-cache format: TEST INFRASTRUCTURE, not a product path.

The paper names KV-cache quantisation as the next step of the method (its Future Work section) without fixing a
format.  This build takes the OCP 8-bit floating point format E4M3 ("e4m3fn": 1 sign, 4 exponent, 3 mantissa
bits, bias 7, no infinities, the all-ones pattern S.1111.111 is NaN, largest finite value 448) with one scale per
tensor kind.  The paper leaves the quantisation step open as well; the reading taken (and documented as the
storage contract in the library's public header) is
    code = nearest E4M3 value, ties to even, saturated to +-448, of  y = fl32(x * fl32(1 / scale)),
i.e. the scale is applied as ONE float32 reciprocal and ONE float32 product, each rounded once, and value =
decode(code) * scale.  The other natural reading, the exactly divided x / scale, differs from it only where x / scale
falls on (or within a float32 rounding of) the midpoint of two codes; ``quantize_bf16_bits_exact_division`` implements
that reading so that a test can show where the two part and that the choice is a choice.  Everything here is written out from that definition with Python integers and exact rationals; only ``tests/`` may
import it.  **parity unpinned** against the paper (it gives no format); pinned against the format's published
constants, its own inverse, exact midpoints and an independent library conversion in ``tests/test_fp8.py``.
"""
from __future__ import annotations

from fractions import Fraction as F
from typing import List

import numpy as np

BIAS = 7
MAX_FINITE = 448
NAN_CODE = 0x7F


def decode_one(code: int) -> F | None:
    """Exact value of one code; None for the two NaN patterns."""
    s, e, m = code >> 7, (code >> 3) & 0xF, code & 7
    if e == 0xF and m == 7:
        return None
    mag = F(m, 8) * F(2) ** (1 - BIAS) if e == 0 else (1 + F(m, 8)) * F(2) ** (e - BIAS)
    return -mag if s else mag


# the 127 non-negative finite values in code order (code i -> POSITIVE[i]); strictly increasing
POSITIVE: List[F] = [decode_one(c) for c in range(0x7F)]


def encode_one(x: F) -> int:
    """Nearest code of an exact rational, ties to the code with an even mantissa bit, saturating."""
    s = 0x80 if x < 0 else 0
    a = -x if x < 0 else x
    if a >= MAX_FINITE:
        return s | 0x7E
    lo = 0
    for i, v in enumerate(POSITIVE):          # plain search: the largest value <= a
        if v <= a:
            lo = i
    hi = lo + 1                                # hi <= 0x7E because a < 448
    d_lo, d_hi = a - POSITIVE[lo], POSITIVE[hi] - a
    if d_lo < d_hi or (d_lo == d_hi and lo % 2 == 0):
        return s | lo
    return s | hi


def decode(codes: np.ndarray) -> np.ndarray:
    """uint8 codes -> float32 values (exact: every E4M3 value is a float32); NaN codes give NaN."""
    table = np.array([float("nan") if decode_one(c) is None else float(decode_one(c)) for c in range(256)],
                     dtype=np.float32)
    return table[np.ascontiguousarray(codes, dtype=np.uint8)]


def encode(x: np.ndarray) -> np.ndarray:
    """float32 values -> uint8 codes, element by element through encode_one; NaN gives the NaN code (sign kept)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    patterns, where = np.unique(x.reshape(-1).view(np.uint32), return_inverse=True)   # one decision per bit pattern
    codes = np.empty(len(patterns), dtype=np.uint8)
    for i, v in enumerate(patterns.view(np.float32)):
        if np.isnan(v):
            c = NAN_CODE | (0x80 if np.signbit(v) else 0)
        elif np.isinf(v):
            c = (0x80 if v < 0 else 0) | 0x7E
        else:
            c = encode_one(F(float(v)))
            if v == 0 and np.signbit(v):
                c |= 0x80
        codes[i] = c
    return codes[where].reshape(x.shape)


def quantize_bf16_bits(bits: np.ndarray, scale: float) -> np.ndarray:
    """The storage contract: bf16 bit patterns -> codes of y = fl32(x * inv) with inv = fl32(1 / fl32(scale)), both
    roundings to float32 nearest-even; the code is then decided exactly (``encode``)."""
    x = (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    inv = np.float32(1.0) / np.float32(scale)
    with np.errstate(invalid="ignore", over="ignore"):   # NaN and infinite inputs are part of the domain
        y = (x * inv).astype(np.float32)
    return encode(y)


def quantize_bf16_bits_exact_division(bits: np.ndarray, scale: float) -> np.ndarray:
    """The reading NOT taken: codes of the exact quotient x / fl32(scale) (rational arithmetic, no intermediate
    rounding).  Finite inputs only; kept to show where the two readings differ."""
    x = (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    sc = F(float(np.float32(scale)))
    out = np.empty(x.shape, dtype=np.uint8)
    flat = out.reshape(-1)
    for i, v in enumerate(x.reshape(-1)):
        c = encode_one(F(float(v)) / sc)
        if v == 0 and np.signbit(v):
            c |= 0x80
        flat[i] = c
    return out
