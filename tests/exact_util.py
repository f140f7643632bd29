"""Exact rational arithmetic on fp16 values, for tests that check the oracle by brute force."""
import bisect
from fractions import Fraction

import numpy as np


def f16_fraction(b):
    """Exact value of a finite fp16 bit pattern."""
    b = int(b)
    sign = -1 if b >> 15 else 1
    e, f = (b >> 10) & 0x1f, b & 0x3ff
    return sign * (Fraction(f, 1 << 24) if e == 0 else Fraction(1024 + f, 1) * Fraction(2) ** (e - 25))


_VALS = None


def nearest_f16(x):
    """Brute force: the finite fp16 nearest to the exact rational x, ties to even mantissa."""
    global _VALS
    if _VALS is None:
        _VALS = [f16_fraction(c) for c in range(0x7c00)]  # ascending magnitudes
    ax = abs(x)
    i = bisect.bisect_left(_VALS, ax)
    best = None
    for c in (i - 1, i):
        if 0 <= c < len(_VALS):
            d = abs(_VALS[c] - ax)
            if best is None or d < best[0] or (d == best[0] and c % 2 == 0):
                best = (d, c)
    return np.uint16(best[1] | (0x8000 if x < 0 else 0))
