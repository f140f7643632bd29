"""Pins for the oracle's binary16 helpers: the IEEE 754 format definition,
written here with Python integers/fractions, and numpy's own conversion as a
library cross-check."""
from fractions import Fraction

import numpy as np

import oracle


def _exact_value(bits):
    """binary16 value as an exact Fraction, straight from the format."""
    sign = -1 if bits >> 15 else 1
    e = (bits >> 10) & 0x1F
    f = bits & 0x3FF
    if e == 31:
        return None
    if e == 0:
        return sign * Fraction(f, 1 << 24)
    return sign * Fraction(1024 + f, 1024) * Fraction(2) ** (e - 15)


def test_decode_every_bit_pattern():
    L = oracle.lib()
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = allbits.view(np.float16).astype(np.float64)
    for b in range(65536):
        v = L.oracle_f16_to_double(b)
        ex = _exact_value(b)
        if ex is None:
            if b & 0x3FF:
                assert v != v
            else:
                assert v == (float("-inf") if b >> 15 else float("inf"))
            continue
        assert Fraction(v) == ex, hex(b)
        assert v == ref[b] and np.signbit(v) == np.signbit(ref[b])


def test_encode_round_trip_every_finite_pattern():
    L = oracle.lib()
    for b in range(65536):
        if (b & 0x7C00) == 0x7C00 and (b & 0x3FF):
            continue  # NaN payloads are not preserved
        assert L.oracle_double_to_f16(L.oracle_f16_to_double(b)) == b, hex(b)


def test_encode_midpoints_go_to_even_and_neighbours_round_correctly():
    L = oracle.lib()
    for b in range(0, 0x7BFF):  # positive finite, b+1 also finite
        lo, hi = L.oracle_f16_to_double(b), L.oracle_f16_to_double(b + 1)
        mid = (lo + hi) / 2  # exact in double
        even = b if b % 2 == 0 else b + 1
        assert L.oracle_double_to_f16(mid) == even
        assert L.oracle_double_to_f16(-mid) == (even | 0x8000)
        assert L.oracle_double_to_f16(np.nextafter(mid, 0.0)) == b
        assert L.oracle_double_to_f16(np.nextafter(mid, 1e9)) == b + 1


def test_encode_overflow_and_underflow():
    L = oracle.lib()
    assert L.oracle_double_to_f16(65504.0) == 0x7BFF
    assert L.oracle_double_to_f16(65519.999) == 0x7BFF
    assert L.oracle_double_to_f16(65520.0) == 0x7C00  # tie goes to "even" = infinity
    assert L.oracle_double_to_f16(-1e9) == 0xFC00
    assert L.oracle_double_to_f16(2.0 ** -25) == 0  # tie to even (zero)
    assert L.oracle_double_to_f16(np.nextafter(2.0 ** -25, 1.0)) == 1
    assert L.oracle_double_to_f16(-0.0) == 0x8000


def test_encode_matches_numpy_on_random_doubles():
    L = oracle.lib()
    rng = np.random.default_rng(11)
    vals = np.concatenate([rng.standard_normal(20000) * s for s in (1e-7, 1e-4, 1.0, 50.0, 3e4)])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    for v, r in zip(vals, ref):
        assert L.oracle_double_to_f16(float(v)) == int(r)
