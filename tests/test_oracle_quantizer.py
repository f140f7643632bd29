"""Pins for the absmax quantizer Q (Section 2.1) as the oracle applies it per
row (Section 3.1): rounding to the nearest integer, ties to even, of the exact
rational 127*x/c.  The reference here is pure integer arithmetic: every finite
fp16 is an integer multiple of 2^-24."""
import numpy as np

import oracle


def _as_int(bits):
    """fp16 bit patterns -> value * 2^24 as int64 (exact)."""
    bits = bits.astype(np.int64)
    e = (bits >> 10) & 0x1F
    f = bits & 0x3FF
    mag = np.where(e == 0, f, (1024 + f) << np.maximum(e - 1, 0))
    return np.where(bits >> 15 != 0, -mag, mag)


def _q_integer(xb, cb):
    """Round-half-even of 127*x/c by integer floor division and remainder."""
    X = _as_int(xb)
    Cc = _as_int(cb)
    sign = np.sign(X)
    num = 127 * np.abs(X)
    safe = np.where(Cc == 0, 1, Cc)
    q = num // safe
    r = num - q * safe
    up = (2 * r > safe) | ((2 * r == safe) & (q % 2 == 1))
    q = np.where(Cc == 0, 0, q + up)
    return (sign * q).astype(np.int64), (2 * r == safe) & (Cc != 0)


def _sweep(c_bits, x_max_bits, negate):
    """Row i holds c_bits[i] first, then every non-negative pattern <= it
    (zero padded), so the row constant is c_bits[i]."""
    s = len(c_bits)
    h = int(x_max_bits) + 2
    cols = np.arange(h - 1, dtype=np.int64)
    X = np.zeros((s, h), dtype=np.uint16)
    X[:, 0] = c_bits
    body = np.where(cols[None, :] <= c_bits[:, None].astype(np.int64), cols[None, :], 0)
    X[:, 1:] = body.astype(np.uint16)
    if negate:
        X[:, 1:] |= 0x8000
    Xq, cx = oracle.quantize_rows(X, np.zeros(0, np.int32))
    assert np.array_equal(cx.view(np.uint16), c_bits.astype(np.uint16))
    ref, ties = _q_integer(X, np.broadcast_to(c_bits[:, None], X.shape))
    assert np.array_equal(Xq.astype(np.int64), ref)
    return int(ties.sum())


def test_q_exhaustive_over_one_binade_of_constants():
    # constants 1.0 .. 1.999 (all 1024 mantissas), every |x| <= c, both signs
    c = np.arange(0x3C00, 0x4000, dtype=np.int64)
    ties = _sweep(c, 0x3FFF, False)
    ties += _sweep(c, 0x3FFF, True)
    assert ties > 1000  # the tie rule is exercised


def test_q_typical_row_constants_and_top_binade():
    # 4.0 .. 7.99: where row constants of N(0,1) data live
    assert _sweep(np.arange(0x4400, 0x4800, dtype=np.int64), 0x47FF, True) > 500
    # 32768 .. 65504: largest finite constants, x over the whole finite range
    assert _sweep(np.arange(0x7800, 0x7C00, 8, dtype=np.int64), 0x7BFF, False) > 50


def test_q_subnormal_constants():
    c = np.arange(1, 0x0400, dtype=np.int64)  # every subnormal constant
    _sweep(c, 0x03FF, False)
    _sweep(c, 0x03FF, True)
    c = np.arange(0x0400, 0x0800, dtype=np.int64)  # smallest normal binade
    _sweep(c, 0x07FF, False)


def test_q_scalar_special_values():
    assert oracle.q(0.0, 0.0) == 0
    assert oracle.q(0.0, 3.0) == 0
    for c in (2.0 ** -24, 0.1240234375, 1.0, 5.3984375, 65504.0):
        assert oracle.q(c, c) == 127 and oracle.q(-c, c) == -127
    # constructed ties: c = 1270 * 2^e, x = 5 * k * 2^e  =>  127 x / c = k / 2
    for e in (-8, -3, 0, 2):
        c = 1270.0 * 2.0 ** e
        for k, want in ((1, 0), (3, 2), (5, 2), (7, 4), (253, 126), (-3, -2), (-5, -2), (-253, -126)):
            assert oracle.q(5.0 * k * 2.0 ** e, c) == want


def test_row_constant_is_max_over_non_outlier_columns_and_maps_to_127():
    rng = np.random.default_rng(3)
    X = rng.standard_normal((37, 300)).astype(np.float16)
    X[::3, 5] = 40.0
    X[1::2, 123] = -17.0
    idx = oracle.find_outliers(X, 6.0)
    assert idx.tolist() == [5, 123]
    Xq, cx = oracle.quantize_rows(X, idx)
    keep = np.ones(300, bool)
    keep[idx] = False
    a = np.abs(X.astype(np.float64))
    assert np.array_equal(cx.astype(np.float64), a[:, keep].max(axis=1))
    assert np.all(cx.astype(np.float64) < 6.0)
    assert np.all(Xq[:, idx] == 0)
    # the absmax element of each row is coded +-127, nothing exceeds 127
    pos = np.where(keep)[0][a[:, keep].argmax(axis=1)]
    assert np.all(np.abs(Xq[np.arange(37), pos]) == 127)
    assert Xq.min() >= -127 and Xq.max() <= 127
    # signs survive
    nz = Xq != 0
    assert np.all(np.sign(Xq[nz]) == np.sign(X.astype(np.float64)[nz]))


def test_zero_rows_and_zero_columns_quantize_to_zero():
    X = np.zeros((3, 16), np.float16)
    X[1, :] = 1.5
    Xq, cx = oracle.quantize_rows(X, np.zeros(0, np.int32))
    assert cx.tolist() == [0.0, 1.5, 0.0] and np.all(Xq[0] == 0) and np.all(Xq[1] == 127)
    W = np.zeros((16, 4), np.float16)
    W[:, 2] = -0.25
    Wq, cw = oracle.quantize_weight(W)
    assert cw.tolist() == [0.0, 0.0, 0.25, 0.0] and np.all(Wq[:, 2] == -127) and np.all(Wq[:, [0, 1, 3]] == 0)


def test_half_step_bound_on_dequantized_values():
    # rounding to nearest => |x - q c / 127| <= c / 254 for every coded element
    rng = np.random.default_rng(5)
    X = (rng.standard_normal((64, 512)) * 1.3).astype(np.float16)
    Xq, cx = oracle.quantize_rows(X, np.zeros(0, np.int32))
    x = X.astype(np.float64)
    c = cx.astype(np.float64)[:, None]
    err = np.abs(x - Xq.astype(np.float64) * c / 127.0)
    assert np.all(err <= c / 254.0 * (1 + 1e-12))
    W = (rng.standard_normal((512, 48)) * 0.02).astype(np.float16)
    Wq, cw = oracle.quantize_weight(W)
    c = cw.astype(np.float64)[None, :]
    err = np.abs(W.astype(np.float64) - Wq.astype(np.float64) * c / 127.0)
    assert np.all(err <= c / 254.0 * (1 + 1e-12))


def test_weight_constant_is_column_max_over_all_rows():
    rng = np.random.default_rng(6)
    W = (rng.standard_normal((130, 70)) * 0.02).astype(np.float16)
    Wq, cw = oracle.quantize_weight(W)
    assert np.array_equal(cw.astype(np.float64), np.abs(W.astype(np.float64)).max(axis=0))
    ref, _ = _q_integer(W.view(np.uint16), np.broadcast_to(cw.view(np.uint16)[None, :], W.shape))
    assert np.array_equal(Wq.astype(np.int64), ref)
