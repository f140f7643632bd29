"""Pins of the oracle's zeropoint variant (Section 2.1, Eq. 1-5, applied per row of X and per column
of W; Table 1 "zeropoint vector-wise" and, with the decomposition, "Zeropoint LLM.int8()").

Expected values come from exact rational arithmetic written out here, from the identity of Eq. 4 and
Eq. 5, from the absmax oracle (already pinned) on ranges symmetric about zero, where both
quantizers are the same function, and from inputs on an integer grid whose codes are known."""
from fractions import Fraction

import numpy as np
import pytest

from exact_util import f16_fraction, nearest_f16
from paper_2208_07339_amd import workloads as wl


def rne(fr):
    return round(fr)  # Fraction.__round__: nearest integer, ties to even


def exact_vector(vals):
    """lo, hi, zp and codes of one vector of Fractions, from Eq. 1-3."""
    if not vals:
        return Fraction(0), Fraction(0), 0, []
    lo, hi = min(vals), max(vals)
    D = hi - lo
    if D == 0:
        return lo, hi, 0, [0] * len(vals)
    u = [rne(254 * v / D) for v in vals]
    zp = rne(254 * lo / D) + 127
    return lo, hi, zp, [x - zp for x in u]


def exact_zp_linear(X, W, alpha):
    s, h = X.shape
    o = W.shape[1]
    xf = [[f16_fraction(b) for b in row] for row in X.view(np.uint16)]
    wf = [[f16_fraction(b) for b in row] for row in W.view(np.uint16)]
    O = [j for j in range(h) if np.isfinite(alpha) and any(abs(xf[i][j]) >= Fraction(alpha) for i in range(s))]
    keep = [j for j in range(h) if j not in O]
    rows = [exact_vector([xf[i][j] for j in keep]) for i in range(s)]
    cols = [exact_vector([wf[k][j] for k in range(h)]) for j in range(o)]
    Xq = np.zeros((s, h), np.int64)
    for i in range(s):
        Xq[i, keep] = rows[i][3]
    Wq = np.array([c[3] for c in cols], np.int64).T.reshape(h, o)
    T = [[sum((int(Xq[i, k]) + rows[i][2]) * (int(Wq[k, j]) + cols[j][2]) for k in keep) for j in range(o)]
         for i in range(s)]
    Out = [[nearest_f16(T[i][j] * (rows[i][1] - rows[i][0]) * (cols[j][1] - cols[j][0]) / 64516
                        + sum(xf[i][k] * wf[k][j] for k in O)) for j in range(o)] for i in range(s)]
    return O, rows, cols, Xq, Wq, np.array(T, dtype=object), np.array(Out, np.uint16)


def small_case(seed=3):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(6, 14)).astype(np.float16)
    W = (0.05 * rng.normal(size=(14, 5))).astype(np.float16)
    X[0] = np.abs(X[0])                  # one-sided row (the ReLU case of Section 2.1): lo >= 0
    X[1] = X[1] + np.float16(3.0)        # a range far from zero: a large zeropoint
    X[2] = np.float16(0.0)               # constant rows: D = 0
    X[3] = np.float16(1.25)
    X[4, 9], X[5, 9] = 17.0, -40.0       # an outlier column
    W[:, 2] = np.abs(W[:, 2])
    return X, W


@pytest.mark.parametrize("alpha", [6.0, float("inf")])
def test_every_stage_equals_exact_rational_arithmetic(oracle_mod, alpha):
    X, W = small_case()
    O, rows, cols, Xq, Wq, T, Out = exact_zp_linear(X, W, alpha)
    r = oracle_mod.zp_linear(X, W, alpha)
    assert list(r["idx"]) == O
    assert [f16_fraction(b) for b in r["lo_x"].view(np.uint16)] == [q[0] for q in rows]
    assert [f16_fraction(b) for b in r["hi_x"].view(np.uint16)] == [q[1] for q in rows]
    assert [f16_fraction(b) for b in r["lo_w"].view(np.uint16)] == [q[0] for q in cols]
    assert [f16_fraction(b) for b in r["hi_w"].view(np.uint16)] == [q[1] for q in cols]
    assert list(r["zp_x"]) == [q[2] for q in rows] and list(r["zp_w"]) == [q[2] for q in cols]
    assert np.array_equal(r["Xq"], Xq) and np.array_equal(r["Wq"], Wq)
    assert np.array_equal(r["rowsum"], Xq.sum(axis=1)) and np.array_equal(r["colsum"], Wq.sum(axis=0))
    assert np.array_equal(r["C"], Xq @ Wq)
    assert np.array_equal(r["T"].astype(object), T)
    got = r["Out"].view(np.uint16)
    assert ((got == Out) | (((got | Out) & 0x7fff) == 0)).all()
    if alpha == 6.0:
        assert O == [9] and not r["Xq"][:, 9].any()
    assert r["zp_x"][1] > 127 and r["zp_x"][2] == 0 and r["zp_x"][3] == 0  # far-from-zero row; constant rows
    assert r["zp_x"][0] == 127 + rne(254 * rows[0][0] / (rows[0][1] - rows[0][0]))


def test_u_is_the_correctly_rounded_quotient_over_wide_ranges(oracle_mod):
    """nearbyint of the double quotient against exact rationals, also where D needs ~40 bits and where the
    quotient is huge (data far from zero relative to its spread), plus constructed ties."""
    rng = np.random.default_rng(9)
    bits = rng.integers(0, 0x7c00, size=(400, 3)).astype(np.uint16)
    bits[:40, 0] = rng.integers(0x7800, 0x7c00, 40)   # hi near the top of the range ..
    bits[:40, 1] = rng.integers(1, 0x0400, 40)        # .. lo subnormal
    bits[40:80, 1] = bits[40:80, 0] - 1               # lo just below hi: one quantum of spread
    for hb, lb, xb in bits:
        hi, lo, x = f16_fraction(hb), f16_fraction(lb), f16_fraction(xb)
        for sl, sx in ((1, 1), (-1, 1), (-1, -1)):
            l, h_ = sorted((sl * lo, hi))
            D = h_ - l
            if D == 0:
                continue
            got = oracle_mod.zp_u(float(sx * x), float(D))
            assert got == rne(254 * sx * x / D), (hex(hb), hex(lb), hex(xb))
    # constructed ties
    D = Fraction(127, 32)          # = 3.96875, an fp16 value; 254 / D = 64
    for k in (1, 3, 5, -7, 255):   # x = k / 128 -> 64 x = k / 2: a tie for odd k
        x = Fraction(k, 128)
        assert oracle_mod.zp_u(float(x), float(D)) == rne(Fraction(k, 2))
    assert oracle_mod.zp_u(1.0, 0.0) == 0


def test_codes_use_the_full_range_and_stay_within_half_a_step(oracle_mod):
    d = wl.make_custom(48, 160, 64, 3, seed=21)
    X = np.maximum(d["X"], np.float16(0))        # one-sided data, as after a ReLU
    X[:, d["planted"]] = d["X"][:, d["planted"]]
    W = d["W"]
    idx = oracle_mod.find_outliers(X, 6.0)
    q = oracle_mod.zp_quantize_rows(X, idx)
    keep = np.ones(160, bool)
    keep[idx] = False
    codes = q["Xq"][:, keep].astype(np.int64)
    assert codes.min(axis=1).tolist() == [-127] * 48 and codes.max(axis=1).tolist() == [127] * 48
    assert not q["Xq"][:, ~keep].any()
    # absmax would leave the negative half of the codes unused on such rows; zeropoint halves the step
    lo, hi = q["lo"].astype(np.float64), q["hi"].astype(np.float64)
    D = (hi - lo)[:, None]
    back = (codes + q["zp"][:, None]) * D / 254.0
    assert np.abs(back - X[:, keep].astype(np.float64)).max() <= (D / 508.0).max() * (1 + 1e-12)
    assert (np.abs(back - X[:, keep].astype(np.float64)) <= D / 508.0 * (1 + 1e-12)).all()
    # zero is represented exactly: code + zp = 0
    zr, zc = np.nonzero(X[:, keep] == 0)
    assert len(zr) > 100 and ((codes + q["zp"][:, None])[zr, zc] == 0).all()
    w = oracle_mod.zp_quantize_weight(W)
    assert np.abs(w["Wq"]).max() == 127 and w["Wq"].min(axis=0).tolist() == [-127] * 64
    assert np.array_equal(w["colsum"], w["Wq"].astype(np.int64).sum(axis=0))


def test_symmetric_ranges_reduce_to_the_absmax_quantizer(oracle_mod):
    """lo = -hi gives D = 2 hi, u(x) = round(127 x / hi) and zp = 0: the same codes, the same integer
    product and the same output as the vector-wise absmax oracle."""
    d = wl.make_custom(20, 96, 40, 2, seed=31)
    X, W = d["X"].copy(), d["W"].copy()
    O = set(oracle_mod.find_outliers(X, 6.0).tolist())
    free = [j for j in range(96) if j not in O]
    for i in range(20):   # every row gets +m and -m, m its largest non-outlier magnitude
        m = np.abs(X[i, free]).max()
        X[i, free[0]], X[i, free[1]] = m, -m
    for j in range(40):
        m = np.abs(W[:, j]).max()
        W[0, j], W[1, j] = m, -m
    assert set(oracle_mod.find_outliers(X, 6.0).tolist()) == O
    a = oracle_mod.linear(X, W, 6.0)
    z = oracle_mod.zp_linear(X, W, 6.0)
    assert not z["zp_x"].any() and not z["zp_w"].any()
    assert np.array_equal(z["Xq"], a["Xq"]) and np.array_equal(z["Wq"], a["Wq"])
    assert np.array_equal(z["C"], a["C"]) and np.array_equal(z["T"], a["C"].astype(np.int64))
    assert np.array_equal(z["hi_x"].view(np.uint16), a["cx"].view(np.uint16))
    assert np.array_equal(z["Out"].view(np.uint16), a["Out"].view(np.uint16))


def test_unrolled_form_of_eq5_gives_the_sum_of_eq4(oracle_mod):
    """T = A B + zb rowsum(A) + za colsum'(B) + (h - |O|) za zb, with colsum' over the non-outlier rows."""
    d = wl.make_custom(30, 128, 50, 3, seed=41)
    X = d["X"] + np.float16(0.5)
    r = oracle_mod.zp_linear(X, d["W"], 6.0)
    keep = np.ones(128, bool)
    keep[r["idx"]] = False
    A, B = r["Xq"].astype(np.int64), r["Wq"].astype(np.int64)
    za, zb = r["zp_x"].astype(np.int64)[:, None], r["zp_w"].astype(np.int64)[None, :]
    cs_keep = B[keep].sum(axis=0)[None, :]
    T = A @ B + zb * r["rowsum"].astype(np.int64)[:, None] + za * cs_keep + keep.sum() * za * zb
    assert np.array_equal(T, r["T"])
    assert np.array_equal(cs_keep[0], r["colsum"] - B[~keep].sum(axis=0))


def test_integer_grid_inputs_have_known_codes(oracle_mod):
    """Rows of X = integers in [a, a + 254] over 64 with both ends present: nd = 64, u(x) = 64 x, so
    code + zp is the integer itself; same for W over 512.  Then T = N M exactly and Out = fp16(N M / 32768)."""
    rng = np.random.default_rng(5)
    s, h, o = 7, 48, 9
    a = rng.integers(-200, 60, size=s)
    N = a[:, None] + rng.integers(0, 255, size=(s, h))
    N[:, 0], N[:, 1] = a, a + 254
    b = rng.integers(-150, -80, size=o)
    M = b[None, :] + rng.integers(0, 255, size=(h, o))
    M[0, :], M[1, :] = b, b + 254
    X, W = (N / 64).astype(np.float16), (M / 512).astype(np.float16)
    assert np.array_equal(X.astype(np.float64) * 64, N) and np.array_equal(W.astype(np.float64) * 512, M)
    r = oracle_mod.zp_linear(X, W, float("inf"))
    assert np.array_equal(r["zp_x"], a + 127) and np.array_equal(r["zp_w"], b + 127)
    assert np.array_equal(r["Xq"] + r["zp_x"][:, None], N) and np.array_equal(r["Wq"] + r["zp_w"][None, :], M)
    assert np.array_equal(r["T"], N @ M)
    assert np.array_equal(r["Out"], ((N @ M) / 32768.0).astype(np.float16))


def test_sampled_outputs_equal_the_full_computation(oracle_mod):
    d = wl.make_custom(33, 160, 70, 3, seed=12)
    X = np.maximum(d["X"], np.float16(-0.5))
    full = oracle_mod.zp_linear(X, d["W"], 6.0)
    rng = np.random.default_rng(0)
    rows, cols = rng.integers(0, 33, 50), rng.integers(0, 70, 50)
    Cs, Os = oracle_mod.zp_sampled(X, d["W"], full["idx"], rows, cols)
    assert np.array_equal(Cs, full["C"][rows, cols])
    assert np.array_equal(Os.view(np.uint16), full["Out"][rows, cols].view(np.uint16))
