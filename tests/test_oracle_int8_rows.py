"""Pins of the oracle's int8-rows variant (the outlier rows of W rebuilt from the codes, W^ =
fp16(W_i8 * c_w / 127), in place of W_f16 in Eq. 8): exact rational arithmetic for W^, the
half-step bound of the absmax quantizer it inverts (Section 2.1), a float64 library matmul of the
dequantized weights for alpha = 0, and agreement with the fp16-rows oracle where W is exactly
representable by its codes."""
from fractions import Fraction

import numpy as np

from exact_util import f16_fraction, nearest_f16
from paper_2208_07339_amd import workloads as wl


def test_dequant_weight_is_the_correctly_rounded_quotient(oracle_mod):
    rng = np.random.default_rng(5)
    cws = np.concatenate([rng.integers(1, 0x7c00, 150), [1, 2, 0x3ff, 0x400, 0x7bff, 0x2e66, 0x3c00]])
    for cwb in cws:
        cw = np.uint16(cwb).view(np.float16)
        for q in (-127, -126, -64, -3, -1, 0, 1, 2, 63, 100, 127):
            got = oracle_mod.dequant_weight(q, cw)
            want = nearest_f16(Fraction(q) * f16_fraction(cwb) / 127)
            assert got.view(np.uint16) == want or (q == 0 and got == 0), (q, hex(cwb))
    # +-127 gives back the constant itself, 0 gives 0
    assert oracle_mod.dequant_weight(127, np.float16(0.75)) == np.float16(0.75)
    assert oracle_mod.dequant_weight(-127, np.float16(0.75)) == np.float16(-0.75)
    assert oracle_mod.dequant_weight(0, np.float16(0.75)) == 0


def test_dequantized_rows_stay_within_half_a_step_of_the_weights(oracle_mod):
    W = wl.make_w(96, 80, seed=3)
    Wq, cw = oracle_mod.quantize_weight(W)
    idx = np.array([0, 7, 50, 95], np.int32)
    rows = oracle_mod.dequant_rows(Wq, cw, idx).astype(np.float64)
    c = cw.astype(np.float64)[None, :]
    err = np.abs(rows - W[idx].astype(np.float64))
    # half a quantization step plus half an fp16 ulp of the rebuilt value
    assert np.all(err <= c / 254 + np.abs(rows) * 2.0 ** -11 + 2.0 ** -25)
    # each row reproduces its codes when quantized again with the same constants
    for t, k in enumerate(idx):
        for j in range(W.shape[1]):
            assert oracle_mod.q(float(rows[t, j]), float(cw[j])) == Wq[k, j]


def test_alpha_zero_is_a_matmul_with_the_dequantized_weights(oracle_mod):
    d = wl.make_custom(6, 40, 24, 2, seed=11)
    X, W = d["X"], d["W"]
    Wq, cw = oracle_mod.quantize_weight(W)
    idx = oracle_mod.find_outliers(X, 0.0)
    assert len(idx) == 40
    Xq, cx = oracle_mod.quantize_rows(X, idx)
    Cm = oracle_mod.igemm(Xq, Wq)
    assert not Cm.any()
    Out = oracle_mod.output_dq(Cm, cx, cw, X, Wq, idx)
    What = oracle_mod.dequant_rows(Wq, cw, np.arange(40, dtype=np.int32)).astype(np.float64)
    ref = (X.astype(np.float64) @ What).astype(np.float16)
    # float64 matmul then one rounding; the oracle adds in a different order, so allow the last fp16 bit
    diff = np.abs(Out.view(np.int16).astype(np.int32) - ref.view(np.int16).astype(np.int32))
    assert diff.max() <= 1 and (diff == 0).mean() > 0.95


def test_brute_force_and_agreement_with_fp16_rows_on_representable_weights(oracle_mod):
    d = wl.make_custom(5, 32, 12, 3, seed=13)
    X = d["X"]
    # weights that are exactly q * c / 127 rounded to fp16: rebuilding them from the codes is lossless
    rng = np.random.default_rng(17)
    c = np.float16(127.0 / 64)  # step 1/64: q * c / 127 = q / 64 exactly
    q = rng.integers(-127, 128, size=(32, 12))
    q[0, :] = 127
    W = (q / 64.0).astype(np.float16)
    Wq, cw = oracle_mod.quantize_weight(W)
    assert np.array_equal(Wq, q) and np.all(cw == c)
    r = oracle_mod.linear(X, W, 6.0)
    Out_dq = oracle_mod.output_dq(r["C"], r["cx"], r["cw"], X, r["Wq"], r["idx"])
    assert np.array_equal(Out_dq.view(np.uint16), r["Out"].view(np.uint16))
    # pure-Python loops with exact rationals for one general case
    W2 = wl.make_w(32, 12, seed=19)
    r2 = oracle_mod.linear(X, W2, 6.0)
    Out2 = oracle_mod.output_dq(r2["C"], r2["cx"], r2["cw"], X, r2["Wq"], r2["idx"])
    for i in range(5):
        for j in range(12):
            acc = Fraction(int(r2["C"][i, j])) * f16_fraction(r2["cx"].view(np.uint16)[i]) * \
                f16_fraction(r2["cw"].view(np.uint16)[j]) / 16129
            for k in r2["idx"]:
                what = nearest_f16(Fraction(int(r2["Wq"][k, j])) * f16_fraction(r2["cw"].view(np.uint16)[j]) / 127)
                acc += f16_fraction(X.view(np.uint16)[i, k]) * f16_fraction(what)
            # the oracle sums in double: allow one fp16 ulp against the exact sum
            got = int(Out2.view(np.int16)[i, j])
            want = int(nearest_f16(acc).view(np.int16))
            assert abs(got - want) <= 1, (i, j)
