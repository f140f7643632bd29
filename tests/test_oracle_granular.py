"""Pins of the oracle's coarser-constant baselines (Table 1: tensor-wise absmax of Section 2.1,
row-wise, vector-wise of Section 3.1, each with and without the decomposition of Section 3.2).

Nothing here re-uses the oracle's own arithmetic: the expected values come from exact rational
arithmetic written out below, from integer-valued inputs whose codes are known in closed form, or
from the already pinned vector-wise functions on inputs where the granularities must coincide."""
from fractions import Fraction

import numpy as np
import pytest

from exact_util import f16_fraction, nearest_f16
from paper_2208_07339_amd import workloads as wl

MODES = ("vectorwise", "rowwise", "tensorwise")


def exact_linear(X, W, alpha, mode):
    """The whole method in rational arithmetic, straight from Sections 2.1, 3.1, 3.2 (tiny inputs)."""
    s, h = X.shape
    o = W.shape[1]
    xf = [[f16_fraction(b) for b in row] for row in X.view(np.uint16)]
    wf = [[f16_fraction(b) for b in row] for row in W.view(np.uint16)]
    a = Fraction(alpha) if np.isfinite(alpha) else None
    O = [j for j in range(h) if a is not None and any(abs(xf[i][j]) >= a for i in range(s))]
    keep = [j for j in range(h) if j not in O]
    rowmax = [max([abs(xf[i][j]) for j in keep], default=Fraction(0)) for i in range(s)]
    colmax = [max(abs(wf[k][j]) for k in range(h)) for j in range(o)]
    if mode == "tensorwise":
        rowmax = [max(rowmax)] * s
    if mode != "vectorwise":
        colmax = [max(colmax)] * o
    code = lambda v, c: 0 if c == 0 else round(127 * v / c)  # Fraction.__round__: nearest, ties to even
    Xq = [[0 if j in O else code(xf[i][j], rowmax[i]) for j in range(h)] for i in range(s)]
    Wq = [[code(wf[k][j], colmax[j]) for j in range(o)] for k in range(h)]
    Cm = [[sum(Xq[i][k] * Wq[k][j] for k in range(h)) for j in range(o)] for i in range(s)]
    Out = [[nearest_f16(Cm[i][j] * rowmax[i] * colmax[j] / 16129 + sum(xf[i][k] * wf[k][j] for k in O))
            for j in range(o)] for i in range(s)]
    return O, rowmax, colmax, np.array(Xq), np.array(Wq), np.array(Cm), np.array(Out, dtype=np.uint16)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("alpha", [6.0, float("inf"), 0.0])
def test_every_stage_equals_exact_rational_arithmetic(oracle_mod, mode, alpha):
    rng = np.random.default_rng(11)
    X = rng.normal(size=(5, 12)).astype(np.float16)
    W = (0.05 * rng.normal(size=(12, 7))).astype(np.float16)
    X[1, 3] = 9.5      # one outlier column
    X[4, 3] = -31.0
    X[2, :] *= np.float16(0.25)   # rows and columns of clearly different size, so the
    W[:, 5] *= np.float16(4.0)    # granularities give different codes
    O, rowmax, colmax, Xq, Wq, Cm, Out = exact_linear(X, W, alpha, mode)
    r = oracle_mod.linear_granular(X, W, alpha, mode)
    assert list(r["idx"]) == O
    assert [f16_fraction(b) for b in r["cx"].view(np.uint16)] == rowmax
    assert [f16_fraction(b) for b in r["cw"].view(np.uint16)] == colmax
    assert np.array_equal(r["Xq"], Xq) and np.array_equal(r["Wq"], Wq)
    assert np.array_equal(r["C"], Cm)
    got = r["Out"].view(np.uint16)
    same = (got == Out) | (((got | Out) & 0x7fff) == 0)  # +0 and -0 are the same result
    assert same.all()


def test_the_three_granularities_differ_on_that_input(oracle_mod):
    """Guards the test above against passing because the modes were never told apart."""
    rng = np.random.default_rng(11)
    X = rng.normal(size=(5, 12)).astype(np.float16)
    W = (0.05 * rng.normal(size=(12, 7))).astype(np.float16)
    X[2, :] *= np.float16(0.25)
    W[:, 5] *= np.float16(4.0)
    v, r, t = (oracle_mod.linear_granular(X, W, float("inf"), m) for m in MODES)
    assert not np.array_equal(v["Wq"], r["Wq"]) and np.array_equal(v["Xq"], r["Xq"])
    assert not np.array_equal(r["Xq"], t["Xq"]) and np.array_equal(r["Wq"], t["Wq"])


def test_integer_valued_inputs_give_their_own_codes_tensorwise(oracle_mod):
    """X = A / 8, W = B / 32 with integer A, B in [-127, 127] that reach 127: the tensor-wise constants
    are 127/8 and 127/32, so the codes are A and B themselves and Out = fp16(A B / 256), a plain
    integer matrix product."""
    rng = np.random.default_rng(2)
    A = rng.integers(-127, 128, size=(9, 40))
    B = rng.integers(-127, 128, size=(40, 13))
    A[np.arange(9), rng.integers(0, 40, 9)] = 127 * rng.choice([-1, 1], 9)   # every row reaches 127 ..
    A[5, :] = rng.integers(-64, 65, size=40)                                   # .. except this one
    A[5, 0] = 64
    B[11, 2] = 127
    X, W = (A / 8).astype(np.float16), (B / 32).astype(np.float16)
    assert np.array_equal(X.astype(np.float64) * 8, A) and np.array_equal(W.astype(np.float64) * 32, B)
    t = oracle_mod.linear_granular(X, W, float("inf"), "tensorwise")
    assert np.array_equal(t["Xq"], A) and np.array_equal(t["Wq"], B)
    assert np.array_equal(t["C"], A @ B)
    assert (t["cx"] == np.float16(127 / 8)).all() and (t["cw"] == np.float16(127 / 32)).all()
    assert np.array_equal(t["Out"], ((A @ B) / 256.0).astype(np.float16))  # quotient exact in float64
    # row-wise: the short row is stretched to the full range, rne(127 a / 64); the others keep A
    r = oracle_mod.linear_granular(X, W, float("inf"), "rowwise")
    want5 = [round(Fraction(127 * int(a), 64)) for a in A[5]]
    assert list(r["Xq"][5]) == want5 and np.array_equal(np.delete(r["Xq"], 5, 0), np.delete(A, 5, 0))
    assert r["cx"][5] == np.float16(8.0) and np.array_equal(r["Wq"], B)


def test_granularities_coincide_when_rows_and_columns_share_one_maximum(oracle_mod):
    """If every row of X (outlier columns aside) and every column of W has the same largest magnitude,
    one constant per tensor is the same thing as one per vector."""
    d = wl.make_custom(24, 96, 40, 3, seed=4)
    X, W = d["X"].copy(), d["W"].copy()
    O = oracle_mod.find_outliers(X, 6.0)
    free = [j for j in range(96) if j not in set(O.tolist())]
    for i in range(24):
        X[i, free[i % 7]] = np.float16(5.5 if i % 2 else -5.5)   # below alpha, above every N(0,1) draw here
    for j in range(40):
        W[(3 * j) % 96, j] = np.float16(0.75)
    assert np.array_equal(oracle_mod.find_outliers(X, 6.0), O)
    v = oracle_mod.linear(X, W, 6.0)
    assert (v["cx"] == np.float16(5.5)).all() and (v["cw"] == np.float16(0.75)).all()
    for mode in MODES:
        g = oracle_mod.linear_granular(X, W, 6.0, mode)
        for key in ("idx", "Xq", "Wq", "C"):
            assert np.array_equal(g[key], v[key]), (mode, key)
        assert np.array_equal(g["cx"].view(np.uint16), v["cx"].view(np.uint16))
        assert np.array_equal(g["cw"].view(np.uint16), v["cw"].view(np.uint16))
        assert np.array_equal(g["Out"].view(np.uint16), v["Out"].view(np.uint16))


def test_shared_constant_is_the_largest_of_the_vector_constants(oracle_mod):
    d = wl.make_custom(40, 128, 48, 4, seed=8)
    X, W = d["X"], d["W"]
    v = oracle_mod.linear(X, W, 6.0)
    r = oracle_mod.linear_granular(X, W, 6.0, "rowwise")
    t = oracle_mod.linear_granular(X, W, 6.0, "tensorwise")
    assert np.array_equal(r["cx"].view(np.uint16), v["cx"].view(np.uint16))
    assert (r["cw"] == v["cw"].max()).all() and (t["cw"] == v["cw"].max()).all()
    assert (t["cx"] == v["cx"].max()).all() and t["cx"].max() < 6.0
    # half-step bound of rounding to nearest with the shared constant (Section 2.1)
    Xd, c = X.astype(np.float64), float(t["cx"][0])
    keep = np.ones(128, bool)
    keep[t["idx"]] = False
    assert np.abs(Xd[:, keep] - t["Xq"][:, keep] * c / 127).max() <= c / 254 * (1 + 1e-12)
    assert not t["Xq"][:, ~keep].any()
    # the row / column that holds the maximum maps to +-127, and no code leaves [-127, 127]
    assert np.abs(t["Xq"]).max() == 127 and np.abs(t["Wq"]).max() == 127
    assert np.abs(r["Xq"]).max(axis=1).min() == 127


@pytest.mark.parametrize("mode", ["rowwise", "tensorwise"])
def test_sampled_outputs_equal_the_full_computation(oracle_mod, mode):
    d = wl.make_custom(33, 160, 70, 3, seed=12)
    X, W = d["X"], d["W"]
    full = oracle_mod.linear_granular(X, W, 6.0, mode)
    rng = np.random.default_rng(0)
    rows, cols = rng.integers(0, 33, 50), rng.integers(0, 70, 50)
    Cs, Os = oracle_mod.sampled_granular(X, W, full["idx"], rows, cols, mode)
    assert np.array_equal(Cs, full["C"][rows, cols])
    assert np.array_equal(Os.view(np.uint16), full["Out"][rows, cols].view(np.uint16))
