"""HIP path vs CPU oracle for the zeropoint variant (Section 2.1, Eq. 1-5, per row of X and per
column of W, with and without the decomposition of Section 3.2).  Ranges, zeropoints, codes, row and
column sums and the plain int8 product bit for bit; outputs within 1e-3 of the largest output."""
import numpy as np
import pytest

import oracle
from paper_2208_07339_amd import workloads as wl
from gpu_util import assert_out_close, bits

pytestmark = pytest.mark.gpu

INF = float("inf")


def upload(X, W):
    import torch
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16)
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    return Xd, Wd


def unpack(zc):
    """[n, 4] int32 records -> lo bits, hi bits, zp, sum."""
    zc = zc.cpu().numpy()
    w0 = zc[:, 0].astype(np.int64) & 0xffffffff
    assert not zc[:, 3].any()
    return (w0 & 0xffff).astype(np.uint16), (w0 >> 16).astype(np.uint16), zc[:, 1], zc[:, 2]


def zp_compare(X, W, alpha, cap=32):
    import torch

    import paper_2208_07339_amd as L
    s, h = X.shape
    o = W.shape[1]
    ref = oracle.zp_linear(X, W, alpha)
    assert len(ref["idx"]) <= cap
    Xd, Wd = upload(X, W)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.zp_quantize_weight(Wd, ws)
    lo, hi, zp, cs = unpack(qw.zc)
    assert np.array_equal(lo, bits(ref["lo_w"])) and np.array_equal(hi, bits(ref["hi_w"]))
    assert np.array_equal(zp, ref["zp_w"]) and np.array_equal(cs, ref["colsum"])
    wq_host = L.export_weight(L.QuantizedWeight(qw.Wq, None, None, h, o)).cpu().numpy()
    assert np.array_equal(wq_host, ref["Wq"])
    # staged calls
    outl = L.find_outliers(Xd, alpha, cap, ws)
    rows = L.zp_quantize_rows(Xd, outl)
    out, Cd = L.zp_matmul(rows, outl, qw, ws, want_c_i32=True)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == ref["idx"].tolist()
    lo, hi, zp, rs = unpack(rows.zc)
    assert np.array_equal(lo, bits(ref["lo_x"])) and np.array_equal(hi, bits(ref["hi_x"]))
    assert np.array_equal(zp, ref["zp_x"]) and np.array_equal(rs, ref["rowsum"])
    xq_host = L.export_rows(L.QuantizedRows(rows.Xq, None, None, s, h)).cpu().numpy()
    assert np.array_equal(xq_host, ref["Xq"])
    Xo = rows.Xo.cpu().numpy()
    assert np.array_equal(bits(Xo[:, :n]), bits(X[:, ref["idx"]])) and not bits(Xo[:, n:]).any()
    assert np.array_equal(Cd.cpu().numpy(), ref["C"])
    assert_out_close(out.cpu().numpy(), ref["Out"])
    # one call, into buffers holding junk, twice
    outl2 = L.Outliers(torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                       torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                       torch.full((1,), -7, dtype=torch.int32, device="cuda"), cap)
    rows2 = L.ZpRows(torch.full((L.xq_bytes(s, h),), 99, dtype=torch.int8, device="cuda"),
                     torch.full((s, 4), 12345, dtype=torch.int32, device="cuda"),
                     torch.full((s, L.opad(cap)), 7.0, dtype=torch.float16, device="cuda"), s, h)
    for _ in range(2):
        out2 = L.zp_linear(Xd, qw, alpha, outl2, rows2, ws)
    torch.cuda.synchronize()
    assert int(outl2.count.item()) == n and int(outl2.status.item()) == 0
    assert torch.equal(outl2.idx[:n], outl.idx[:n]) and torch.equal(rows2.Xo, rows.Xo)
    assert torch.equal(rows2.zc, rows.zc) and torch.equal(rows2.Xq, rows.Xq)
    assert_out_close(out2.cpu().numpy(), ref["Out"])
    return ref


def one_sided(d, shift=0.0):
    """The recipe's inputs made asymmetric: non-outlier entries clipped at -0.25 (a leaky ReLU-like
    cut), optionally shifted; the planted outlier columns are kept."""
    X = np.maximum(d["X"], np.float16(-0.25)) + np.float16(shift)
    X[:, d["planted"]] = d["X"][:, d["planted"]]
    return np.ascontiguousarray(X.astype(np.float16))


SHAPES = [(8, 256, 512, 2), (16, 1024, 2048, 5), (13, 200, 61, 2), (32, 4160, 96, 6),   # weight-streaming path
          (33, 64, 32, 1), (100, 300, 200, 3), (256, 1024, 512, 4), (333, 520, 260, 5),  # tiled path
          (48, 1000, 264, 4), (64, 384, 96, 7)]                       # ... with two row tiles of X


@pytest.mark.parametrize("alpha", [6.0, INF])
@pytest.mark.parametrize("s,h,o,ncol", SHAPES)
def test_zeropoint_on_one_sided_inputs(s, h, o, ncol, alpha):
    d = wl.make_custom(s, h, o, ncol, seed=5 * s + h)
    ref = zp_compare(one_sided(d), d["W"], alpha)
    if alpha == 6.0:
        assert (ref["zp_x"] != 0).all()  # these rows are far from symmetric


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5])
def test_every_prefill_tile_shape(cfg):
    """Each workgroup tile of the prefill GEMM in its zeropoint form (staged calls with the accumulator export:
    guarded epilogue; one call: records and column factors staged through LDS, stores without guards), on grids
    with full tiles next to ragged ones: 7 and 20 outlier columns, a
    16-slot outlier buffer, one-sided and shifted inputs (zeropoints far from 0: the correction terms of Eq. 5
    are large and cancel)."""
    import paper_2208_07339_amd as L
    L.debug_prefill_tile(cfg)
    try:
        d = wl.make_custom(512, 1024, 1024, 7, seed=91)
        zp_compare(one_sided(d), d["W"], 6.0)
        d = wl.make_custom(600, 640, 776, 20, seed=92)
        zp_compare(one_sided(d, shift=1.5), d["W"], 6.0)
        d = wl.make_custom(256, 256, 512, 3, seed=93)
        zp_compare(one_sided(d), d["W"], 6.0, cap=8)
        d = wl.make_custom(384, 512, 768, 0, seed=94)
        zp_compare(one_sided(d, shift=-2.0), d["W"], INF)
        d = wl.make_custom(443, 384, 768, 12, seed=95)  # the last tile of tokens is ragged, s odd
        zp_compare(one_sided(d, shift=0.75), d["W"], 6.0)
        d = wl.make_custom(320, 384, 520, 6, seed=96)   # 64-slot outlier buffer, 6 columns: the unguarded kernel
        zp_compare(one_sided(d), d["W"], 6.0, cap=64)
        d = wl.make_custom(320, 384, 520, 40, seed=97)  # ... 40 columns: the guarded one, launched behind it
        zp_compare(one_sided(d), d["W"], 6.0, cap=64)
    finally:
        L.debug_prefill_tile(-1)


def test_short_x_through_the_tiled_kernel():
    """The zeropoint form of the tiled kernel on 32 tokens and fewer (the library sends them there only for
    some shapes of W; the test hook switches the weight-streaming kernel off): column factors from the
    short-X pre-pass, a single ragged token tile.  Then a W for which the library makes that choice itself."""
    import paper_2208_07339_amd as L
    L.debug_decode_shape(0)
    try:
        for s, h, o, ncol, seed in [(16, 512, 776, 5, 41), (1, 256, 264, 1, 42), (32, 1152, 520, 20, 43)]:
            d = wl.make_custom(s, h, o, ncol, seed=seed)
            zp_compare(one_sided(d, shift=0.5), d["W"], 6.0)
    finally:
        L.debug_decode_shape(-1)
    d = wl.make_custom(16, 128, 20480, 2, seed=44)  # 640 column tiles
    zp_compare(one_sided(d), d["W"], 6.0)


@pytest.mark.parametrize("s,h,o", [(16, 512, 256), (150, 384, 320)])
def test_zeropoint_on_the_symmetric_recipe_and_a_shifted_one(s, h, o):
    d = wl.make_custom(s, h, o, 3, seed=77)
    zp_compare(d["X"], d["W"], 6.0)
    zp_compare(one_sided(d, shift=2.5), np.ascontiguousarray(d["W"] + np.float16(0.03)), 6.0)  # large zeropoints


def test_constant_and_zero_vectors():
    d = wl.make_custom(40, 128, 64, 2, seed=3)
    X, W = d["X"].copy(), d["W"].copy()
    X[3] = 0
    X[7] = np.float16(1.5)
    W[:, 5] = 0
    W[:, 9] = np.float16(-0.25)
    ref = zp_compare(X, W, 6.0)
    assert ref["zp_x"][3] == 0 and not ref["Xq"][7].any() and not ref["Wq"][:, 9].any()
    zp_compare(np.zeros((5, 64), np.float16), np.zeros((64, 32), np.float16), 6.0)


def test_prefill_13b_ffn_up_full_size():
    """Full benchmark size: ranges, zeropoints, sums and both int8 tensors in full; accumulators and
    outputs on random samples the oracle computes one by one."""
    import torch

    import paper_2208_07339_amd as L
    d = wl.make("ffn13b")
    X, W = one_sided(d), d["W"]
    s, h, o, cap = d["s"], d["h"], d["o"], 32
    Xd, Wd = upload(X, W)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.zp_quantize_weight(Wd, ws)
    outl = L.Outliers(torch.empty(cap, dtype=torch.int32, device="cuda"),
                      torch.empty(1, dtype=torch.int32, device="cuda"),
                      torch.empty(1, dtype=torch.int32, device="cuda"), cap)
    rows = L.ZpRows(torch.empty(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                    torch.empty((s, 4), dtype=torch.int32, device="cuda"),
                    torch.empty((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h)
    out = L.zp_linear(Xd, qw, 6.0, outl, rows, ws)
    _, Cd = L.zp_matmul(rows, outl, qw, ws, want_c_i32=True)
    torch.cuda.synchronize()
    idx = oracle.find_outliers(X, 6.0)
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    w = oracle.zp_quantize_weight(W)
    lo, hi, zp, cs = unpack(qw.zc)
    assert np.array_equal(lo, bits(w["lo"])) and np.array_equal(hi, bits(w["hi"]))
    assert np.array_equal(zp, w["zp"]) and np.array_equal(cs, w["colsum"])
    assert np.array_equal(L.export_weight(L.QuantizedWeight(qw.Wq, None, None, h, o)).cpu().numpy(), w["Wq"])
    x = oracle.zp_quantize_rows(X, idx)
    lo, hi, zp, rs = unpack(rows.zc)
    assert np.array_equal(lo, bits(x["lo"])) and np.array_equal(hi, bits(x["hi"]))
    assert np.array_equal(zp, x["zp"]) and np.array_equal(rs, x["rowsum"])
    assert np.array_equal(L.export_rows(L.QuantizedRows(rows.Xq, None, None, s, h)).cpu().numpy(), x["Xq"])
    rng = np.random.default_rng(78)
    ri, ci = rng.integers(0, s, 1200), rng.integers(0, o, 1200)
    Cs, Os = oracle.zp_sampled(X, W, idx, ri, ci)
    assert np.array_equal(Cd.cpu().numpy()[ri, ci], Cs)
    assert_out_close(out.cpu().numpy()[ri, ci], Os, float(np.abs(Os.astype(np.float64)).max()))


@pytest.mark.parametrize("s", [24, 200])
def test_codes_at_exact_ties(s):
    """Every third row has the range D = 254 / 2^k and entries that are odd multiples of 2^-(k+1): each quotient
    254 x / D is an integer plus one half, so each code is decided by the round-half-even rule alone (a
    quotient that is off by one unit in the last place lands on the wrong side).  Codes, sums and the
    product bit-exact as everywhere else; the rows in between are ordinary ones."""
    rng = np.random.default_rng(400 + s)
    h, o = 1040, 72
    d = wl.make_custom(s, h, o, 3, seed=17)
    X = one_sided(d)
    free = [c for c in range(h) if c not in set(d["planted"].tolist())]
    for i in range(0, s, 3):
        k = int(rng.integers(5, 8))                              # D / 2 < 4: no new outlier columns
        D = 254.0 / 2.0 ** k
        row = (rng.integers(-127, 127, h) + 0.5) / 2.0 ** k      # |row| < D / 2, exact in fp16
        row[free[0]], row[free[1]] = -D / 2, D / 2               # the row's range, exactly
        keep = X[i, d["planted"]].copy()
        X[i] = row.astype(np.float16)
        assert np.array_equal(X[i].astype(np.float64), row)
        X[i, d["planted"]] = keep
    zp_compare(np.ascontiguousarray(X), d["W"], 6.0)


def test_more_outlier_columns_than_cap():
    """Only the first cap columns count as outliers; the rest are quantized like any other column (their
    large entries then widen the row ranges).  The oracle is given exactly that set."""
    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(90, 512, 128, 9, seed=61)
    X, W, cap = one_sided(d), d["W"], 4
    full = oracle.find_outliers(X, 6.0)
    assert len(full) > cap
    O = full[:cap]
    Xd, Wd = upload(X, W)
    ws = L.Workspace.allocate(90, 512, 128, cap)
    qw = L.zp_quantize_weight(Wd, ws)
    outl = L.find_outliers(Xd, 6.0, cap, ws)
    rows = L.zp_quantize_rows(Xd, outl)
    out, Cd = L.zp_matmul(rows, outl, qw, ws, want_c_i32=True)
    torch.cuda.synchronize()
    assert int(outl.status.item()) == 1 and outl.idx.cpu().numpy().tolist() == O.tolist()
    x = oracle.zp_quantize_rows(X, O)
    w = oracle.zp_quantize_weight(W)
    lo, hi, zp, rs = unpack(rows.zc)
    assert np.array_equal(lo, bits(x["lo"])) and np.array_equal(hi, bits(x["hi"]))
    assert np.array_equal(zp, x["zp"]) and np.array_equal(rs, x["rowsum"])
    assert np.array_equal(L.export_rows(L.QuantizedRows(rows.Xq, None, None, 90, 512)).cpu().numpy(), x["Xq"])
    assert np.array_equal(Cd.cpu().numpy(), oracle.igemm(x["Xq"], w["Wq"]))
    ri, ci = np.repeat(np.arange(90), 128), np.tile(np.arange(128), 90)
    _, Os = oracle.zp_sampled(X, W, O, ri, ci)
    assert_out_close(out.cpu().numpy().reshape(-1), Os)


@pytest.mark.parametrize("s", [12, 70])
def test_one_call_with_an_outlier_buffer_too_large_for_the_column_job(s):
    """cap > 256: the per-column factors come from zp_kcol_kernel as in the staged calls, not from extra
    workgroups of a pre-pass kernel (the short-X one for 12 tokens, the one that takes the rows' ranges for 70).
    Same outputs as the staged calls, Out against the oracle."""
    d = wl.make_custom(s, 264, 72, 5, seed=91)
    zp_compare(one_sided(d), d["W"], 6.0, cap=300)


@pytest.mark.parametrize("s", [7, 32, 33, 57, 64])
def test_short_x_in_one_call_with_more_outlier_columns_than_cap(s):
    """The two-kernel pre-pass of a short X (s <= 32) inside llmint8_zp_linear, when more columns qualify
    than the buffer takes: the row ranges are taken again over everything but the first cap columns.  Every
    output of the call against the staged calls (which the test above pins to the oracle), Out against the
    oracle."""
    import torch

    import paper_2208_07339_amd as L
    h, o, cap = 520, 136, 4
    d = wl.make_custom(s, h, o, 9, seed=62 + s)
    X, W = one_sided(d, shift=0.5), d["W"]
    full = oracle.find_outliers(X, 6.0)
    assert len(full) > cap
    O = full[:cap]
    Xd, Wd = upload(X, W)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.zp_quantize_weight(Wd, ws)
    outl = L.find_outliers(Xd, 6.0, cap, ws)
    rows = L.zp_quantize_rows(Xd, outl)
    torch.cuda.synchronize()
    x = oracle.zp_quantize_rows(X, O)
    lo, hi, zp, rs = unpack(rows.zc)
    assert np.array_equal(lo, bits(x["lo"])) and np.array_equal(zp, x["zp"]) and np.array_equal(rs, x["rowsum"])
    outl2 = L.Outliers(torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                       torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                       torch.full((1,), -7, dtype=torch.int32, device="cuda"), cap)
    rows2 = L.ZpRows(torch.full((L.xq_bytes(s, h),), 99, dtype=torch.int8, device="cuda"),
                     torch.full((s, 4), 12345, dtype=torch.int32, device="cuda"),
                     torch.full((s, L.opad(cap)), 7.0, dtype=torch.float16, device="cuda"), s, h)
    for _ in range(2):
        out2 = L.zp_linear(Xd, qw, 6.0, outl2, rows2, ws)
    torch.cuda.synchronize()
    assert int(outl2.count.item()) == cap and int(outl2.status.item()) == 1
    assert outl2.idx.cpu().numpy().tolist() == O.tolist()
    assert torch.equal(rows2.zc, rows.zc) and torch.equal(rows2.Xq, rows.Xq) and torch.equal(rows2.Xo, rows.Xo)
    ri, ci = np.repeat(np.arange(s), o), np.tile(np.arange(o), s)
    _, Os = oracle.zp_sampled(X, W, O, ri, ci)
    assert_out_close(out2.cpu().numpy().reshape(-1), Os)


def test_argument_errors_are_reported_not_executed():
    import ctypes as C

    import torch

    import paper_2208_07339_amd as L
    lib = L.lib()
    p = lambda t: C.c_void_p(t.data_ptr())
    W = torch.zeros((64, 32), dtype=torch.float16, device="cuda")
    X = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    Wq = torch.empty(L.wq_bytes(64, 32), dtype=torch.int8, device="cuda")
    Xq = torch.empty(L.xq_bytes(4, 64), dtype=torch.int8, device="cuda")
    zw = torch.zeros((32, 4), dtype=torch.int32, device="cuda")
    zx = torch.zeros((4, 4), dtype=torch.int32, device="cuda")
    idx = torch.zeros(16, dtype=torch.int32, device="cuda")
    Xo = torch.zeros((4, 16), dtype=torch.float16, device="cuda")
    out = torch.zeros((4, 32), dtype=torch.float16, device="cuda")
    ws = L.Workspace.allocate(4, 64, 32, 16)
    INVALID, SHAPE, WORKSPACE = 1, 2, 3
    assert lib.llmint8_zp_quantize_weight(None, 64, 32, p(Wq), p(zw), p(ws.buf), ws.nbytes, None) == INVALID
    assert lib.llmint8_zp_quantize_weight(p(W), 64, 32, p(Wq), p(zw), p(ws.buf), 16, None) == WORKSPACE
    assert lib.llmint8_zp_quantize_weight(p(W), 133145, 32, p(Wq), p(zw), p(ws.buf), ws.nbytes, None) == SHAPE
    assert lib.llmint8_zp_quantize_rows(p(X), 4, 64, p(idx), p(idx), 0, p(Xq), p(zx), p(Xo), None) == INVALID
    # the 16-bit weights are required by this variant
    assert lib.llmint8_zp_matmul(p(Xq), p(zx), p(Xo), p(idx), p(idx), 16, p(Wq), p(zw), None, 4, 64, 32, p(out), None,
                                 p(ws.buf), ws.nbytes, None) == INVALID
    assert lib.llmint8_zp_matmul(p(Xq), p(zx), p(Xo), p(idx), p(idx), 16, p(Wq), p(zw), p(W), 4, 64, 32, p(out), None,
                                 p(ws.buf), 64, None) == WORKSPACE
    # records must be 16-byte aligned
    off = torch.zeros(4 * 4 + 1, dtype=torch.int32, device="cuda")[1:]
    assert lib.llmint8_zp_quantize_rows(p(X), 4, 64, p(idx), p(idx), 16, p(Xq), p(off), p(Xo), None) == INVALID
    assert lib.llmint8_zp_linear(p(X), 4, 64, 6.0, p(Wq), p(zw), p(W), 32, p(idx), 16, p(idx), None, p(Xq), p(zx),
                                 p(Xo), p(out), p(ws.buf), 64, None) == WORKSPACE


def test_random_shapes():
    """Seeded random shapes on both GEMM paths, aligned and ragged, random numbers of outlier columns,
    one-sided and shifted inputs, with and without the decomposition: every stage against the oracle."""
    rng = np.random.default_rng(20240611)
    for case in range(16):
        s = int(rng.choice([rng.integers(1, 33), rng.integers(33, 300)]))
        h = int(rng.choice([8 * rng.integers(4, 200), rng.integers(20, 1200)]))
        o = int(rng.choice([8 * rng.integers(2, 80), rng.integers(9, 500)]))
        ncol = int(rng.integers(0, min(h, 20)))
        alpha = float(rng.choice([6.0, 6.0, INF]))
        shift = float(rng.choice([0.0, 0.0, 1.5, -0.75]))
        d = wl.make_custom(s, h, o, ncol, seed=2000 + case)
        X = one_sided(d, shift)
        if len(oracle.find_outliers(X, alpha)) > 32:
            continue
        try:
            zp_compare(X, d["W"], alpha)
        except AssertionError as e:
            raise AssertionError(f"case {case}: s={s} h={h} o={o} ncol={ncol} alpha={alpha} shift={shift}: {e}") from e
