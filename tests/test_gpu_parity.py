"""HIP path vs CPU oracle through the C-ABI, element by element, at sizes the
oracle finishes in seconds: several tiles, ragged tails, both GEMM paths, and
the degenerate cases of the method.  Integer stages bit-exact; fp16 output
within 1e-3 * max|Out|."""
import numpy as np
import pytest

import oracle
from paper_2208_07339_amd import workloads as wl
from gpu_util import assert_out_close, bits, hip_weight_i8, run_hip

pytestmark = pytest.mark.gpu


def full_compare(d, alpha=None, cap=32):
    alpha = d["alpha"] if alpha is None else alpha
    X, W = d["X"], d["W"]
    r = oracle.linear(X, W, alpha)
    g = run_hip(X, W, alpha, cap)
    assert g["status"] == 0
    assert g["idx"].tolist() == r["idx"].tolist()
    assert np.array_equal(bits(g["cw"]), bits(r["cw"]))
    assert np.array_equal(hip_weight_i8(g["qw"]), r["Wq"])
    assert np.array_equal(bits(g["cx"]), bits(r["cx"]))
    assert np.array_equal(g["Xq"], r["Xq"])
    n = len(r["idx"])
    assert np.array_equal(bits(g["Xo"][:, :n]), bits(X[:, r["idx"]]))
    assert not bits(g["Xo"][:, n:]).any()
    assert np.array_equal(g["C"], r["C"])
    assert_out_close(g["Out"], r["Out"])
    return g, r


def test_tiny_config():
    g, r = full_compare(wl.make("tiny"))
    assert g["idx"].tolist() == [17, 200]


@pytest.mark.parametrize("s,h,o,ncol", [
    (1, 64, 32, 1),          # single token, single tile
    (16, 1024, 2048, 5),     # decode path, aligned
    (13, 200, 61, 2),        # decode path, nothing aligned (scalar load/store paths)
    (32, 384, 96, 3),        # largest decode token count
    (33, 384, 96, 3),        # smallest prefill token count
    (300, 1000, 520, 4),     # prefill, two token blocks, three column blocks, ragged everywhere
    (257, 4160, 264, 6),     # one row into the second block, K not a multiple of 128
    (512, 2048, 1024, 7),    # aligned multi-block
])
def test_shapes_against_full_oracle(s, h, o, ncol):
    full_compare(wl.make_custom(s, h, o, ncol, seed=s * 7 + o))


@pytest.fixture
def forced_tile():
    import paper_2208_07339_amd as L
    yield L.debug_prefill_tile
    L.debug_prefill_tile(-1)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5])
def test_every_prefill_tile_shape(cfg, forced_tile):
    """Each workgroup tile of the prefill GEMM through the staged calls with the accumulator export, i.e. the
    kernels with the guarded epilogue: full and ragged tiles, 7 and 20 outlier columns, a 16-slot outlier
    buffer, more outlier columns than the unguarded kernels stage (40), and a shape where nothing is aligned."""
    forced_tile(cfg)
    full_compare(wl.make_custom(512, 2048, 1024, 7, seed=1))
    full_compare(wl.make_custom(600, 640, 776, 20, seed=2))
    full_compare(wl.make_custom(256, 256, 512, 3, seed=3), cap=8)
    full_compare(wl.make_custom(300, 384, 520, 40, seed=4), cap=48)
    full_compare(wl.make_custom(300, 1000, 515, 4, seed=5))
    full_compare(wl.make_custom(330, 128, 264, 0, seed=6))


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5])
def test_every_prefill_tile_shape_through_the_one_call_path(cfg, forced_tile):
    """llmint8_linear exports no accumulators, so with o % 8 == 0 the kernels with the epilogue that is fed from
    LDS and stores without guards run: the code the bench times.  Every workgroup tile, vector-wise constants
    (a wrong index into the staged c_x / c_w / Xo / W rows would show), on grids with full tiles next to tiles
    that reach past the last token or column (their operand requests clamped, their stores cut off by the
    buffer bounds): 7 and 20 outlier columns (one and two fp16 k-steps), a 16-slot outlier buffer (opad = 16),
    a wide ragged grid, no outlier column at all, and more columns than the buffer takes."""
    forced_tile(cfg)
    linear_compare(wl.make_custom(512, 2048, 1024, 7, seed=61))             # every tile full (cfg 0: 2 x 4)
    linear_compare(wl.make_custom(600, 640, 776, 20, seed=62))              # full + ragged in both directions
    linear_compare(wl.make_custom(256, 256, 512, 3, seed=63), cap=8)        # opad = 16
    linear_compare(wl.make_custom(520, 384, 1544, 12, seed=64), cap=16)     # opad = 16, wide grid, ragged edges
    linear_compare(wl.make_custom(384, 512, 768, 0, seed=65))               # no outlier product
    linear_compare(wl.make_custom(320, 256, 640, 9, seed=66), cap=4)        # |O| > cap: the first four only
    linear_compare(wl.make_custom(512, 1152, 576, 30, seed=67))             # nearly full 32-slot buffer
    linear_compare(wl.make_custom(72, 256, 768, 5, seed=68))                # every token tile ragged
    linear_compare(wl.make_custom(200, 320, 384, 18, seed=69))
    linear_compare(wl.make_custom(325, 256, 640, 9, seed=70))               # s odd: the last piece of c_x is part empty
    # an outlier buffer of more than 32 columns: the unguarded and the guarded kernel are both launched, the count
    # decides on the device which of them runs
    linear_compare(wl.make_custom(320, 384, 520, 5, seed=72), cap=64)       # 5 columns found: the unguarded one
    linear_compare(wl.make_custom(300, 320, 776, 29, seed=73), cap=48)      # 29: two fp16 k-steps from a 48-slot row
    linear_compare(wl.make_custom(320, 384, 520, 40, seed=74), cap=64)      # 40: the guarded one


@pytest.mark.parametrize("s", [2300, 2296])
@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5])
def test_workgroups_walk_full_and_ragged_tiles_in_turn(cfg, s, forced_tile):
    """A tile grid larger than the chip with ragged edges in both directions (2300 or 2296 tokens, 10 008
    columns: 360 to 1 422 tiles on 256 workgroups), so that a persistent workgroup goes from a full tile (its
    stores still in flight when the next tile starts) to one that reaches past the last token or column
    (operand requests clamped, stores cut off by the buffer bounds; with 2300 tokens the last piece of c_x is
    part empty) and back, for every tile shape.  Every output of llmint8_linear (unguarded epilogue) against
    the staged calls with the accumulator export (guarded epilogue), and samples of both against the oracle."""
    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(s, 384, 10008, 7, seed=71)
    X, W = d["X"], d["W"]
    o = 10008
    forced_tile(cfg)
    g = run_hip(X, W, d["alpha"], cap=32)
    idx = oracle.find_outliers(X, d["alpha"])
    assert g["idx"].tolist() == idx.tolist()
    for _ in range(2):
        out = L.linear(g["Xd"], g["qw"], d["alpha"], g["outl"], g["rows"], g["ws"])
    torch.cuda.synchronize()
    lin = out.cpu().numpy()
    scale = float(np.abs(g["Out"].astype(np.float64)).max())
    assert_out_close(lin, g["Out"], scale)
    rng = np.random.default_rng(5)
    ri = np.concatenate([rng.integers(0, s, 600), np.full(40, s - 1), rng.integers(2048, s, 100)])
    ci = np.concatenate([rng.integers(0, o, 600), rng.integers(0, o, 40), rng.integers(9984, o, 100)])
    Cs, Os = oracle.sampled(X, W, idx, ri, ci)
    assert np.array_equal(g["C"][ri, ci], Cs)
    assert_out_close(lin[ri, ci], Os, scale)
    assert_out_close(g["Out"][ri, ci], Os, scale)


@pytest.mark.parametrize("s,o", [(8, 64), (40, 96), (300, 264)])
def test_accumulator_at_the_int32_bound(s, o):
    """Section 2.1: the int8 products are accumulated as 32-bit integers.  At the largest feature dimension
    the library accepts (h = 133 144) with every code at +-127 the accumulator reaches h * 127^2 =
    2 147 479 576 = 2^31 - 4 072: weight-streaming path (s = 8) and tiled path (s = 40, 300), k-tile padding
    included, and the dequantization of a value that large."""
    import paper_2208_07339_amd as L
    h = 133144
    X = np.full((s, h), 1.0, np.float16)
    X[1::2] = -0.5                                   # odd tokens: codes -127, constant 0.5
    W = np.full((h, o), 0.25, np.float16)
    W[:, 1::3] = -0.125                              # every third column: codes -127, constant 0.125
    g = run_hip(X, W, 6.0, 32)
    assert g["count"] == 0
    sign = np.where(np.arange(s) % 2 == 1, -1, 1)[:, None] * np.where(np.arange(o) % 3 == 1, -1, 1)[None, :]
    want = (sign * (h * 16129)).astype(np.int64)
    assert want.max() == 2147479576 and want.min() == -2147479576
    assert np.array_equal(g["C"].astype(np.int64), want)
    Xq, cx = oracle.quantize_rows(X, np.zeros(0, np.int32))
    Wq, cw = oracle.quantize_weight(W)
    assert np.all(np.abs(Xq) == 127) and np.all(np.abs(Wq) == 127)
    assert np.array_equal(g["Xq"], Xq) and np.array_equal(hip_weight_i8(g["qw"]), Wq)
    rows = np.arange(min(s, 4))
    Cm = oracle.igemm(np.ascontiguousarray(Xq[rows]), Wq)
    assert np.array_equal(Cm.astype(np.int64), want[rows])
    ref = oracle.output(Cm, cx[rows], cw, np.ascontiguousarray(X[rows]), W, np.zeros(0, np.int32))
    assert_out_close(g["Out"][rows], ref)
    # closed form for all rows: Out = h * c_x * c_w with the signs, exactly representable products
    closed = want / 16129.0 * cx.astype(np.float64)[:, None] * cw.astype(np.float64)[None, :]
    assert_out_close(g["Out"], closed.astype(np.float16))
    # and through the one-call path (no accumulator export: the LDS-fed epilogue where o % 8 == 0)
    import torch
    out = L.linear(g["Xd"], g["qw"], 6.0, g["outl"], g["rows"], g["ws"])
    torch.cuda.synchronize()
    assert_out_close(out.cpu().numpy(), closed.astype(np.float16))


@pytest.mark.parametrize("s,h,o,ncol", [(33, 384, 32768, 3), (48, 200, 32800, 5), (41, 520, 40960, 20), (47, 64, 33000, 0),
                                        (49, 128, 32768, 2)])
def test_two_token_tiles_through_the_weight_streaming_kernel(s, h, o, ncol):
    """33 to 48 tokens against a weight matrix of at least 32 736 columns take the weight-streaming kernel with
    two token tiles per workgroup (narrower ones, and 49 tokens, go to the tiled kernel).  Every stage against
    the oracle, staged with the accumulator export and through the one-call path; the last column tiles are
    ragged."""
    d = wl.make_custom(s, h, o, ncol, seed=3 * s + ncol)
    full_compare(d)
    linear_compare(d)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_every_decode_work_split(cfg):
    import paper_2208_07339_amd as L
    L.debug_decode_shape(cfg)
    try:
        full_compare(wl.make_custom(16, 1024, 2048, 5, seed=1))
        full_compare(wl.make_custom(13, 200, 61, 2, seed=2))      # nothing aligned, last column tile ragged
        full_compare(wl.make_custom(32, 4160, 96 * 5, 20, seed=3))  # more outlier columns than are prefetched
        full_compare(wl.make_custom(7, 128 * 11, 64, 0, seed=4))  # odd number of k batches
    finally:
        L.debug_decode_shape(-1)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3, 4, 5])
def test_short_x_through_the_tiled_kernel(cfg, forced_tile):
    """32 tokens and fewer normally go to the weight-streaming kernel; for some shapes of W the library sends
    them to the tiled kernel instead (one 128 x 128 tile per compute unit beats two part-filled rounds of the
    other).  With the weight-streaming kernel switched off, every tile shape on 1 to 32 tokens: a single row
    tile of X repeated across the token tiles of a workgroup, all of them ragged; the staged calls with the
    accumulator export (guarded epilogue) and the one-call path (unguarded)."""
    import paper_2208_07339_amd as L
    forced_tile(cfg)
    L.debug_decode_shape(0)
    try:
        full_compare(wl.make_custom(16, 1024, 2048, 5, seed=1))
        full_compare(wl.make_custom(13, 200, 61, 2, seed=2))
        full_compare(wl.make_custom(1, 640, 520, 3, seed=5))
        linear_compare(wl.make_custom(32, 1152, 776, 20, seed=3))
        linear_compare(wl.make_custom(7, 512, 1544, 0, seed=4))
        linear_compare(wl.make_custom(1, 256, 264, 1, seed=6))
        linear_compare(wl.make_custom(24, 384, 768, 9, seed=7), cap=4)       # more columns qualify than fit
        int8_rows_compare(wl.make_custom(16, 512, 520, 6, seed=8), via_linear=True)
    finally:
        L.debug_decode_shape(-1)


def test_short_x_goes_to_the_tiled_kernel_where_w_has_two_to_four_column_tiles_per_compute_unit():
    """The library's own choice on such a W (640 column tiles, K = 256) and the weight-streaming kernel forced
    on the same buffers: both within tolerance of the oracle."""
    import torch

    import paper_2208_07339_amd as L
    s, h, o = 16, 256, 20480
    d = wl.make_custom(s, h, o, 3, seed=9)
    g = run_hip(d["X"], d["W"], d["alpha"], cap=32, want_c=False)
    outs = []
    try:
        for route in (-1, 1):
            L.debug_decode_shape(route)
            out = torch.zeros((s, o), dtype=torch.float16, device="cuda")
            L.linear(g["Xd"], g["qw"], d["alpha"], g["outl"], g["rows"], g["ws"], out)
            torch.cuda.synchronize()
            outs.append(out.cpu().numpy())
    finally:
        L.debug_decode_shape(-1)
    ref = oracle.linear(d["X"], d["W"], d["alpha"])
    assert_out_close(outs[0], ref["Out"])
    assert_out_close(outs[1], ref["Out"])


def test_alpha_zero_is_pure_fp16_matmul_on_both_paths():
    d = wl.make("tiny")
    g, r = full_compare(d, alpha=0.0, cap=256)
    assert g["count"] == 256 and not g["C"].any()
    d = wl.make_custom(40, 96, 64, 2, seed=5)
    g, r = full_compare(d, alpha=0.0, cap=96)
    assert g["count"] == 96


def test_alpha_infinity_is_vector_wise_only():
    d = wl.make("tiny")
    g, r = full_compare(d, alpha=float("inf"))
    assert g["count"] == 0
    full_compare(wl.make_custom(70, 256, 128, 3, seed=9), alpha=1e9)


def test_capacity_overflow_sets_status_and_clamps():
    d = wl.make_custom(48, 512, 96, 9, seed=21)
    X, W = d["X"], d["W"]
    full = oracle.find_outliers(X, 6.0)
    assert len(full) >= 9
    g = run_hip(X, W, 6.0, cap=4)
    assert g["status"] == 1 and g["count"] == 4
    assert g["idx"].tolist() == full[:4].tolist()
    # the rest of the pipeline treats exactly the reported columns as outliers
    Xq, cx = oracle.quantize_rows(X, full[:4])
    assert np.array_equal(g["Xq"], Xq) and np.array_equal(bits(g["cx"]), bits(cx))
    Wq, cw = oracle.quantize_weight(W)
    Cm = oracle.igemm(Xq, Wq)
    assert np.array_equal(g["C"], Cm)
    assert_out_close(g["Out"], oracle.output(Cm, cx, cw, X, W, full[:4]))


def test_zero_rows_and_zero_weight_columns():
    d = wl.make_custom(40, 256, 96, 2, seed=3)
    d["X"][5] = 0
    d["X"][39] = 0
    d["W"][:, 7] = 0
    d["W"][:, 95] = 0
    g, r = full_compare(d)
    assert g["cx"][5] == 0 and g["cw"][7] == 0
    assert not g["Out"][5].any() and not g["Out"][:, 7].any()


def test_row_made_only_of_outlier_columns():
    X = np.zeros((34, 64), np.float16)
    X[:, 3] = 9.0
    X[1, 10] = 1.0
    W = wl.make_w(64, 64, seed=8)
    d = dict(X=X, W=W, alpha=6.0)
    g, r = full_compare(d)
    assert g["idx"].tolist() == [3] and g["cx"][0] == 0


def test_threshold_boundary_values():
    X = wl.normal_f16(40, 128, 0.5, 17)
    X[3, 5] = 6.0
    X[7, 9] = -6.0
    X[9, 11] = np.nextafter(np.float16(6.0), np.float16(0))
    W = wl.make_w(128, 64, seed=18)
    g, r = full_compare(dict(X=X, W=W, alpha=6.0))
    assert g["idx"].tolist() == [5, 9]


def quantizer_sweep(lo, hi, xmax, neg):
    """Rows = the row constants lo .. hi-1 (fp16 bit patterns), columns = every magnitude 0 .. xmax that does
    not exceed the row's constant: codes and constants against the oracle, bit for bit."""
    import torch

    import paper_2208_07339_amd as L
    c = np.arange(lo, hi, dtype=np.int64)
    cols = np.arange(xmax + 1, dtype=np.int64)
    X = np.zeros((len(c), xmax + 2), np.uint16)
    X[:, 0] = c
    X[:, 1:] = np.where(cols[None, :] <= c[:, None], cols[None, :], 0).astype(np.uint16)
    if neg:
        X[:, 1:] |= 0x8000
    Xf = X.view(np.float16)
    want, cx = oracle.quantize_rows(Xf, np.zeros(0, np.int32))
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(Xd.shape[0], Xd.shape[1], 32, 16)
    outl = L.find_outliers(Xd, float("inf"), 16, ws)
    rows = L.quantize_rows(Xd, outl)
    got = L.export_rows(rows).cpu().numpy()
    assert np.array_equal(bits(rows.cx.cpu().numpy()), bits(cx))
    assert np.array_equal(got, want)


@pytest.mark.parametrize("first", range(0, 31, 4))
def test_quantizer_on_every_pair_of_fp16_values(first):
    """Exhaustive: every finite row constant c > 0 (31 binades of 1024 patterns, the subnormal one included)
    against every magnitude |x| <= c, the sign alternating by binade.  The quantizer divides through a
    reciprocal and a correction step; this is the proof that it still rounds the exact quotient."""
    for b in range(first, min(first + 4, 31)):
        lo, hi = max(1, b * 1024), (b + 1) * 1024
        quantizer_sweep(lo, hi, hi - 1, neg=bool(b & 1))


def test_weight_quantizer_sweep():
    """The same sweep through the column constants of llmint8_quantize_weight (one binade each of typical,
    subnormal and maximal constants)."""
    import torch

    import paper_2208_07339_amd as L
    for lo, hi in [(0x2000, 0x2400), (0x0001, 0x0400), (0x7800, 0x7C00)]:
        c = np.arange(lo, hi, dtype=np.int64)
        rowsv = np.arange(hi, dtype=np.int64)
        W = np.zeros((hi + 1, len(c)), np.uint16)
        W[0, :] = c
        W[1:, :] = np.where(rowsv[:, None] <= c[None, :], rowsv[:, None], 0).astype(np.uint16)
        W[1::2, :] |= 0x8000
        Wf = W.view(np.float16)
        want, cw = oracle.quantize_weight(Wf)
        Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
        qw = L.quantize_weight(Wd)
        assert np.array_equal(bits(qw.cw.cpu().numpy()), bits(cw))
        assert np.array_equal(hip_weight_i8(qw), want)


def test_two_runs_are_bit_identical():
    d = wl.make_custom(300, 1000, 520, 4, seed=99)
    a = run_hip(d["X"], d["W"], 6.0, 32)
    b = run_hip(d["X"], d["W"], 6.0, 32)
    for k in ("idx", "Xq", "C"):
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(bits(a["Out"]), bits(b["Out"]))
    assert np.array_equal(bits(a["cx"]), bits(b["cx"]))


def test_linear_entry_point_matches_step_by_step():
    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(100, 512, 256, 3, seed=41)
    g = run_hip(d["X"], d["W"], 6.0, 32, want_c=False)
    out = L.linear(g["Xd"], g["qw"], 6.0, g["outl"], g["rows"], g["ws"])
    torch.cuda.synchronize()
    assert np.array_equal(bits(out.cpu().numpy()), bits(g["Out"]))


def linear_compare(d, alpha=None, cap=32):
    """llmint8_linear (for s <= 32 it runs the fused two-kernel pre-pass) against the oracle, stage by stage."""
    import torch

    import paper_2208_07339_amd as L
    alpha = d["alpha"] if alpha is None else alpha
    X, W = d["X"], d["W"]
    s, h = X.shape
    o = W.shape[1]
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16)
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.quantize_weight(Wd, ws)
    outl = L.Outliers(torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda"), cap)
    rows = L.QuantizedRows(torch.full((L.xq_bytes(s, h),), 99, dtype=torch.int8, device="cuda"),
                           torch.full((s,), 7.0, dtype=torch.float16, device="cuda"),
                           torch.full((s, L.opad(cap)), 7.0, dtype=torch.float16, device="cuda"), s, h)
    for _ in range(2):  # twice: the scratch of the first call must not disturb the second
        out = L.linear(Xd, qw, alpha, outl, rows, ws)
    torch.cuda.synchronize()
    full = oracle.find_outliers(X, alpha)
    want_idx = full[:cap]
    n = int(outl.count.item())
    assert n == len(want_idx) and int(outl.status.item()) == (1 if len(full) > cap else 0)
    assert outl.idx[:n].cpu().numpy().tolist() == want_idx.tolist()
    Xq, cx = oracle.quantize_rows(X, want_idx)
    assert np.array_equal(bits(rows.cx.cpu().numpy()), bits(cx))
    assert np.array_equal(L.export_rows(rows).cpu().numpy(), Xq)
    Xo = rows.Xo.cpu().numpy()
    assert np.array_equal(bits(Xo[:, :n]), bits(X[:, want_idx])) and not bits(Xo[:, n:]).any()
    Wq, cw = oracle.quantize_weight(W)
    ref = oracle.output(oracle.igemm(Xq, Wq), cx, cw, X, W, want_idx)
    assert_out_close(out.cpu().numpy(), ref)


@pytest.mark.parametrize("s,h,o,ncol", [(1, 64, 32, 1), (16, 1024, 2048, 5), (13, 200, 61, 2), (32, 384, 96, 3),
                                        (8, 4160, 128, 6), (16, 12288, 256, 7), (32, 40000, 64, 5),
                                        (17, 70000, 32, 9), (9, 1100, 64, 3)])
def test_linear_short_x(s, h, o, ncol):
    linear_compare(wl.make_custom(s, h, o, ncol, seed=s * 11 + h))


def test_linear_prefill_sizes():
    """llmint8_linear for s > 32: the row constants and the quantizer read the scan's column lists."""
    linear_compare(wl.make_custom(100, 512, 256, 3, seed=41))
    linear_compare(wl.make_custom(300, 1000, 515, 4, seed=42))
    linear_compare(wl.make_custom(257, 4160, 264, 6, seed=43))
    linear_compare(wl.make_custom(70, 384, 96, 9, seed=44), cap=4)          # |O| > cap
    linear_compare(wl.make_custom(40, 96, 64, 2, seed=45), alpha=0.0, cap=96)  # every column
    linear_compare(wl.make_custom(64, 600, 64, 300, seed=46, frac=0.3), cap=300)  # a full list of 256
    linear_compare(wl.make_custom(48, 256, 64, 0, seed=47), alpha=float("inf"))


def test_linear_with_33_to_64_tokens():
    """Two row tiles of X, the smallest prefill shapes (and, against a wide W, the weight-streaming kernel with
    two token tiles).  Every stage of llmint8_linear against the oracle: ragged h, more qualifying columns than
    the buffer takes, every column an outlier, none, a row of zeros in the second tile, a long outlier buffer,
    and no 16-bit weights."""
    import dataclasses

    import torch

    import paper_2208_07339_amd as L
    linear_compare(wl.make_custom(33, 384, 96, 3, seed=81))
    linear_compare(wl.make_custom(64, 1000, 264, 5, seed=82))
    linear_compare(wl.make_custom(47, 4160, 64, 20, seed=83))
    linear_compare(wl.make_custom(50, 1536, 64, 9, seed=84), cap=4)       # |O| > cap
    linear_compare(wl.make_custom(40, 96, 64, 2, seed=85), alpha=0.0, cap=96)
    linear_compare(wl.make_custom(48, 256, 64, 0, seed=86), alpha=float("inf"))
    linear_compare(wl.make_custom(64, 600, 64, 300, seed=87, frac=0.3), cap=300)
    linear_compare(wl.make_custom(65, 512, 96, 3, seed=88))
    d = wl.make_custom(45, 512, 96, 2, seed=89)
    d["X"][37] = 0
    linear_compare(d)
    d = wl.make_custom(40, 520, 136, 6, seed=90)
    g = run_hip(d["X"], d["W"], d["alpha"], 32, want_c=False)
    qw = dataclasses.replace(g["qw"], W=None)
    staged = L.matmul(g["rows"], g["outl"], qw, g["ws"]).clone()
    out = L.linear(g["Xd"], qw, d["alpha"], g["outl"], g["rows"], g["ws"])
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), staged.view(torch.int16))


def test_linear_prefill_branches_of_the_prepass():
    """llmint8_linear for s > 32 on shapes that take every branch of its pre-pass: several row slabs, a single
    512-column block, ragged K, |O| > cap, every column an outlier, thousands of outlier columns (with and
    without overflow), rows that are all zero, no outlier at all."""
    linear_compare(wl.make_custom(100, 512, 256, 3, seed=41))
    linear_compare(wl.make_custom(300, 1000, 520, 4, seed=42))
    linear_compare(wl.make_custom(257, 4160, 264, 6, seed=43))
    linear_compare(wl.make_custom(2500, 320, 64, 5, seed=48))                 # 2 500 rows: three passes of a scan workgroup
    linear_compare(wl.make_custom(33, 64, 32, 1, seed=49))                    # one 64-column block
    linear_compare(wl.make_custom(50, 8, 16, 1, seed=50))                     # one 8-column chunk
    linear_compare(wl.make_custom(70, 384, 96, 9, seed=44), cap=4)            # |O| > cap
    linear_compare(wl.make_custom(40, 96, 64, 2, seed=45), alpha=0.0, cap=96)   # every column
    linear_compare(wl.make_custom(64, 600, 64, 300, seed=46, frac=0.3), cap=300)
    linear_compare(wl.make_custom(40, 2048, 64, 3, seed=81), alpha=0.0, cap=2048)   # 2 048 outlier columns
    linear_compare(wl.make_custom(40, 2048, 64, 3, seed=82), alpha=0.0, cap=1500)   # ... and |O| > cap on top
    linear_compare(wl.make_custom(48, 256, 64, 0, seed=47))
    d = wl.make_custom(200, 1024, 128, 4, seed=83)
    d["X"][7] = 0
    d["X"][199] = 0
    linear_compare(d)


def test_linear_row_maximum_inside_an_outlier_column():
    """Rows whose largest magnitude below alpha sits in an outlier column (alone, or tied with a regular
    column): the row constant must come from the regular columns only."""
    d = wl.make_custom(200, 1024, 128, 4, seed=51)
    X = d["X"]
    j0, j1 = int(d["planted"][0]), int(d["planted"][-1])
    free = [j for j in range(1024) if j not in set(d["planted"].tolist())]
    quiet = np.nonzero(np.abs(X[:, j0].astype(np.float32)) < 6.0)[0]
    assert len(quiet) >= 20
    X[quiet[:10], j0] = np.float16(5.5)            # alone at the top of the row
    X[quiet[10:15], j0] = np.float16(-5.75)
    X[quiet[10:15], free[3]] = np.float16(5.75)    # tied with a regular column
    X[quiet[15:20], j1] = np.float16(5.9)
    X[quiet[15:20], j0] = np.float16(5.9)          # two outlier columns share it
    linear_compare(d)
    linear_compare(d, cap=2)                        # ... and with the columns beyond cap counted as regular
    linear_compare(wl.make_custom(64, 333, 64, 3, seed=52))   # h not a multiple of 8: the three-pass pre-pass


def test_linear_short_x_degenerate_cases():
    linear_compare(wl.make("tiny"))
    linear_compare(wl.make("tiny"), alpha=0.0, cap=256)           # every column an outlier
    linear_compare(wl.make("tiny"), alpha=0.0, cap=100)           # ... and more of them than fit
    linear_compare(wl.make("tiny"), alpha=float("inf"))           # none
    linear_compare(wl.make_custom(24, 1536, 64, 9, seed=77), cap=4)   # |O| > cap: first cap columns only
    linear_compare(wl.make_custom(20, 1100, 64, 600, seed=78, frac=0.3), cap=700)  # lists longer than 512 per call
    d = wl.make_custom(12, 512, 96, 2, seed=79)
    d["X"][5] = 0
    linear_compare(d)


def test_rebuilt_outlier_rows_match_the_oracle_bit_for_bit():
    """llmint8_dequantize_rows: fp16(W_i8 * c_w / 127) in integer arithmetic on the GPU against the oracle's
    double-precision path, over column constants from the subnormal range to the largest fp16."""
    import torch

    import paper_2208_07339_amd as L
    rng = np.random.default_rng(3)
    h, o, cap = 160, 4096, 48
    W = wl.make_w(h, o, seed=31).astype(np.float32)
    scale = np.exp2(rng.integers(-19, 20, size=o)).astype(np.float32)  # 0.02 * 2^-19 .. 0.02 * 2^19
    W = np.clip(W * scale[None, :], -60000, 60000).astype(np.float16)
    W[:, 5] = 0
    W[3, 7] = 65504
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(64, h, o, cap)
    qw = L.quantize_weight(Wd, ws)
    Wq, cw = oracle.quantize_weight(W)
    assert np.array_equal(hip_weight_i8(qw), Wq)
    rows = np.sort(rng.choice(h, size=40, replace=False)).astype(np.int32)
    outl = L.Outliers(torch.zeros(cap, dtype=torch.int32, device="cuda"), torch.tensor([40], dtype=torch.int32, device="cuda"),
                      torch.zeros(1, dtype=torch.int32, device="cuda"), cap)
    outl.idx[:40] = torch.from_numpy(rows).cuda()
    got = L.dequantize_rows(qw, outl).cpu().numpy()
    want = oracle.dequant_rows(Wq, cw, rows)
    assert np.array_equal(bits(got[:40]), bits(want))
    assert not bits(got[40:]).any()
    assert np.isfinite(got.astype(np.float32)).all()
    sub = (np.abs(want.astype(np.float32)) < 6.2e-5) & (want != 0)
    assert sub.sum() > 100  # the subnormal branch was exercised


def int8_rows_compare(d, cap=32, via_linear=False):
    """The variant without 16-bit weights (W_f16 = NULL) against the oracle's int8-rows branch."""
    import dataclasses

    import torch

    import paper_2208_07339_amd as L
    X, W = d["X"], d["W"]
    g = run_hip(X, W, d["alpha"], cap, want_c=False)
    qw = dataclasses.replace(g["qw"], W=None)
    if via_linear:
        # (for s <= 32 the second pre-pass kernel rebuilds the rows itself: the same bits as the staged call)
        staged = L.matmul(g["rows"], g["outl"], qw, g["ws"]).clone()
        out = L.linear(g["Xd"], qw, d["alpha"], g["outl"], g["rows"], g["ws"])
        assert torch.equal(out.view(torch.int16), staged.view(torch.int16))
    else:
        out = L.matmul(g["rows"], g["outl"], qw, g["ws"])
    torch.cuda.synchronize()
    r = oracle.linear(X, W, d["alpha"])
    ref = oracle.output_dq(r["C"], r["cx"], r["cw"], X, r["Wq"], r["idx"][:cap])
    assert_out_close(out.cpu().numpy(), ref)
    # and it is a different result from the fp16-rows one wherever outliers contribute
    if len(r["idx"]):
        assert not np.array_equal(bits(out.cpu().numpy()), bits(g["Out"]))


@pytest.mark.parametrize("cap", [4, 300])
def test_int8_rows_one_call_equals_staged_calls_when_more_columns_qualify_than_fit(cap):
    """Short X, no 16-bit weights: the second pre-pass kernel of llmint8_linear rebuilds the rows of the first
    cap outlier columns from the column lists (cap = 4 < |O| = 9); with an outlier buffer of more than 256
    columns (cap = 300) it leaves that to llmint8_dequantize_rows, as llmint8_matmul always does via idx /
    count.  Same bits, and the rows are those of the oracle."""
    import dataclasses

    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(20, 520, 136, 9, seed=56)
    g = run_hip(d["X"], d["W"], d["alpha"], cap, want_c=False)
    assert int(g["outl"].status.item()) == (1 if cap == 4 else 0)
    qw = dataclasses.replace(g["qw"], W=None)
    staged = L.matmul(g["rows"], g["outl"], qw, g["ws"]).clone()
    out = L.linear(g["Xd"], qw, d["alpha"], g["outl"], g["rows"], g["ws"])
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), staged.view(torch.int16))
    O = oracle.find_outliers(d["X"], d["alpha"])[:cap]
    Xq, cx = oracle.quantize_rows(d["X"], O)
    Wq, cw = oracle.quantize_weight(d["W"])
    ref = oracle.output_dq(oracle.igemm(Xq, Wq), cx, cw, d["X"], Wq, O)
    assert_out_close(out.cpu().numpy(), ref)


@pytest.mark.parametrize("via_linear", [False, True])
def test_int8_rows_variant(via_linear):
    int8_rows_compare(wl.make("tiny"), via_linear=via_linear)
    int8_rows_compare(wl.make_custom(16, 1024, 2048, 5, seed=51), via_linear=via_linear)       # decode kernel
    int8_rows_compare(wl.make_custom(13, 200, 61, 2, seed=52), via_linear=via_linear)          # ... unaligned
    int8_rows_compare(wl.make_custom(512, 2048, 1024, 7, seed=53), via_linear=via_linear)      # prefill, LDS-fed epilogue
    int8_rows_compare(wl.make_custom(300, 1000, 515, 20, seed=54), via_linear=via_linear)      # prefill, guarded epilogue
    int8_rows_compare(wl.make_custom(300, 384, 520, 40, seed=55), cap=48, via_linear=via_linear)  # > 32 outlier columns


def test_argument_errors_are_reported_not_executed():
    import ctypes as C

    import paper_2208_07339_amd as L
    lib = L.lib()
    assert lib.llmint8_find_outliers(None, 4, 4, 6.0, None, 4, None, None, None, 0, None) == 1
    import torch
    X = torch.zeros((4, 8), dtype=torch.float16, device="cuda")
    idx = torch.zeros(8, dtype=torch.int32, device="cuda")
    p = lambda t: C.c_void_p(t.data_ptr())
    # workspace too small
    assert lib.llmint8_find_outliers(p(X), 4, 8, 6.0, p(idx), 8, p(idx), None, p(idx), 16, None) == 3
    # feature dimension above the int32 accumulation bound
    assert lib.llmint8_find_outliers(p(X), 1, 133145, 6.0, p(idx), 8, p(idx), None, p(idx), 1 << 30, None) == 2
    # cap < 1
    assert lib.llmint8_find_outliers(p(X), 4, 8, 6.0, p(idx), 0, p(idx), None, p(idx), 1 << 20, None) == 1
    with pytest.raises(L.Llmint8Error):
        L.binding._check(3)


def test_random_shapes_through_the_one_call_path():
    """Seeded random shapes on both sides of the 32-token split, aligned and ragged, with random outlier
    counts, capacities (some too small) and thresholds: llmint8_linear against the oracle, stage by stage."""
    rng = np.random.default_rng(20240607)
    for case in range(24):
        s = int(rng.choice([rng.integers(1, 33), rng.integers(33, 400)]))
        h = int(rng.choice([8 * rng.integers(4, 260), rng.integers(20, 1500)]))
        o = int(rng.choice([8 * rng.integers(2, 90), rng.integers(9, 600)]))
        ncol = int(rng.integers(0, min(h, 40)))
        cap = int(rng.choice([32, 16, 48, max(1, ncol // 2)]))
        alpha = float(rng.choice([6.0, 6.0, 4.5, 9.0]))
        d = wl.make_custom(s, h, o, ncol, seed=1000 + case)
        try:
            linear_compare(d, alpha=alpha, cap=cap)
        except AssertionError as e:
            raise AssertionError(f"case {case}: s={s} h={h} o={o} ncol={ncol} cap={cap} alpha={alpha}: {e}") from e


def test_every_tile_shape_gives_the_same_bits(forced_tile):
    """The accumulation is exact and every tile shape runs the same epilogue arithmetic per output, so the outputs
    of llmint8_linear must not depend on the tile shape, on the guarded or unguarded epilogue (o % 8, outlier
    buffer size), or on the number of columns found: seeded random shapes, every tile shape against the first,
    bit for bit; short X also through the tiled kernel with the weight-streaming kernel switched off."""
    import torch

    import paper_2208_07339_amd as L
    rng = np.random.default_rng(77)
    try:
        for case in range(10):
            s = int(rng.choice([rng.integers(1, 33), rng.integers(33, 700)]))
            h = int(8 * rng.integers(4, 200))
            o = int(rng.choice([8 * rng.integers(8, 200), rng.integers(60, 1500)]))
            ncol = int(rng.integers(0, 36))
            cap = int(rng.choice([32, 16, 64]))
            d = wl.make_custom(s, h, o, min(ncol, cap), seed=2000 + case)
            g = run_hip(d["X"], d["W"], d["alpha"], cap=cap, want_c=False)
            L.debug_decode_shape(0)
            ref = None
            for cfg in range(6):
                forced_tile(cfg)
                out = torch.zeros((s, o), dtype=torch.float16, device="cuda")
                L.linear(g["Xd"], g["qw"], d["alpha"], g["outl"], g["rows"], g["ws"], out)
                torch.cuda.synchronize()
                if ref is None:
                    ref = out
                    assert_out_close(out.cpu().numpy(), oracle.linear(d["X"], d["W"], d["alpha"])["Out"])
                else:
                    assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), \
                        f"case {case}: s={s} h={h} o={o} ncol={ncol} cap={cap}: tile {cfg} differs from tile 0"
                if cfg in (0, 3):  # the guarded epilogue (accumulator export) of two of the shapes as well
                    out2, _ = L.matmul(g["rows"], g["outl"], g["qw"], g["ws"], want_c_i32=True)
                    torch.cuda.synchronize()
                    assert torch.equal(out2.view(torch.int16), ref.view(torch.int16)), \
                        f"case {case}: s={s} h={h} o={o} ncol={ncol} cap={cap}: guarded epilogue of tile {cfg} differs"
            L.debug_decode_shape(-1)
    finally:
        L.debug_decode_shape(-1)


@pytest.mark.parametrize("s,h,o", [(16, 1024, 768), (200, 640, 384)])  # weight-streaming path, tiled path
def test_linear_replayed_from_a_captured_graph(s, h, o):
    """The one-call entry point allocates nothing and enqueues kernels only, so a caller may capture it
    in a graph: every replay, on new contents of X (other outlier columns, other constants), must give
    what the oracle gives, with the program's own eager work between the replays."""
    import torch

    import paper_2208_07339_amd as L
    cap = 32
    inputs = [wl.make_custom(s, h, o, n, seed=50 + n) for n in (3, 0, 6)]
    W = inputs[0]["W"]
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.quantize_weight(Wd, ws)
    Wq_ref, cw_ref = oracle.quantize_weight(W)
    Xd = torch.zeros((s, h), dtype=torch.float16, device="cuda")
    out = torch.zeros((s, o), dtype=torch.float16, device="cuda")
    outl = L.Outliers(torch.zeros(cap, dtype=torch.int32, device="cuda"),
                      torch.zeros(1, dtype=torch.int32, device="cuda"),
                      torch.zeros(1, dtype=torch.int32, device="cuda"), cap)
    rows = L.QuantizedRows(torch.zeros(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                           torch.zeros(s, dtype=torch.float16, device="cuda"),
                           torch.zeros((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h)
    L.linear(Xd, qw, 6.0, outl, rows, ws, out=out)   # once outside: one-time set-up (kernel attributes) is not captured
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        L.linear(Xd, qw, 6.0, outl, rows, ws, out=out)
    for d in inputs + inputs[:1]:
        X = d["X"]
        Xd.copy_(torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16))   # eager work between replays
        out.fill_(7.0)
        graph.replay()
        torch.cuda.synchronize()
        idx = oracle.find_outliers(X, 6.0)
        n = int(outl.count.item())
        assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
        Xq, cx = oracle.quantize_rows(X, idx)
        assert np.array_equal(bits(rows.cx.cpu().numpy()), bits(cx))
        assert np.array_equal(L.export_rows(rows).cpu().numpy(), Xq)
        ref = oracle.output(oracle.igemm(Xq, Wq_ref), cx, cw_ref, X, W, idx)
        assert_out_close(out.cpu().numpy(), ref)


@pytest.mark.parametrize("s,h,o,ncol", [(1, 1, 1, 0), (1, 1, 1, 1), (1, 3, 7, 1), (2, 5, 5, 2), (3, 2, 1, 0), (31, 7, 9, 3),
                                        (33, 1, 1, 0), (33, 1, 2, 1), (40, 7, 3, 2), (64, 3, 9, 1), (70, 9, 1, 4)])
def test_smallest_dimensions(s, h, o, ncol):
    """One feature, one output column, one token, on both sides of the 32-token split: everything is padding."""
    linear_compare(wl.make_custom(s, h, o, ncol, seed=7 * s + h + o))
    zp = oracle.zp_linear  # the zeropoint variant on the same inputs
    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(s, h, o, ncol, seed=7 * s + h + o)
    X, W = d["X"], d["W"]
    ref = zp(X, W, 6.0)
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16)
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, 32)
    qw = L.zp_quantize_weight(Wd, ws)
    outl = L.find_outliers(Xd, 6.0, 32, ws)
    rows = L.zp_quantize_rows(Xd, outl)
    out, Cd = L.zp_matmul(rows, outl, qw, ws, want_c_i32=True)
    torch.cuda.synchronize()
    assert np.array_equal(Cd.cpu().numpy(), ref["C"])
    assert_out_close(out.cpu().numpy(), ref["Out"])


def test_calls_on_two_streams_with_their_own_workspaces_do_not_disturb_each_other():
    """The library keeps no state between calls: two streams, each with its own inputs, buffers and
    workspace, issue their calls interleaved (a tiled-path call next to a weight-streaming one, so that
    kernels of both are in flight together); every output is what the oracle gives for its own input."""
    import torch

    import paper_2208_07339_amd as L
    cap = 32
    jobs = []
    for (s, h, o, ncol, seed) in [(300, 1024, 768, 4, 1), (16, 4096, 1024, 6, 2)]:
        d = wl.make_custom(s, h, o, ncol, seed=seed)
        st = torch.cuda.Stream()
        with torch.cuda.stream(st):
            Xd = torch.from_numpy(d["X"].view(np.int16)).cuda().view(torch.float16)
            Wd = torch.from_numpy(d["W"].view(np.int16)).cuda().view(torch.float16)
            ws = L.Workspace.allocate(s, h, o, cap)
            qw = L.quantize_weight(Wd, ws)
            outl = L.Outliers(torch.zeros(cap, dtype=torch.int32, device="cuda"),
                              torch.zeros(1, dtype=torch.int32, device="cuda"),
                              torch.zeros(1, dtype=torch.int32, device="cuda"), cap)
            rows = L.QuantizedRows(torch.zeros(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                                   torch.zeros(s, dtype=torch.float16, device="cuda"),
                                   torch.zeros((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h)
            outs = [torch.zeros((s, o), dtype=torch.float16, device="cuda") for _ in range(6)]
        jobs.append(dict(d=d, st=st, Xd=Xd, qw=qw, ws=ws, outl=outl, rows=rows, outs=outs))
    torch.cuda.synchronize()
    for k in range(6):
        for j in jobs:
            with torch.cuda.stream(j["st"]):
                L.linear(j["Xd"], j["qw"], 6.0, j["outl"], j["rows"], j["ws"], out=j["outs"][k])
    torch.cuda.synchronize()
    for j in jobs:
        ref = oracle.linear(j["d"]["X"], j["d"]["W"], 6.0)
        for out in j["outs"]:
            assert_out_close(out.cpu().numpy(), ref["Out"])
        assert np.array_equal(bits(j["rows"].cx.cpu().numpy()), bits(ref["cx"]))


def test_calls_from_two_host_threads():
    """The library may be called from several threads (its one-time per-device set-up is taken under a lock):
    two threads, each with its own stream, inputs and workspace, call llmint8_linear concurrently (ctypes
    releases the interpreter lock during the call); every output is what the oracle gives for its input."""
    import threading

    import torch

    import paper_2208_07339_amd as L
    cap = 32
    jobs, errors = [], []
    for (s, h, o, ncol, seed) in [(300, 1024, 768, 4, 11), (200, 640, 520, 3, 12)]:
        d = wl.make_custom(s, h, o, ncol, seed=seed)
        Xd = torch.from_numpy(d["X"].view(np.int16)).cuda().view(torch.float16)
        Wd = torch.from_numpy(d["W"].view(np.int16)).cuda().view(torch.float16)
        ws = L.Workspace.allocate(s, h, o, cap)
        qw = L.quantize_weight(Wd, ws)
        outl = L.Outliers(torch.zeros(cap, dtype=torch.int32, device="cuda"),
                          torch.zeros(1, dtype=torch.int32, device="cuda"),
                          torch.zeros(1, dtype=torch.int32, device="cuda"), cap)
        rows = L.QuantizedRows(torch.zeros(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                               torch.zeros(s, dtype=torch.float16, device="cuda"),
                               torch.zeros((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h)
        out = torch.zeros((s, o), dtype=torch.float16, device="cuda")
        jobs.append(dict(d=d, Xd=Xd, qw=qw, ws=ws, outl=outl, rows=rows, out=out, st=torch.cuda.Stream()))
    torch.cuda.synchronize()

    def work(j):
        try:
            with torch.cuda.stream(j["st"]):
                for _ in range(50):
                    L.linear(j["Xd"], j["qw"], 6.0, j["outl"], j["rows"], j["ws"], out=j["out"])
            j["st"].synchronize()
        except Exception as e:  # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(j,)) for j in jobs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for j in jobs:
        ref = oracle.linear(j["d"]["X"], j["d"]["W"], 6.0)
        assert_out_close(j["out"].cpu().numpy(), ref["Out"])
        assert np.array_equal(bits(j["rows"].cx.cpu().numpy()), bits(ref["cx"]))


def test_graph_capture_after_init_only_in_a_fresh_process():
    """llmint8_init does the whole per-device set-up, so a process may capture its very first call of any
    shape: a fresh interpreter calls llmint8_init, captures llmint8_linear for a tiled shape and for a
    weight-streaming shape without any eager call before, replays each twice and compares with an eager call."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r'''
import numpy as np, torch, sys
sys.path.insert(0, %r)
import paper_2208_07339_amd as L
from paper_2208_07339_amd import workloads as wl
torch.cuda.init()
L.init()
cap = 32
for (s, h, o) in [(300, 640, 776), (16, 1024, 768)]:
    d = wl.make_custom(s, h, o, 4, seed=5)
    Xd = torch.from_numpy(d["X"].view(np.int16)).cuda().view(torch.float16)
    Wd = torch.from_numpy(d["W"].view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.quantize_weight(Wd, ws)
    mk = lambda: (L.Outliers(torch.zeros(cap, dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"),
                             torch.zeros(1, dtype=torch.int32, device="cuda"), cap),
                  L.QuantizedRows(torch.zeros(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"), torch.zeros(s, dtype=torch.float16, device="cuda"),
                                  torch.zeros((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h),
                  torch.zeros((s, o), dtype=torch.float16, device="cuda"))
    outl, rows, out = mk()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        L.linear(Xd, qw, 6.0, outl, rows, ws, out=out)
    res = []
    for _ in range(2):
        out.fill_(7.0)
        g.replay()
        torch.cuda.synchronize()
        res.append(out.clone())
    outl2, rows2, out2 = mk()
    L.linear(Xd, qw, 6.0, outl2, rows2, ws, out=out2)
    torch.cuda.synchronize()
    assert torch.equal(res[0].view(torch.int16), out2.view(torch.int16)) and torch.equal(res[1].view(torch.int16), out2.view(torch.int16))
    assert out2.abs().max().item() > 0
print("graph after init ok")
''' % root
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "graph after init ok" in r.stdout, r.stdout + r.stderr


@pytest.mark.parametrize("s", [16, 300])
def test_non_finite_inputs_do_not_fault(s):
    """NaN / Inf in X or W are outside the contract (results unspecified) but must not fault: both paths run to
    completion, the columns of X that hold them count as outlier columns (their magnitude bits reach any
    threshold), and outputs whose row of X and column of W are finite stay finite."""
    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(s, 512, 256, 3, seed=97)
    X, W = d["X"].copy(), d["W"].copy()
    X[2, 100] = np.float16("nan")
    X[5, 300] = np.float16("inf")
    X[7, 301] = -np.float16("inf")
    W[40, 9] = np.float16("inf")
    W[41, 200] = np.float16("nan")
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16)
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    cap = 32
    ws = L.Workspace.allocate(s, 512, 256, cap)
    qw = L.quantize_weight(Wd, ws)
    outl = L.Outliers(torch.zeros(cap, dtype=torch.int32, device="cuda"), torch.zeros(1, dtype=torch.int32, device="cuda"),
                      torch.zeros(1, dtype=torch.int32, device="cuda"), cap)
    rows = L.QuantizedRows(torch.zeros(L.xq_bytes(s, 512), dtype=torch.int8, device="cuda"),
                           torch.zeros(s, dtype=torch.float16, device="cuda"),
                           torch.zeros((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, 512)
    out = L.linear(Xd, qw, 6.0, outl, rows, ws)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    got = set(outl.idx[:n].cpu().numpy().tolist())
    assert {100, 300, 301} <= got and set(d["planted"].tolist()) <= got
    o = out.cpu().numpy().astype(np.float32)
    clean_rows = [i for i in range(s) if i not in (2, 5, 7)]
    clean_cols = [j for j in range(256) if j not in (9, 200)]
    assert np.isfinite(o[np.ix_(clean_rows, clean_cols)]).all()
