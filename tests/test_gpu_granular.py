"""HIP path vs CPU oracle for the baselines of Table 1 with coarser absmax constants (row-wise:
one constant for all of W; tensor-wise: also one for all of X), with and without the decomposition
of Section 3.2.  Integer stages bit for bit, outputs within 1e-3 of the largest output."""
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


def granular_compare(d, mode, alpha, cap=32):
    """Both ways through the library (the staged calls, which also give the int32 accumulators, and
    llmint8_linear_granular) against oracle.linear_granular."""
    import torch

    import paper_2208_07339_amd as L
    X, W = d["X"], d["W"]
    s, h = X.shape
    o = W.shape[1]
    ref = oracle.linear_granular(X, W, alpha, mode)
    assert len(ref["idx"]) <= cap
    Xd, Wd = upload(X, W)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.quantize_weight(Wd, ws, granularity=mode)
    assert np.array_equal(bits(qw.cw.cpu().numpy()), bits(ref["cw"]))
    assert np.array_equal(L.export_weight(qw).cpu().numpy(), ref["Wq"])
    # staged
    outl = L.find_outliers(Xd, alpha, cap, ws)
    rows = L.quantize_rows(Xd, outl, granularity=mode)
    out, Cd = L.matmul(rows, outl, qw, ws, want_c_i32=True)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == ref["idx"].tolist()
    assert np.array_equal(bits(rows.cx.cpu().numpy()), bits(ref["cx"]))
    assert np.array_equal(L.export_rows(rows).cpu().numpy(), ref["Xq"])
    assert np.array_equal(Cd.cpu().numpy(), ref["C"])
    assert_out_close(out.cpu().numpy(), ref["Out"])
    # one call, into buffers holding junk; twice, as the second call meets the first one's scratch
    outl2 = L.Outliers(torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                       torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                       torch.full((1,), -7, dtype=torch.int32, device="cuda"), cap)
    rows2 = L.QuantizedRows(torch.full((L.xq_bytes(s, h),), 99, dtype=torch.int8, device="cuda"),
                            torch.full((s,), 7.0, dtype=torch.float16, device="cuda"),
                            torch.full((s, L.opad(cap)), 7.0, dtype=torch.float16, device="cuda"), s, h)
    for _ in range(2):
        out2 = L.linear(Xd, qw, alpha, outl2, rows2, ws, granularity=mode)
    torch.cuda.synchronize()
    assert int(outl2.count.item()) == len(ref["idx"]) and int(outl2.status.item()) == 0
    assert outl2.idx[:n].cpu().numpy().tolist() == ref["idx"].tolist()
    assert np.array_equal(bits(rows2.cx.cpu().numpy()), bits(ref["cx"]))
    assert np.array_equal(L.export_rows(rows2).cpu().numpy(), ref["Xq"])
    assert_out_close(out2.cpu().numpy(), ref["Out"])


SHAPES = [(8, 256, 512, 2), (16, 1024, 2048, 5), (13, 200, 61, 2), (32, 4160, 96, 6),   # weight-streaming path
          (33, 64, 32, 1), (100, 300, 200, 3), (256, 1024, 512, 4), (333, 520, 260, 5)]  # tiled path


@pytest.mark.parametrize("mode", ["rowwise", "tensorwise"])
@pytest.mark.parametrize("alpha", [6.0, INF])
@pytest.mark.parametrize("s,h,o,ncol", SHAPES)
def test_granular_baselines(s, h, o, ncol, alpha, mode):
    d = wl.make_custom(s, h, o, ncol, seed=3 * s + h)
    X = d["X"].copy()
    X[s // 2] *= np.float16(0.125)  # a row far below the others: its codes depend on the granularity
    d["X"] = X
    granular_compare(d, mode, alpha)


def test_vectorwise_through_the_granular_entry_points():
    """Granularity 0 of the new entry points is the method itself."""
    import torch

    import paper_2208_07339_amd as L
    d = wl.make_custom(70, 384, 160, 3, seed=9)
    Xd, Wd = upload(d["X"], d["W"])
    s, h, o, cap = 70, 384, 160, 32
    ws = L.Workspace.allocate(s, h, o, cap)
    Wq = torch.empty(L.wq_bytes(h, o), dtype=torch.int8, device="cuda")
    cw = torch.empty(o, dtype=torch.float16, device="cuda")
    lib, p = L.lib(), lambda t: t.data_ptr()
    st = torch.cuda.current_stream().cuda_stream
    assert lib.llmint8_quantize_weight_granular(p(Wd), h, o, 0, p(Wq), p(cw), p(ws.buf), ws.nbytes, st) == 0
    qw = L.quantize_weight(Wd, ws)
    torch.cuda.synchronize()
    assert torch.equal(Wq, qw.Wq) and torch.equal(cw, qw.cw)
    ref = oracle.linear(d["X"], d["W"], 6.0)
    assert np.array_equal(bits(cw.cpu().numpy()), bits(ref["cw"]))


def test_unknown_granularity_is_an_argument_error():
    import torch

    import paper_2208_07339_amd as L
    W = torch.zeros((64, 32), dtype=torch.float16, device="cuda")
    ws = L.Workspace.allocate(1, 64, 32, 1)
    Wq = torch.empty(L.wq_bytes(64, 32), dtype=torch.int8, device="cuda")
    cw = torch.empty(32, dtype=torch.float16, device="cuda")
    for g in (-1, 3):
        r = L.lib().llmint8_quantize_weight_granular(W.data_ptr(), 64, 32, g, Wq.data_ptr(), cw.data_ptr(),
                                                     ws.buf.data_ptr(), ws.nbytes, None)
        assert r == 1  # LLMINT8_INVALID_ARG, nothing enqueued


def test_all_zero_inputs_give_zero_constants_and_outputs():
    import paper_2208_07339_amd as L
    X = np.zeros((40, 128), np.float16)
    W = np.zeros((128, 64), np.float16)
    for mode in ("rowwise", "tensorwise"):
        granular_compare(dict(X=X, W=W), mode, 6.0)
    assert L is not None


@pytest.mark.parametrize("mode,alpha", [("rowwise", INF), ("tensorwise", 6.0)])
def test_prefill_13b_ffn_up_full_size(mode, alpha):
    """Full benchmark size: every constant and both int8 tensors in full, accumulators and outputs on
    random samples the oracle computes one by one."""
    import torch

    import paper_2208_07339_amd as L
    d = wl.make("ffn13b")
    X, W = d["X"], d["W"]
    s, h, o, cap = d["s"], d["h"], d["o"], 32
    Xd, Wd = upload(X, W)
    ws = L.Workspace.allocate(s, h, o, cap)
    qw = L.quantize_weight(Wd, ws, granularity=mode)
    outl = L.Outliers(torch.empty(cap, dtype=torch.int32, device="cuda"),
                      torch.empty(1, dtype=torch.int32, device="cuda"),
                      torch.empty(1, dtype=torch.int32, device="cuda"), cap)
    rows = L.QuantizedRows(torch.empty(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                           torch.empty(s, dtype=torch.float16, device="cuda"),
                           torch.empty((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h)
    out = L.linear(Xd, qw, alpha, outl, rows, ws, granularity=mode)
    _, Cd = L.matmul(rows, outl, qw, ws, want_c_i32=True)
    torch.cuda.synchronize()
    idx = oracle.find_outliers(X, alpha)
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    Wq, cw = oracle.quantize_weight_tensor(W)
    assert np.array_equal(bits(qw.cw.cpu().numpy()), bits(cw))
    assert np.array_equal(L.export_weight(qw).cpu().numpy(), Wq)
    Xq, cx = (oracle.quantize_rows_tensor if mode == "tensorwise" else oracle.quantize_rows)(X, idx)
    assert np.array_equal(bits(rows.cx.cpu().numpy()), bits(cx))
    assert np.array_equal(L.export_rows(rows).cpu().numpy(), Xq)
    rng = np.random.default_rng(77)
    ri, ci = rng.integers(0, s, 1200), rng.integers(0, o, 1200)
    Cs, Os = oracle.sampled_granular(X, W, idx, ri, ci, mode)
    assert np.array_equal(Cd.cpu().numpy()[ri, ci], Cs)
    assert_out_close(out.cpu().numpy()[ri, ci], Os, float(np.abs(Os.astype(np.float64)).max()))


def test_granular_with_rows_rebuilt_from_the_codes():
    """The coarser constants combine with the variant that keeps no 16-bit weights (W_f16 = NULL): the
    rebuilt rows use the shared constant."""
    import dataclasses

    import torch

    import paper_2208_07339_amd as L
    for (s, h, o), mode in (((16, 512, 256), "tensorwise"), ((120, 384, 192), "rowwise")):
        d = wl.make_custom(s, h, o, 4, seed=s + 7)
        X, W, cap = d["X"], d["W"], 32
        ref = oracle.linear_granular(X, W, 6.0, mode)
        want = oracle.output_dq(ref["C"], ref["cx"], ref["cw"], X, ref["Wq"], ref["idx"])
        Xd, Wd = upload(X, W)
        ws = L.Workspace.allocate(s, h, o, cap)
        qw = dataclasses.replace(L.quantize_weight(Wd, ws, granularity=mode), W=None)
        outl = L.Outliers(torch.empty(cap, dtype=torch.int32, device="cuda"),
                          torch.empty(1, dtype=torch.int32, device="cuda"),
                          torch.empty(1, dtype=torch.int32, device="cuda"), cap)
        rows = L.QuantizedRows(torch.empty(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                               torch.empty(s, dtype=torch.float16, device="cuda"),
                               torch.empty((s, L.opad(cap)), dtype=torch.float16, device="cuda"), s, h)
        out = L.linear(Xd, qw, 6.0, outl, rows, ws, granularity=mode)
        torch.cuda.synchronize()
        assert_out_close(out.cpu().numpy(), want)


def test_granularity_argument_errors():
    import ctypes as C

    import torch

    import paper_2208_07339_amd as L
    lib = L.lib()
    p = lambda t: C.c_void_p(t.data_ptr())
    X = torch.zeros((4, 64), dtype=torch.float16, device="cuda")
    Xq = torch.empty(L.xq_bytes(4, 64), dtype=torch.int8, device="cuda")
    idx = torch.zeros(16, dtype=torch.int32, device="cuda")
    cx = torch.zeros(4, dtype=torch.float16, device="cuda")
    Xo = torch.zeros((4, 16), dtype=torch.float16, device="cuda")
    for g in (-1, 3, 100):
        assert lib.llmint8_quantize_rows_granular(p(X), 4, 64, p(idx), p(idx), 16, g, p(Xq), p(cx), p(Xo), None) == 1
    assert lib.llmint8_quantize_rows_granular(p(X), 4, 64, p(idx), p(idx), 16, 2, p(Xq), p(cx), p(Xo), None) == 0
    torch.cuda.synchronize()


def test_random_shapes():
    """Seeded random shapes, granularities and thresholds on both GEMM paths against the oracle."""
    rng = np.random.default_rng(20240612)
    for case in range(16):
        s = int(rng.choice([rng.integers(1, 33), rng.integers(33, 300)]))
        h = int(rng.choice([8 * rng.integers(4, 200), rng.integers(20, 1200)]))
        o = int(rng.choice([8 * rng.integers(2, 80), rng.integers(9, 500)]))
        ncol = int(rng.integers(0, min(h, 20)))
        mode = str(rng.choice(["rowwise", "tensorwise"]))
        alpha = float(rng.choice([6.0, 6.0, INF]))
        d = wl.make_custom(s, h, o, ncol, seed=3000 + case)
        try:
            granular_compare(d, mode, alpha)
        except AssertionError as e:
            raise AssertionError(f"case {case}: s={s} h={h} o={o} ncol={ncol} {mode} alpha={alpha}: {e}") from e
