"""llmint8_linear_static, the entry point that allocates nothing (scratch in a static device array of
the library), against llmint8_linear with a caller's workspace: two calls in a row on the same GPU, the
second with a smaller input, so that whatever the first call left in the shared scratch lies under
the second; then a larger one again, both GEMM paths, and the size limit."""
import numpy as np
import pytest

import oracle
from paper_2208_07339_amd import workloads as wl
from gpu_util import assert_out_close, bits

pytestmark = pytest.mark.gpu

CAP = 32


def buffers(L, s, h, o):
    import torch
    outl = L.Outliers(torch.full((CAP,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda"), CAP)
    rows = L.QuantizedRows(torch.full((L.xq_bytes(s, h),), 99, dtype=torch.int8, device="cuda"),
                           torch.full((s,), 7.0, dtype=torch.float16, device="cuda"),
                           torch.full((s, L.opad(CAP)), 7.0, dtype=torch.float16, device="cuda"), s, h)
    out = torch.full((s, o), 7.0, dtype=torch.float16, device="cuda")
    return outl, rows, out


def both_ways(d, alpha=6.0, int8_rows=False):
    """One input through llmint8_linear (own workspace) and through llmint8_linear_static; returns the
    static call's results after checking them against the other's bit for bit and against the oracle."""
    import dataclasses

    import torch

    import paper_2208_07339_amd as L
    X, W = d["X"], d["W"]
    s, h = X.shape
    o = W.shape[1]
    Xd = torch.from_numpy(X.view(np.int16)).cuda().view(torch.float16)
    Wd = torch.from_numpy(W.view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, CAP)
    qw = L.quantize_weight(Wd, ws)
    if int8_rows:
        qw = dataclasses.replace(qw, W=None)
    a_outl, a_rows, a_out = buffers(L, s, h, o)
    b_outl, b_rows, b_out = buffers(L, s, h, o)
    L.linear(Xd, qw, alpha, a_outl, a_rows, ws, out=a_out)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    L.linear_static(Xd, qw, alpha, b_outl, b_rows, b_out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    n = int(a_outl.count.item())
    assert int(b_outl.count.item()) == n and int(b_outl.status.item()) == int(a_outl.status.item())
    assert torch.equal(a_outl.idx[:n], b_outl.idx[:n])
    assert torch.equal(a_rows.cx.view(torch.int16), b_rows.cx.view(torch.int16))
    assert torch.equal(a_rows.Xq, b_rows.Xq)
    assert torch.equal(a_rows.Xo.view(torch.int16), b_rows.Xo.view(torch.int16))
    assert torch.equal(a_out.view(torch.int16), b_out.view(torch.int16))
    # and against the oracle (integer stages bit-exact, outputs within 1e-3 * max|Out|)
    full = oracle.find_outliers(X, alpha)
    idx = full[:CAP]
    assert b_outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    Xq, cx = oracle.quantize_rows(X, idx)
    assert np.array_equal(bits(b_rows.cx.cpu().numpy()), bits(cx))
    assert np.array_equal(L.export_rows(b_rows).cpu().numpy(), Xq)
    Wq, cw = oracle.quantize_weight(W)
    Cm = oracle.igemm(Xq, Wq)
    ref = oracle.output_dq(Cm, cx, cw, X, Wq, idx) if int8_rows else oracle.output(Cm, cx, cw, X, W, idx)
    assert_out_close(b_out.cpu().numpy(), ref)


def test_two_calls_in_a_row_the_second_smaller():
    import paper_2208_07339_amd as L
    L.init()
    both_ways(wl.make_custom(600, 4160, 776, 20, seed=71))     # tiled path, 17 lists, ragged tiles
    both_ways(wl.make_custom(70, 384, 96, 3, seed=72))         # smaller: 2 lists, lies inside the first call's scratch
    both_ways(wl.make_custom(16, 1024, 2048, 5, seed=73))      # weight-streaming path and the short pre-pass
    both_ways(wl.make_custom(9, 200, 61, 2, seed=74))          # smaller again, nothing aligned
    both_ways(wl.make_custom(300, 1000, 520, 4, seed=75), int8_rows=True)   # outlier rows rebuilt into the scratch
    both_ways(wl.make_custom(40, 256, 64, 2, seed=76), int8_rows=True)
    both_ways(wl.make_custom(300, 1000, 520, 40, seed=77))     # more outlier columns than cap
    both_ways(wl.make_custom(48, 256, 64, 0, seed=78), alpha=float("inf"))


def test_sizes_beyond_the_static_scratch_are_refused():
    import ctypes as C

    import torch

    import paper_2208_07339_amd as L
    s, h, o = 64, 64, 1 << 20
    assert L.workspace_bytes(s, h, o, CAP) > L.STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.int32, device="cuda")
    p = C.c_void_p(t.data_ptr())
    # the pointers are never touched: the size check comes first and nothing is enqueued
    rc = L.lib().llmint8_linear_static(p, s, h, C.c_float(6.0), p, p, p, o, p, CAP, p, p, p, p, p, p, None)
    assert rc == 5
    torch.cuda.synchronize()
    assert not t.any()
