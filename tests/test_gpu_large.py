"""Shapes in which one tensor has more than 2^31 elements (X, then Out, then W): every offset past
that bound must be computed in 64 bits.  The inputs repeat a random block with power-of-two row
scales, so that rows one 2^31-element wrap apart differ, and carry planted values in the far part;
the oracle computes rows, columns and outputs sampled around and beyond the bound."""
import numpy as np
import pytest

import oracle
from gpu_util import assert_out_close, bits

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

CAP = 32


def tiled_matrix(rows, cols, block, sigma, seed):
    """M[r] = B[r % block] * 2^-((r // block) % 4) with B ~ N(0, sigma^2) in fp16 (the scaling is exact)."""
    rng = np.random.default_rng(seed)
    B = (rng.standard_normal((block, cols), dtype=np.float32) * sigma).astype(np.float16)
    scaled = [(B.astype(np.float32) * 2.0 ** -e).astype(np.float16) for e in range(4)]
    M = np.empty((rows, cols), np.float16)
    for b0 in range(0, rows, block):
        n = min(block, rows - b0)
        M[b0:b0 + n] = scaled[(b0 // block) % 4][:n]
    return M


def upload(a):
    import torch
    return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)


def buffers(L, s, h):
    import torch
    outl = L.Outliers(torch.empty(CAP, dtype=torch.int32, device="cuda"),
                      torch.empty(1, dtype=torch.int32, device="cuda"),
                      torch.empty(1, dtype=torch.int32, device="cuda"), CAP)
    rows = L.QuantizedRows(torch.empty(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                           torch.empty(s, dtype=torch.float16, device="cuda"),
                           torch.empty((s, L.opad(CAP)), dtype=torch.float16, device="cuda"), s, h)
    return outl, rows


def sample_rows(rng, s, wrap, n):
    """Rows at the start, around the row where the element offset passes 2^31, at the end, and random."""
    fixed = np.r_[0:8, wrap - 40:wrap + 40, s - 40:s]
    return np.unique(np.r_[fixed, rng.integers(0, s, n)]).astype(np.int64)


@pytest.fixture(scope="module")
def big_x():
    """X with s * h > 2^31 (host and device), a small W, and the outlier columns of X."""
    s, h, o, block = 66000, 32768, 64, 2048
    assert s * h > 2 ** 31
    X = tiled_matrix(s, h, block, 1.0, 1)
    planted = {(10, 3): -9.0, (65900, 777): 20.0, (s - 1, h - 1): 7.5, (40000, 20001): 6.0}
    for (i, j), v in planted.items():
        X[i, j] = v
    W = (np.random.default_rng(2).standard_normal((h, o), dtype=np.float32) * 0.02).astype(np.float16)
    # The rows outside the first block are scaled-down copies of it, apart from the planted values: the
    # first block and the planted rows decide every column maximum.
    decisive = np.r_[0:block, sorted({i for i, _ in planted})]
    idx = oracle.find_outliers(np.ascontiguousarray(X[decisive]), 6.0)
    assert {3, 777, 20001, h - 1} <= set(idx.tolist()) and len(idx) <= CAP
    return X, W, idx, upload(X), upload(W)


def test_more_than_2_31_elements_in_x(big_x):
    import torch

    import paper_2208_07339_amd as L
    X, W, idx, Xd, Wd = big_x
    (s, h), o = X.shape, W.shape[1]
    ws = L.Workspace.allocate(s, h, o, CAP)
    qw = L.quantize_weight(Wd, ws)
    outl, rows = buffers(L, s, h)
    out = L.linear(Xd, qw, 6.0, outl, rows, ws)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert int(outl.status.item()) == 0
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()

    rng = np.random.default_rng(3)
    rsel = sample_rows(rng, s, 2 ** 31 // h, 1500)
    Xq_ref, cx_ref = oracle.quantize_rows(np.ascontiguousarray(X[rsel]), idx)
    rsel_d = torch.from_numpy(rsel).cuda()
    assert np.array_equal(bits(rows.cx[rsel_d].cpu().numpy()), bits(cx_ref))
    assert np.array_equal(L.export_rows(rows)[rsel_d].cpu().numpy(), Xq_ref)
    Xo = rows.Xo[rsel_d].cpu().numpy()
    assert np.array_equal(bits(Xo[:, :n]), bits(X[rsel][:, idx])) and not Xo[:, n:].any()
    ri = np.repeat(rsel[::4], 4)
    ci = rng.integers(0, o, len(ri))
    _, Os = oracle.sampled(X, W, idx, ri, ci)
    got = out[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
    assert_out_close(got, Os, float(np.abs(Os.astype(np.float64)).max()))
    # the same rows through the staged calls (three-pass pre-pass)
    outl2 = L.find_outliers(Xd, 6.0, CAP, ws)
    rows2 = L.quantize_rows(Xd, outl2)
    torch.cuda.synchronize()
    assert outl2.idx[:n].cpu().numpy().tolist() == idx.tolist()
    assert torch.equal(rows2.cx, rows.cx) and torch.equal(rows2.Xq, rows.Xq)


def zp_buffers(L, s, h):
    import torch
    outl, _ = buffers(L, 1, 32)
    rows = L.ZpRows(torch.empty(L.xq_bytes(s, h), dtype=torch.int8, device="cuda"),
                    torch.empty((s, 4), dtype=torch.int32, device="cuda"),
                    torch.empty((s, L.opad(CAP)), dtype=torch.float16, device="cuda"), s, h)
    return outl, rows


def unpack(zc):
    """[n, 4] int32 records -> lo bits, hi bits, zp, sum."""
    zc = zc.cpu().numpy()
    w0 = zc[:, 0].astype(np.int64) & 0xffffffff
    return (w0 & 0xffff).astype(np.uint16), (w0 >> 16).astype(np.uint16), zc[:, 1], zc[:, 2]


def test_zeropoint_more_than_2_31_elements_in_x(big_x):
    import torch

    import paper_2208_07339_amd as L
    X, W, idx, Xd, Wd = big_x
    (s, h), o = X.shape, W.shape[1]
    ws = L.Workspace.allocate(s, h, o, CAP)
    qw = L.zp_quantize_weight(Wd, ws)
    outl, rows = zp_buffers(L, s, h)
    out = L.zp_linear(Xd, qw, 6.0, outl, rows, ws)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    rng = np.random.default_rng(8)
    rsel = sample_rows(rng, s, 2 ** 31 // h, 800)
    ref = oracle.zp_quantize_rows(np.ascontiguousarray(X[rsel]), idx)
    rsel_d = torch.from_numpy(rsel).cuda()
    lo, hi, zp, rs = unpack(rows.zc[rsel_d])
    assert np.array_equal(lo, bits(ref["lo"])) and np.array_equal(hi, bits(ref["hi"]))
    assert np.array_equal(zp, ref["zp"]) and np.array_equal(rs, ref["rowsum"])
    xq = L.export_rows(L.QuantizedRows(rows.Xq, None, None, s, h))[rsel_d].cpu().numpy()
    assert np.array_equal(xq, ref["Xq"])
    ri = np.repeat(rsel[::4], 4)
    ci = rng.integers(0, o, len(ri))
    _, Os = oracle.zp_sampled(X, W, idx, ri, ci)
    got = out[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
    assert_out_close(got, Os, float(np.abs(Os.astype(np.float64)).max()))


def test_more_than_2_31_elements_in_out():
    import torch

    import paper_2208_07339_amd as L
    s, h, o = 66000, 64, 32768
    assert s * o > 2 ** 31
    rng = np.random.default_rng(4)
    X = rng.standard_normal((s, h), dtype=np.float32).astype(np.float16)
    X[:, 5] *= np.float16(0.25)
    X[s - 3, 5] = 11.0   # an outlier column decided by a row in the far part
    X[:, 17] *= np.float16(8.0)
    W = (rng.standard_normal((h, o), dtype=np.float32) * 0.05).astype(np.float16)
    idx = oracle.find_outliers(X, 6.0)
    assert 5 in idx and 17 in idx and len(idx) <= CAP
    Xd, Wd = upload(X), upload(W)
    ws = L.Workspace.allocate(s, h, o, CAP)
    qw = L.quantize_weight(Wd, ws)
    outl, rows = buffers(L, s, h)
    out = L.linear(Xd, qw, 6.0, outl, rows, ws)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    ri = np.repeat(sample_rows(rng, s, 2 ** 31 // o, 600), 4)
    ci = np.r_[rng.integers(0, o, len(ri) - 8), [0, 1, o - 2, o - 1, 255, 256, 257, 16384]]
    _, Os = oracle.sampled(X, W, idx, ri, ci)
    got = out[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
    assert_out_close(got, Os, float(np.abs(Os.astype(np.float64)).max()))


@pytest.fixture(scope="module")
def big_w():
    """W with h * o > 2^31, on the host and on the device, and its quantized form (shared by both cases)."""
    import torch

    import paper_2208_07339_amd as L
    h, o = 65536, 33024
    assert h * o > 2 ** 31
    W = tiled_matrix(h, o, 2048, 0.02, 5)
    W[h - 1, o - 1] = 0.5    # the constant of the last column comes from the last row
    Wd = upload(W)
    qw = L.quantize_weight(Wd, L.Workspace.allocate(1, h, o, CAP))
    torch.cuda.synchronize()
    return W, qw, Wd


def test_more_than_2_31_elements_in_w_quantized(big_w):
    import torch

    import paper_2208_07339_amd as L
    W, qw, _ = big_w
    o = W.shape[1]
    rng = np.random.default_rng(6)
    csel = np.unique(np.r_[0:4, o - 40:o, rng.integers(0, o, 400)])
    Wq_ref, cw_ref = oracle.quantize_weight(np.ascontiguousarray(W[:, csel]))
    csel_d = torch.from_numpy(csel).cuda()
    assert np.array_equal(bits(qw.cw[csel_d].cpu().numpy()), bits(cw_ref))
    assert np.array_equal(L.export_weight(qw)[:, csel_d].cpu().numpy(), Wq_ref)


@pytest.mark.parametrize("s", [16, 40])  # weight-streaming path, tiled path
def test_more_than_2_31_elements_in_w(big_w, s):
    import torch

    import paper_2208_07339_amd as L
    W, qw, _ = big_w
    h, o = W.shape
    rng = np.random.default_rng(7 + s)
    X = rng.standard_normal((s, h), dtype=np.float32).astype(np.float16)
    for k in (5, 40000, h - 1):   # rows of the 16-bit weights up to the very last one
        X[k % s, k] = 30.0
    idx = oracle.find_outliers(X, 6.0)
    assert {5, 40000, h - 1} <= set(idx.tolist()) and len(idx) <= CAP
    Xd = upload(X)
    ws = L.Workspace.allocate(s, h, o, CAP)
    outl, rows = buffers(L, s, h)
    out = L.linear(Xd, qw, 6.0, outl, rows, ws)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    ri = rng.integers(0, s, 600)
    ci = np.r_[rng.integers(0, o, 560), np.arange(o - 40, o)]
    _, Os = oracle.sampled(X, W, idx, ri, ci)
    got = out[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
    assert_out_close(got, Os, float(np.abs(Os.astype(np.float64)).max()))


@pytest.mark.parametrize("s", [16, 40])
def test_zeropoint_more_than_2_31_elements_in_w(big_w, s):
    import torch

    import paper_2208_07339_amd as L
    W, _, Wd = big_w
    h, o = W.shape
    rng = np.random.default_rng(9 + s)
    X = np.abs(rng.standard_normal((s, h), dtype=np.float32)).astype(np.float16)   # one-sided rows
    for k in (5, 40000, h - 1):
        X[k % s, k] = 30.0
    idx = oracle.find_outliers(X, 6.0)
    assert {5, 40000, h - 1} <= set(idx.tolist()) and len(idx) <= CAP
    ws = L.Workspace.allocate(s, h, o, CAP)
    qw = L.zp_quantize_weight(Wd, ws)
    torch.cuda.synchronize()
    csel = np.unique(np.r_[0:4, o - 40:o, rng.integers(0, o, 200)])
    ref = oracle.zp_quantize_weight(np.ascontiguousarray(W[:, csel]))
    csel_d = torch.from_numpy(csel).cuda()
    lo, hi, zp, cs = unpack(qw.zc[csel_d])
    assert np.array_equal(lo, bits(ref["lo"])) and np.array_equal(hi, bits(ref["hi"]))
    assert np.array_equal(zp, ref["zp"]) and np.array_equal(cs, ref["colsum"])
    wq = L.export_weight(L.QuantizedWeight(qw.Wq, None, None, h, o))[:, csel_d].cpu().numpy()
    assert np.array_equal(wq, ref["Wq"])
    outl, rows = zp_buffers(L, s, h)
    out = L.zp_linear(upload(X), qw, 6.0, outl, rows, ws)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    ri = rng.integers(0, s, 400)
    ci = np.r_[rng.integers(0, o, 360), np.arange(o - 40, o)]
    _, Os = oracle.zp_sampled(X, W, idx, ri, ci)
    got = out[torch.from_numpy(ri).cuda(), torch.from_numpy(ci).cuda()].cpu().numpy()
    assert_out_close(got, Os, float(np.abs(Os.astype(np.float64)).max()))
