"""Helpers of the GPU parity tests: run the HIP path through the C-ABI binding
and fetch every stage to the host; compose oracle stages for row subsets."""
import numpy as np

import oracle


def have_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def run_hip(X, W, alpha, cap, want_c=True, qw=None):
    """All stages of the HIP path on cuda:0.  Returns dict of numpy arrays (+ device handles)."""
    import torch

    import paper_2208_07339_amd as L
    dev = torch.device("cuda:0")
    s, h = X.shape
    o = W.shape[1]
    Xd = torch.from_numpy(X.view(np.int16)).to(dev).view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, cap, dev)
    if qw is None:
        Wd = torch.from_numpy(W.view(np.int16)).to(dev).view(torch.float16)
        qw = L.quantize_weight(Wd, ws)
    outl = L.find_outliers(Xd, alpha, cap, ws)
    rows = L.quantize_rows(Xd, outl)
    res = L.matmul(rows, outl, qw, ws, want_c_i32=want_c)
    Out, Cd = res if want_c else (res, None)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    return dict(
        idx=outl.idx[:n].cpu().numpy(), count=n, status=int(outl.status.item()),
        cx=rows.cx.cpu().numpy(), cw=qw.cw.cpu().numpy(),
        Xq=L.export_rows(rows).cpu().numpy(), Xo=rows.Xo.cpu().numpy(),
        Out=Out.cpu().numpy(), C=None if Cd is None else Cd.cpu().numpy(),
        qw=qw, outl=outl, rows=rows, ws=ws, Xd=Xd,
    )


def hip_weight_i8(qw):
    import paper_2208_07339_amd as L
    return L.export_weight(qw).cpu().numpy()


def oracle_rows(X, W, idx, rows, Wq=None, cw=None):
    """Oracle stages for a subset of rows, with the outlier set of the full X."""
    if Wq is None:
        Wq, cw = oracle.quantize_weight(W)
    Xs = np.ascontiguousarray(X[rows])
    Xq, cx = oracle.quantize_rows(Xs, idx)
    Cm = oracle.igemm(Xq, Wq)
    Out = oracle.output(Cm, cx, cw, Xs, W, idx)
    return dict(Xq=Xq, cx=cx, C=Cm, Out=Out)


def bits(a):
    return np.ascontiguousarray(a).view(np.uint16)


def assert_out_close(got, want, scale=None):
    """spec tolerance: max |diff| <= 1e-3 * max |Out| (of the oracle's full output, or `scale`)."""
    g = got.astype(np.float64)
    w = want.astype(np.float64)
    m = np.abs(w).max() if scale is None else scale
    err = np.abs(g - w).max() if g.size else 0.0
    assert err <= 1e-3 * m, f"max |diff| {err:.3e} > 1e-3 * {m:.3e}"
    return err / m if m > 0 else 0.0
