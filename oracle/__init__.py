"""ctypes front end of the CPU oracle (oracle/llmint8_oracle.c).

Test infrastructure only: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The GPU library never imports this package and
this package never imports the GPU library.

Arrays are numpy: fp16 tensors are passed as np.float16 (or their uint16 bit
patterns), int8/int32 tensors as such, all C-contiguous.
"""
import ctypes as C

import numpy as np

from .build import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build())
        u16p, i8p, i32p = C.POINTER(C.c_uint16), C.POINTER(C.c_int8), C.POINTER(C.c_int32)
        L.oracle_f16_to_double.restype = C.c_double
        L.oracle_f16_to_double.argtypes = [C.c_uint16]
        L.oracle_double_to_f16.restype = C.c_uint16
        L.oracle_double_to_f16.argtypes = [C.c_double]
        L.oracle_q.restype = C.c_int
        L.oracle_q.argtypes = [C.c_double, C.c_double]
        L.oracle_find_outliers.restype = C.c_int
        L.oracle_find_outliers.argtypes = [u16p, C.c_int, C.c_int, C.c_double, i32p, C.c_int]
        L.oracle_quantize_weight.restype = None
        L.oracle_quantize_weight.argtypes = [u16p, C.c_int, C.c_int, i8p, u16p]
        L.oracle_quantize_rows.restype = None
        L.oracle_quantize_rows.argtypes = [u16p, C.c_int, C.c_int, i32p, C.c_int, i8p, u16p]
        L.oracle_igemm.restype = C.c_int
        L.oracle_igemm.argtypes = [i8p, i8p, C.c_int, C.c_int, C.c_int, i32p]
        L.oracle_output.restype = None
        L.oracle_output.argtypes = [i32p, u16p, u16p, u16p, u16p, i32p, C.c_int, C.c_int, C.c_int,
                                    C.c_int, u16p]
        L.oracle_dequant_weight.restype = C.c_uint16
        L.oracle_dequant_weight.argtypes = [C.c_int8, C.c_uint16]
        L.oracle_dequant_rows.restype = None
        L.oracle_dequant_rows.argtypes = [i8p, u16p, C.c_int, C.c_int, i32p, C.c_int, u16p]
        L.oracle_output_dq.restype = None
        L.oracle_output_dq.argtypes = [i32p, u16p, u16p, u16p, i8p, i32p, C.c_int, C.c_int, C.c_int,
                                       C.c_int, u16p]
        L.oracle_linear.restype = C.c_int
        L.oracle_linear.argtypes = [u16p, u16p, C.c_int, C.c_int, C.c_int, C.c_double, i32p, i8p,
                                    u16p, i8p, u16p, i32p, u16p]
        L.oracle_sampled.restype = None
        L.oracle_sampled.argtypes = [u16p, u16p, C.c_int, C.c_int, C.c_int, i32p, C.c_int, i32p,
                                     i32p, C.c_int, i32p, u16p]
        L.oracle_quantize_weight_tensor.restype = None
        L.oracle_quantize_weight_tensor.argtypes = [u16p, C.c_int, C.c_int, i8p, u16p]
        L.oracle_quantize_rows_tensor.restype = None
        L.oracle_quantize_rows_tensor.argtypes = [u16p, C.c_int, C.c_int, i32p, C.c_int, i8p, u16p]
        L.oracle_linear_granular.restype = C.c_int
        L.oracle_linear_granular.argtypes = [u16p, u16p, C.c_int, C.c_int, C.c_int, C.c_double, C.c_int,
                                             i32p, i8p, u16p, i8p, u16p, i32p, u16p]
        L.oracle_sampled_granular.restype = None
        L.oracle_sampled_granular.argtypes = [u16p, u16p, C.c_int, C.c_int, C.c_int, i32p, C.c_int,
                                              C.c_int, i32p, i32p, C.c_int, i32p, u16p]
        i64p = C.POINTER(C.c_int64)
        L.oracle_zp_u.restype = C.c_longlong
        L.oracle_zp_u.argtypes = [C.c_double, C.c_double]
        L.oracle_zp_quantize_weight.restype = None
        L.oracle_zp_quantize_weight.argtypes = [u16p, C.c_int, C.c_int, i8p, u16p, u16p, i32p, i32p]
        L.oracle_zp_quantize_rows.restype = None
        L.oracle_zp_quantize_rows.argtypes = [u16p, C.c_int, C.c_int, i32p, C.c_int, i8p, u16p, u16p, i32p, i32p]
        L.oracle_zp_gemm.restype = None
        L.oracle_zp_gemm.argtypes = [i8p, i32p, i8p, i32p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, i64p]
        L.oracle_zp_output.restype = None
        L.oracle_zp_output.argtypes = [i64p, u16p, u16p, u16p, u16p, u16p, u16p, i32p, C.c_int, C.c_int,
                                       C.c_int, C.c_int, u16p]
        L.oracle_zp_linear.restype = C.c_int
        L.oracle_zp_linear.argtypes = [u16p, u16p, C.c_int, C.c_int, C.c_int, C.c_double, i32p, i8p, u16p,
                                       u16p, i32p, i32p, i8p, u16p, u16p, i32p, i32p, i32p, i64p, u16p]
        L.oracle_zp_sampled.restype = None
        L.oracle_zp_sampled.argtypes = [u16p, u16p, C.c_int, C.c_int, C.c_int, i32p, C.c_int, i32p, i32p,
                                        C.c_int, i32p, u16p]
        L.oracle_num_threads.restype = C.c_int
        L.oracle_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _bits(a):
    """fp16 array (or uint16 bit patterns) -> C-contiguous uint16 view."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16
    return a


def f16_to_double(bits):
    return lib().oracle_f16_to_double(int(bits))


def double_to_f16(v):
    return lib().oracle_double_to_f16(float(v))


def q(x, c):
    return lib().oracle_q(float(x), float(c))


def find_outliers(X, alpha):
    """Section 3.2: ascending feature columns holding any |x| >= alpha."""
    Xb = _bits(X)
    s, h = Xb.shape
    idx = np.zeros(max(h, 1), dtype=np.int32)
    n = lib().oracle_find_outliers(_p(Xb, C.c_uint16), s, h, float(alpha), _p(idx, C.c_int32), h)
    return idx[:n].copy()


def quantize_weight(W):
    """Section 3.1: per-output-column absmax constants and int8 codes."""
    Wb = _bits(W)
    h, o = Wb.shape
    Wq = np.zeros((h, o), dtype=np.int8)
    cw = np.zeros(o, dtype=np.uint16)
    lib().oracle_quantize_weight(_p(Wb, C.c_uint16), h, o, _p(Wq, C.c_int8), _p(cw, C.c_uint16))
    return Wq, cw.view(np.float16)


def quantize_rows(X, idx):
    """Per-row absmax over non-outlier columns; zeros in outlier columns."""
    Xb = _bits(X)
    s, h = Xb.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Xq = np.zeros((s, h), dtype=np.int8)
    cx = np.zeros(s, dtype=np.uint16)
    lib().oracle_quantize_rows(_p(Xb, C.c_uint16), s, h, _p(idx, C.c_int32), len(idx),
                               _p(Xq, C.c_int8), _p(cx, C.c_uint16))
    return Xq, cx.view(np.float16)


def igemm(Xq, Wq):
    """Eq. 7 inner product: int8 x int8 accumulated in int32."""
    Xq = np.ascontiguousarray(Xq, dtype=np.int8)
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    s, h = Xq.shape
    h2, o = Wq.shape
    assert h == h2
    Cm = np.zeros((s, o), dtype=np.int32)
    ovf = lib().oracle_igemm(_p(Xq, C.c_int8), _p(Wq, C.c_int8), s, h, o, _p(Cm, C.c_int32))
    if ovf:
        raise OverflowError("int32 accumulator overflow")
    return Cm


def output(Cm, cx, cw, X, W, idx):
    """Eq. 8: dequantized int8 product plus the 16-bit outlier product."""
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    o = Wb.shape[1]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Cm = np.ascontiguousarray(Cm, dtype=np.int32)
    Out = np.zeros((s, o), dtype=np.uint16)
    lib().oracle_output(_p(Cm, C.c_int32), _p(_bits(cx), C.c_uint16), _p(_bits(cw), C.c_uint16),
                        _p(Xb, C.c_uint16), _p(Wb, C.c_uint16), _p(idx, C.c_int32), len(idx), s, h,
                        o, _p(Out, C.c_uint16))
    return Out.view(np.float16)


def dequant_weight(q, cw):
    """fp16( q * cw / 127 ), the inverse of the absmax quantization, as fp16 bits -> np.float16."""
    b = lib().oracle_dequant_weight(int(q), int(np.float16(cw).view(np.uint16)))
    return np.uint16(b).view(np.float16)


def dequant_rows(Wq, cw, idx):
    """Rows idx of W rebuilt from the codes: [len(idx) x o] fp16."""
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    h, o = Wq.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows = np.zeros((len(idx), o), dtype=np.uint16)
    lib().oracle_dequant_rows(_p(Wq, C.c_int8), _p(_bits(cw), C.c_uint16), h, o, _p(idx, C.c_int32), len(idx),
                              _p(rows, C.c_uint16))
    return rows.view(np.float16)


def output_dq(Cm, cx, cw, X, Wq, idx):
    """Eq. 8 with the outlier rows of W rebuilt from the int8 codes (no 16-bit weights kept)."""
    Xb = _bits(X)
    s, h = Xb.shape
    Wq = np.ascontiguousarray(Wq, dtype=np.int8)
    o = Wq.shape[1]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Cm = np.ascontiguousarray(Cm, dtype=np.int32)
    Out = np.zeros((s, o), dtype=np.uint16)
    lib().oracle_output_dq(_p(Cm, C.c_int32), _p(_bits(cx), C.c_uint16), _p(_bits(cw), C.c_uint16),
                           _p(Xb, C.c_uint16), _p(Wq, C.c_int8), _p(idx, C.c_int32), len(idx), s, h, o,
                           _p(Out, C.c_uint16))
    return Out.view(np.float16)


def linear(X, W, alpha):
    """All six steps.  Returns a dict of every intermediate and the output."""
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    h2, o = Wb.shape
    assert h == h2
    idx = np.zeros(max(h, 1), dtype=np.int32)
    Xq = np.zeros((s, h), dtype=np.int8)
    cx = np.zeros(s, dtype=np.uint16)
    Wq = np.zeros((h, o), dtype=np.int8)
    cw = np.zeros(o, dtype=np.uint16)
    Cm = np.zeros((s, o), dtype=np.int32)
    Out = np.zeros((s, o), dtype=np.uint16)
    n = lib().oracle_linear(_p(Xb, C.c_uint16), _p(Wb, C.c_uint16), s, h, o, float(alpha),
                            _p(idx, C.c_int32), _p(Xq, C.c_int8), _p(cx, C.c_uint16),
                            _p(Wq, C.c_int8), _p(cw, C.c_uint16), _p(Cm, C.c_int32),
                            _p(Out, C.c_uint16))
    if n == -1:
        raise OverflowError("int32 accumulator overflow")
    if n == -2:
        raise ValueError("inputs must be finite")
    return {"idx": idx[:n].copy(), "Xq": Xq, "cx": cx.view(np.float16), "Wq": Wq,
            "cw": cw.view(np.float16), "C": Cm, "Out": Out.view(np.float16)}


def sampled(X, W, idx, rows, cols):
    """C[i,j] and Out[i,j] for listed (i,j) pairs, each from the definition."""
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    o = Wb.shape[1]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    n = len(rows)
    Cs = np.zeros(n, dtype=np.int32)
    Os = np.zeros(n, dtype=np.uint16)
    lib().oracle_sampled(_p(Xb, C.c_uint16), _p(Wb, C.c_uint16), s, h, o, _p(idx, C.c_int32),
                         len(idx), _p(rows, C.c_int32), _p(cols, C.c_int32), n, _p(Cs, C.c_int32),
                         _p(Os, C.c_uint16))
    return Cs, Os.view(np.float16)


GRANULARITY = {"vectorwise": 0, "rowwise": 1, "tensorwise": 2}


def quantize_weight_tensor(W):
    """Section 2.1: one absmax constant for the whole weight matrix (returned in every entry of cw)."""
    Wb = _bits(W)
    h, o = Wb.shape
    Wq = np.zeros((h, o), dtype=np.int8)
    cw = np.zeros(o, dtype=np.uint16)
    lib().oracle_quantize_weight_tensor(_p(Wb, C.c_uint16), h, o, _p(Wq, C.c_int8), _p(cw, C.c_uint16))
    return Wq, cw.view(np.float16)


def quantize_rows_tensor(X, idx):
    """One absmax constant over all non-outlier entries of X; zeros in outlier columns."""
    Xb = _bits(X)
    s, h = Xb.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Xq = np.zeros((s, h), dtype=np.int8)
    cx = np.zeros(s, dtype=np.uint16)
    lib().oracle_quantize_rows_tensor(_p(Xb, C.c_uint16), s, h, _p(idx, C.c_int32), len(idx),
                                      _p(Xq, C.c_int8), _p(cx, C.c_uint16))
    return Xq, cx.view(np.float16)


def linear_granular(X, W, alpha, granularity):
    """linear() with the constants of Table 1's baselines: "vectorwise", "rowwise" or "tensorwise"."""
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    h2, o = Wb.shape
    assert h == h2
    idx = np.zeros(max(h, 1), dtype=np.int32)
    Xq = np.zeros((s, h), dtype=np.int8)
    cx = np.zeros(s, dtype=np.uint16)
    Wq = np.zeros((h, o), dtype=np.int8)
    cw = np.zeros(o, dtype=np.uint16)
    Cm = np.zeros((s, o), dtype=np.int32)
    Out = np.zeros((s, o), dtype=np.uint16)
    n = lib().oracle_linear_granular(_p(Xb, C.c_uint16), _p(Wb, C.c_uint16), s, h, o, float(alpha),
                                     GRANULARITY[granularity], _p(idx, C.c_int32), _p(Xq, C.c_int8),
                                     _p(cx, C.c_uint16), _p(Wq, C.c_int8), _p(cw, C.c_uint16),
                                     _p(Cm, C.c_int32), _p(Out, C.c_uint16))
    if n == -1:
        raise OverflowError("int32 accumulator overflow")
    if n == -2:
        raise ValueError("inputs must be finite")
    assert n >= 0
    return {"idx": idx[:n].copy(), "Xq": Xq, "cx": cx.view(np.float16), "Wq": Wq,
            "cw": cw.view(np.float16), "C": Cm, "Out": Out.view(np.float16)}


def sampled_granular(X, W, idx, rows, cols, granularity):
    """sampled() for "rowwise" / "tensorwise" constants ("vectorwise" is sampled() itself)."""
    if GRANULARITY[granularity] == 0:
        return sampled(X, W, idx, rows, cols)
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    o = Wb.shape[1]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    n = len(rows)
    Cs = np.zeros(n, dtype=np.int32)
    Os = np.zeros(n, dtype=np.uint16)
    lib().oracle_sampled_granular(_p(Xb, C.c_uint16), _p(Wb, C.c_uint16), s, h, o, _p(idx, C.c_int32),
                                  len(idx), GRANULARITY[granularity], _p(rows, C.c_int32),
                                  _p(cols, C.c_int32), n, _p(Cs, C.c_int32), _p(Os, C.c_uint16))
    return Cs, Os.view(np.float16)


def zp_u(x, D):
    """Eq. 3 with the exact nd = 254 / D of Eq. 1: nearest integer to 254 x / D, ties to even."""
    return lib().oracle_zp_u(float(x), float(D))


def zp_quantize_weight(W):
    """Zeropoint quantization of every column of W: codes, lo, hi (fp16), zp, column sums of the codes."""
    Wb = _bits(W)
    h, o = Wb.shape
    Wq = np.zeros((h, o), dtype=np.int8)
    lo, hi = np.zeros(o, dtype=np.uint16), np.zeros(o, dtype=np.uint16)
    zp, cs = np.zeros(o, dtype=np.int32), np.zeros(o, dtype=np.int32)
    lib().oracle_zp_quantize_weight(_p(Wb, C.c_uint16), h, o, _p(Wq, C.c_int8), _p(lo, C.c_uint16),
                                    _p(hi, C.c_uint16), _p(zp, C.c_int32), _p(cs, C.c_int32))
    return dict(Wq=Wq, lo=lo.view(np.float16), hi=hi.view(np.float16), zp=zp, colsum=cs)


def zp_quantize_rows(X, idx):
    """Zeropoint quantization of every row of X over its non-outlier columns (code 0 in the others)."""
    Xb = _bits(X)
    s, h = Xb.shape
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    Xq = np.zeros((s, h), dtype=np.int8)
    lo, hi = np.zeros(s, dtype=np.uint16), np.zeros(s, dtype=np.uint16)
    zp, rs = np.zeros(s, dtype=np.int32), np.zeros(s, dtype=np.int32)
    lib().oracle_zp_quantize_rows(_p(Xb, C.c_uint16), s, h, _p(idx, C.c_int32), len(idx), _p(Xq, C.c_int8),
                                  _p(lo, C.c_uint16), _p(hi, C.c_uint16), _p(zp, C.c_int32), _p(rs, C.c_int32))
    return dict(Xq=Xq, lo=lo.view(np.float16), hi=hi.view(np.float16), zp=zp, rowsum=rs)


def zp_linear(X, W, alpha):
    """The whole call with zeropoint quantization (Eq. 1-5) in place of absmax.  Dict of every stage."""
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    h2, o = Wb.shape
    assert h == h2
    idx = np.zeros(max(h, 1), dtype=np.int32)
    Xq, Wq = np.zeros((s, h), dtype=np.int8), np.zeros((h, o), dtype=np.int8)
    loa, hia, za, rs = (np.zeros(s, np.uint16), np.zeros(s, np.uint16), np.zeros(s, np.int32),
                        np.zeros(s, np.int32))
    lob, hib, zb, cs = (np.zeros(o, np.uint16), np.zeros(o, np.uint16), np.zeros(o, np.int32),
                        np.zeros(o, np.int32))
    Cm = np.zeros((s, o), dtype=np.int32)
    T = np.zeros((s, o), dtype=np.int64)
    Out = np.zeros((s, o), dtype=np.uint16)
    n = lib().oracle_zp_linear(_p(Xb, C.c_uint16), _p(Wb, C.c_uint16), s, h, o, float(alpha), _p(idx, C.c_int32),
                               _p(Xq, C.c_int8), _p(loa, C.c_uint16), _p(hia, C.c_uint16), _p(za, C.c_int32),
                               _p(rs, C.c_int32), _p(Wq, C.c_int8), _p(lob, C.c_uint16), _p(hib, C.c_uint16),
                               _p(zb, C.c_int32), _p(cs, C.c_int32), _p(Cm, C.c_int32), _p(T, C.c_int64),
                               _p(Out, C.c_uint16))
    if n == -1:
        raise OverflowError("int32 accumulator overflow")
    if n == -2:
        raise ValueError("inputs must be finite")
    return {"idx": idx[:n].copy(), "Xq": Xq, "lo_x": loa.view(np.float16), "hi_x": hia.view(np.float16),
            "zp_x": za, "rowsum": rs, "Wq": Wq, "lo_w": lob.view(np.float16), "hi_w": hib.view(np.float16),
            "zp_w": zb, "colsum": cs, "C": Cm, "T": T, "Out": Out.view(np.float16)}


def zp_sampled(X, W, idx, rows, cols):
    """Plain int8 product C[i,j] and Out[i,j] of the zeropoint variant for listed pairs, from the definition."""
    Xb, Wb = _bits(X), _bits(W)
    s, h = Xb.shape
    o = Wb.shape[1]
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    cols = np.ascontiguousarray(cols, dtype=np.int32)
    n = len(rows)
    Cs = np.zeros(n, dtype=np.int32)
    Os = np.zeros(n, dtype=np.uint16)
    lib().oracle_zp_sampled(_p(Xb, C.c_uint16), _p(Wb, C.c_uint16), s, h, o, _p(idx, C.c_int32), len(idx),
                            _p(rows, C.c_int32), _p(cols, C.c_int32), n, _p(Cs, C.c_int32), _p(Os, C.c_uint16))
    return Cs, Os.view(np.float16)


def num_threads():
    return lib().oracle_num_threads()


def set_num_threads(n):
    lib().oracle_set_num_threads(int(n))
