"""ctypes binding of libllmint8.so.  Argument marshalling only."""
import ctypes as C
import os
from dataclasses import dataclass

HERE = os.path.dirname(os.path.abspath(__file__))
# LLMINT8_LIB names another build of the same library (the measurement build libllmint8_stamps.so)
LIB_PATH = os.environ.get("LLMINT8_LIB") or os.path.join(HERE, "libllmint8.so")

SYMBOLS = [
    "llmint8_status_string", "llmint8_last_hip_error", "llmint8_opad", "llmint8_wq_bytes", "llmint8_xq_bytes",
    "llmint8_workspace_bytes", "llmint8_quantize_weight", "llmint8_find_outliers",
    "llmint8_quantize_rows", "llmint8_matmul", "llmint8_linear", "llmint8_linear_events", "llmint8_dequantize_rows",
    "llmint8_init", "llmint8_linear_static", "llmint8_probe_mfma", "llmint8_probe_read",
    "llmint8_quantize_weight_granular", "llmint8_quantize_rows_granular", "llmint8_linear_granular",
    "llmint8_zp_quantize_weight", "llmint8_zp_quantize_rows", "llmint8_zp_matmul", "llmint8_zp_linear",
    "llmint8_export_weight",
    "llmint8_export_rows", "llmint8_debug_prefill_tile", "llmint8_debug_prefill_tile_for",
    "llmint8_debug_decode_shape",
]

_lib = None


class Llmint8Error(RuntimeError):
    pass


def lib():
    """Load the library (built by paper_2208_07339_amd.build); fail loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise Llmint8Error(f"{LIB_PATH} is missing: run `python -m paper_2208_07339_amd.build` "
                           "(hipcc, gfx950). There is no fallback path.")
    # torch first: it ships its own HIP runtime, and the library must bind to the one the tensors and
    # streams it is handed come from (a second runtime loaded earlier sees no device)
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, sz, f32 = C.c_void_p, C.c_int, C.c_size_t, C.c_float
    L.llmint8_status_string.restype = C.c_char_p
    L.llmint8_status_string.argtypes = [i32]
    L.llmint8_last_hip_error.restype = C.c_char_p
    L.llmint8_last_hip_error.argtypes = []
    L.llmint8_opad.restype = i32
    L.llmint8_opad.argtypes = [i32]
    L.llmint8_wq_bytes.restype = sz
    L.llmint8_wq_bytes.argtypes = [i32, i32]
    L.llmint8_xq_bytes.restype = sz
    L.llmint8_xq_bytes.argtypes = [i32, i32]
    L.llmint8_workspace_bytes.restype = sz
    L.llmint8_workspace_bytes.argtypes = [i32, i32, i32, i32]
    L.llmint8_quantize_weight.restype = i32
    L.llmint8_quantize_weight.argtypes = [vp, i32, i32, vp, vp, vp, sz, vp]
    L.llmint8_find_outliers.restype = i32
    L.llmint8_find_outliers.argtypes = [vp, i32, i32, f32, vp, i32, vp, vp, vp, sz, vp]
    L.llmint8_quantize_rows.restype = i32
    L.llmint8_quantize_rows.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    L.llmint8_matmul.restype = i32
    L.llmint8_matmul.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    L.llmint8_linear.restype = i32
    L.llmint8_linear.argtypes = [vp, i32, i32, f32, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.llmint8_init.restype = i32
    L.llmint8_init.argtypes = []
    L.llmint8_linear_static.restype = i32
    L.llmint8_linear_static.argtypes = [vp, i32, i32, f32, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    L.llmint8_probe_mfma.restype = i32
    L.llmint8_probe_mfma.argtypes = [vp, sz, vp, sz, i32, vp, C.POINTER(C.c_double), vp]
    L.llmint8_probe_read.restype = i32
    L.llmint8_probe_read.argtypes = [vp, sz, vp, vp]
    L.llmint8_dequantize_rows.restype = i32
    L.llmint8_dequantize_rows.argtypes = [vp, vp, i32, i32, vp, vp, i32, vp, vp]
    L.llmint8_quantize_weight_granular.restype = i32
    L.llmint8_quantize_weight_granular.argtypes = [vp, i32, i32, i32, vp, vp, vp, sz, vp]
    L.llmint8_quantize_rows_granular.restype = i32
    L.llmint8_quantize_rows_granular.argtypes = [vp, i32, i32, vp, vp, i32, i32, vp, vp, vp, vp]
    L.llmint8_linear_granular.restype = i32
    L.llmint8_linear_granular.argtypes = [vp, i32, i32, f32, i32, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp,
                                          vp, sz, vp]
    L.llmint8_linear_events.restype = i32
    L.llmint8_linear_events.argtypes = L.llmint8_linear_granular.argtypes + [vp, vp]
    L.llmint8_zp_quantize_weight.restype = i32
    L.llmint8_zp_quantize_weight.argtypes = [vp, i32, i32, vp, vp, vp, sz, vp]
    L.llmint8_zp_quantize_rows.restype = i32
    L.llmint8_zp_quantize_rows.argtypes = [vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    L.llmint8_zp_matmul.restype = i32
    L.llmint8_zp_matmul.argtypes = [vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    L.llmint8_zp_linear.restype = i32
    L.llmint8_zp_linear.argtypes = [vp, i32, i32, f32, vp, vp, vp, i32, vp, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.llmint8_export_weight.restype = i32
    L.llmint8_export_weight.argtypes = [vp, i32, i32, vp, vp]
    L.llmint8_export_rows.restype = i32
    L.llmint8_export_rows.argtypes = [vp, i32, i32, vp, vp]
    L.llmint8_debug_prefill_tile.restype = i32
    L.llmint8_debug_prefill_tile.argtypes = [i32]
    L.llmint8_debug_prefill_tile_for.restype = i32
    L.llmint8_debug_prefill_tile_for.argtypes = [i32, i32, i32]
    L.llmint8_debug_decode_shape.restype = i32
    L.llmint8_debug_decode_shape.argtypes = [i32]
    _lib = L
    return L


def _check(code):
    if code != 0:
        detail = f" ({lib().llmint8_last_hip_error().decode()})" if code == 4 else ""
        raise Llmint8Error(f"llmint8 status {code}: {lib().llmint8_status_string(code).decode()}{detail}")


def _torch():
    import torch
    return torch


def _stream():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def opad(cap):
    return lib().llmint8_opad(cap)


def wq_bytes(h, o):
    return lib().llmint8_wq_bytes(h, o)


def xq_bytes(s, h):
    return lib().llmint8_xq_bytes(s, h)


def workspace_bytes(s, h, o, cap):
    return lib().llmint8_workspace_bytes(s, h, o, cap)


@dataclass
class Workspace:
    buf: object  # torch.uint8 device tensor

    @staticmethod
    def allocate(s, h, o, cap, device="cuda"):
        torch = _torch()
        return Workspace(torch.empty(workspace_bytes(s, h, o, cap), dtype=torch.uint8, device=device))

    @property
    def nbytes(self):
        return self.buf.numel()


@dataclass
class QuantizedWeight:
    Wq: object     # uint8/int8 device tensor, private tiled layout
    cw: object     # [o] fp16
    W: object      # [h, o] fp16 original (rows O are read by matmul), or None: rows rebuilt from the codes
    h: int
    o: int


@dataclass
class Outliers:
    idx: object    # [cap] int32
    count: object  # [1] int32
    status: object  # [1] int32
    cap: int


@dataclass
class QuantizedRows:
    Xq: object     # int8 device tensor, private tiled layout
    cx: object     # [s] fp16
    Xo: object     # [s, opad] fp16
    s: int
    h: int


GRANULARITY = {"vectorwise": 0, "rowwise": 1, "tensorwise": 2}  # LLMINT8_VECTORWISE / _ROWWISE / _TENSORWISE


def quantize_weight(W, ws=None, granularity="vectorwise"):
    """llmint8_quantize_weight(_granular): W [h, o] fp16 (device, contiguous) -> QuantizedWeight."""
    torch = _torch()
    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and W.dim() == 2
    h, o = W.shape
    Wq = torch.empty(wq_bytes(h, o), dtype=torch.int8, device=W.device)
    cw = torch.empty(o, dtype=torch.float16, device=W.device)
    if ws is None:
        ws = Workspace.allocate(1, h, o, 1, W.device)
    if granularity == "vectorwise":
        _check(lib().llmint8_quantize_weight(_ptr(W), h, o, _ptr(Wq), _ptr(cw), _ptr(ws.buf), ws.nbytes, _stream()))
    else:
        _check(lib().llmint8_quantize_weight_granular(_ptr(W), h, o, GRANULARITY[granularity], _ptr(Wq), _ptr(cw),
                                                      _ptr(ws.buf), ws.nbytes, _stream()))
    return QuantizedWeight(Wq, cw, W, h, o)


def find_outliers(X, alpha, cap, ws, out=None):
    """llmint8_find_outliers: X [s, h] fp16 -> Outliers (all on device)."""
    torch = _torch()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2
    s, h = X.shape
    if out is None:
        out = Outliers(torch.empty(cap, dtype=torch.int32, device=X.device),
                       torch.empty(1, dtype=torch.int32, device=X.device),
                       torch.empty(1, dtype=torch.int32, device=X.device), cap)
    _check(lib().llmint8_find_outliers(_ptr(X), s, h, float(alpha), _ptr(out.idx), cap, _ptr(out.count),
                                       _ptr(out.status), _ptr(ws.buf), ws.nbytes, _stream()))
    return out


def quantize_rows(X, outl, out=None, granularity="vectorwise"):
    """llmint8_quantize_rows(_granular): X [s, h] fp16 + Outliers -> QuantizedRows."""
    torch = _torch()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2
    s, h = X.shape
    if out is None:
        out = QuantizedRows(torch.empty(xq_bytes(s, h), dtype=torch.int8, device=X.device),
                            torch.empty(s, dtype=torch.float16, device=X.device),
                            torch.empty((s, opad(outl.cap)), dtype=torch.float16, device=X.device), s, h)
    if granularity == "vectorwise":
        _check(lib().llmint8_quantize_rows(_ptr(X), s, h, _ptr(outl.idx), _ptr(outl.count), outl.cap, _ptr(out.Xq),
                                           _ptr(out.cx), _ptr(out.Xo), _stream()))
    else:
        _check(lib().llmint8_quantize_rows_granular(_ptr(X), s, h, _ptr(outl.idx), _ptr(outl.count), outl.cap,
                                                    GRANULARITY[granularity], _ptr(out.Xq), _ptr(out.cx),
                                                    _ptr(out.Xo), _stream()))
    return out


def matmul(rows, outl, qw, ws, out=None, want_c_i32=False):
    """llmint8_matmul -> Out [s, o] fp16 (and the raw int32 accumulators if asked)."""
    torch = _torch()
    s, h, o = rows.s, rows.h, qw.o
    assert h == qw.h
    if out is None:
        out = torch.empty((s, o), dtype=torch.float16, device=rows.Xq.device)
    Cd = torch.empty((s, o), dtype=torch.int32, device=rows.Xq.device) if want_c_i32 else None
    _check(lib().llmint8_matmul(_ptr(rows.Xq), _ptr(rows.cx), _ptr(rows.Xo), _ptr(outl.idx), _ptr(outl.count),
                                outl.cap, _ptr(qw.Wq), _ptr(qw.cw), _ptr(qw.W), s, h, o, _ptr(out), _ptr(Cd),
                                _ptr(ws.buf), ws.nbytes, _stream()))
    return (out, Cd) if want_c_i32 else out


def linear(X, qw, alpha, outl, rows, ws, out=None, events=None, granularity="vectorwise"):
    """llmint8_linear(_granular): the three per-call steps in one C call, into preallocated buffers.
    granularity must be the one qw was quantized with (it selects the constants of X here).
    events = (before_matmul, after_matmul): two torch.cuda.Event(enable_timing=True) that have been
    recorded once already (so that their handles exist); llmint8_linear_events records them again."""
    torch = _torch()
    s, h = X.shape
    if out is None:
        out = torch.empty((s, qw.o), dtype=torch.float16, device=X.device)
    head = (_ptr(X), s, h, float(alpha))
    tail = (_ptr(qw.Wq), _ptr(qw.cw), _ptr(qw.W), qw.o, _ptr(outl.idx), outl.cap,
            _ptr(outl.count), _ptr(outl.status), _ptr(rows.Xq), _ptr(rows.cx), _ptr(rows.Xo), _ptr(out),
            _ptr(ws.buf), ws.nbytes, _stream())
    g = GRANULARITY[granularity]
    if events is not None:
        _check(lib().llmint8_linear_events(*head, g, *tail, C.c_void_p(events[0].cuda_event),
                                           C.c_void_p(events[1].cuda_event)))
    elif g == 0:
        _check(lib().llmint8_linear(*head, *tail))
    else:
        _check(lib().llmint8_linear_granular(*head, g, *tail))
    return out


STATIC_SCRATCH_BYTES = 16 << 20  # LLMINT8_STATIC_SCRATCH_BYTES


def init():
    """llmint8_init: per-device set-up of the current device (optional; the first call does the same)."""
    _check(lib().llmint8_init())


def linear_static(X, qw, alpha, outl, rows, out):
    """llmint8_linear_static: llmint8_linear on the library's static scratch; every buffer is the caller's,
    nothing is allocated (out is required)."""
    s, h = X.shape
    _check(lib().llmint8_linear_static(_ptr(X), s, h, float(alpha), _ptr(qw.Wq), _ptr(qw.cw), _ptr(qw.W), qw.o,
                                       _ptr(outl.idx), outl.cap, _ptr(outl.count), _ptr(outl.status), _ptr(rows.Xq),
                                       _ptr(rows.cx), _ptr(rows.Xo), _ptr(out), _stream()))
    return out


def probe_mfma(A_tiles, B_tiles, iters, sink):
    """llmint8_probe_mfma on two tiled int8 device buffers; returns the int8 operations of the launch."""
    ops = C.c_double(0.0)
    _check(lib().llmint8_probe_mfma(_ptr(A_tiles), A_tiles.numel(), _ptr(B_tiles), B_tiles.numel(), int(iters),
                                    _ptr(sink), C.byref(ops), _stream()))
    return ops.value


def probe_read(buf, sink):
    """llmint8_probe_read over a device buffer (bytes)."""
    _check(lib().llmint8_probe_read(_ptr(buf), buf.numel() * buf.element_size(), _ptr(sink), _stream()))


def debug_prefill_tile(cfg):
    """llmint8_debug_prefill_tile: force the prefill GEMM's workgroup tile (-1 = automatic)."""
    _check(lib().llmint8_debug_prefill_tile(int(cfg)))


def debug_prefill_tile_for(s, h, o):
    """llmint8_debug_prefill_tile_for: the tile the library chooses for [s x h] by [h x o] (no GPU needed)."""
    return int(lib().llmint8_debug_prefill_tile_for(int(s), int(h), int(o)))


def debug_decode_shape(cfg):
    """llmint8_debug_decode_shape: force the decode kernel's work split (-1 = default)."""
    _check(lib().llmint8_debug_decode_shape(int(cfg)))


def dequantize_rows(qw, outl):
    """llmint8_dequantize_rows: rows O of W rebuilt from the codes -> [opad, o] fp16."""
    torch = _torch()
    out = torch.empty((opad(outl.cap), qw.o), dtype=torch.float16, device=qw.Wq.device)
    _check(lib().llmint8_dequantize_rows(_ptr(qw.Wq), _ptr(qw.cw), qw.h, qw.o, _ptr(outl.idx), _ptr(outl.count),
                                         outl.cap, _ptr(out), _stream()))
    return out


# ---- zeropoint variant (Eq. 1-5) -------------------------------------------------

@dataclass
class ZpWeight:
    Wq: object     # int8 device tensor, private tiled layout
    zc: object     # [o, 4] int32 records: lo | hi << 16 (fp16 bits), zp, column sum of the codes, 0
    W: object      # [h, o] fp16 original (rows O are read by zp_matmul)
    h: int
    o: int


@dataclass
class ZpRows:
    Xq: object     # int8 device tensor, private tiled layout
    zc: object     # [s, 4] int32 records: lo | hi << 16, zp, row sum of the codes, 0
    Xo: object     # [s, opad] fp16
    s: int
    h: int


def zp_quantize_weight(W, ws=None):
    """llmint8_zp_quantize_weight: W [h, o] fp16 (device, contiguous) -> ZpWeight."""
    torch = _torch()
    assert W.is_cuda and W.dtype == torch.float16 and W.is_contiguous() and W.dim() == 2
    h, o = W.shape
    Wq = torch.empty(wq_bytes(h, o), dtype=torch.int8, device=W.device)
    zc = torch.empty((o, 4), dtype=torch.int32, device=W.device)
    if ws is None:
        ws = Workspace.allocate(1, h, o, 1, W.device)
    _check(lib().llmint8_zp_quantize_weight(_ptr(W), h, o, _ptr(Wq), _ptr(zc), _ptr(ws.buf), ws.nbytes, _stream()))
    return ZpWeight(Wq, zc, W, h, o)


def zp_quantize_rows(X, outl, out=None):
    """llmint8_zp_quantize_rows: X [s, h] fp16 + Outliers -> ZpRows."""
    torch = _torch()
    assert X.is_cuda and X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2
    s, h = X.shape
    if out is None:
        out = ZpRows(torch.empty(xq_bytes(s, h), dtype=torch.int8, device=X.device),
                     torch.empty((s, 4), dtype=torch.int32, device=X.device),
                     torch.empty((s, opad(outl.cap)), dtype=torch.float16, device=X.device), s, h)
    _check(lib().llmint8_zp_quantize_rows(_ptr(X), s, h, _ptr(outl.idx), _ptr(outl.count), outl.cap, _ptr(out.Xq),
                                          _ptr(out.zc), _ptr(out.Xo), _stream()))
    return out


def zp_matmul(rows, outl, qw, ws, out=None, want_c_i32=False):
    """llmint8_zp_matmul -> Out [s, o] fp16 (and the plain int8 product if asked)."""
    torch = _torch()
    s, h, o = rows.s, rows.h, qw.o
    assert h == qw.h
    if out is None:
        out = torch.empty((s, o), dtype=torch.float16, device=rows.Xq.device)
    Cd = torch.empty((s, o), dtype=torch.int32, device=rows.Xq.device) if want_c_i32 else None
    _check(lib().llmint8_zp_matmul(_ptr(rows.Xq), _ptr(rows.zc), _ptr(rows.Xo), _ptr(outl.idx), _ptr(outl.count),
                                   outl.cap, _ptr(qw.Wq), _ptr(qw.zc), _ptr(qw.W), s, h, o, _ptr(out), _ptr(Cd),
                                   _ptr(ws.buf), ws.nbytes, _stream()))
    return (out, Cd) if want_c_i32 else out


def zp_linear(X, qw, alpha, outl, rows, ws, out=None):
    """llmint8_zp_linear: outlier scan, zeropoint quantization of X and the matmul in one C call."""
    torch = _torch()
    s, h = X.shape
    if out is None:
        out = torch.empty((s, qw.o), dtype=torch.float16, device=X.device)
    _check(lib().llmint8_zp_linear(_ptr(X), s, h, float(alpha), _ptr(qw.Wq), _ptr(qw.zc), _ptr(qw.W), qw.o,
                                   _ptr(outl.idx), outl.cap, _ptr(outl.count), _ptr(outl.status), _ptr(rows.Xq),
                                   _ptr(rows.zc), _ptr(rows.Xo), _ptr(out), _ptr(ws.buf), ws.nbytes, _stream()))
    return out


def export_weight(qw):
    """Private tiled W_i8 -> [h, o] int8 row-major (test support)."""
    torch = _torch()
    out = torch.empty((qw.h, qw.o), dtype=torch.int8, device=qw.Wq.device)
    _check(lib().llmint8_export_weight(_ptr(qw.Wq), qw.h, qw.o, _ptr(out), _stream()))
    return out


def export_rows(rows):
    """Private tiled X_i8 -> [s, h] int8 row-major (test support)."""
    torch = _torch()
    out = torch.empty((rows.s, rows.h), dtype=torch.int8, device=rows.Xq.device)
    _check(lib().llmint8_export_rows(_ptr(rows.Xq), rows.s, rows.h, _ptr(out), _stream()))
    return out
