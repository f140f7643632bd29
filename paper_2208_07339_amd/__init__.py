"""LLM.int8() mixed-precision decomposition matmul for one MI355X (gfx950).

Thin Python binding of the C-ABI library libllmint8.so (include/llmint8.h): the
functions below marshal torch tensors (device memory, current stream) into
the C calls and do nothing else.  There is no CPU or PyTorch fallback: if the
HIP library is missing, loading fails.
"""
from .binding import (  # noqa: F401
    LIB_PATH, Llmint8Error, QuantizedWeight, Outliers, QuantizedRows, Workspace,
    lib, find_outliers, quantize_rows, quantize_weight, matmul, linear, export_rows, export_weight,
    workspace_bytes, wq_bytes, xq_bytes, opad, debug_prefill_tile, debug_prefill_tile_for, debug_decode_shape, dequantize_rows,
    init, linear_static, STATIC_SCRATCH_BYTES, probe_mfma, probe_read,
    GRANULARITY, ZpWeight, ZpRows, zp_quantize_weight, zp_quantize_rows, zp_matmul, zp_linear,
)
