"""No-GPU checks of the boundary: the library loads, exports every symbol the
header declares, and the host-side size functions / argument checks behave."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2208_07339_amd as L
    if not os.path.exists(L.LIB_PATH):
        from paper_2208_07339_amd.build import build
        build()
    return L.lib()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "llmint8.h")).read()
    names = set(re.findall(r"\b(llmint8_[a-z0-9_]+)\s*\(", hdr))
    assert {"llmint8_quantize_weight", "llmint8_find_outliers", "llmint8_quantize_rows", "llmint8_matmul"} <= names
    for n in names:
        assert hasattr(lib, n), n
    from paper_2208_07339_amd.binding import SYMBOLS
    assert set(SYMBOLS) == names


def test_size_functions(lib):
    import paper_2208_07339_amd as L
    assert L.opad(1) == 16 and L.opad(16) == 16 and L.opad(17) == 32 and L.opad(0) == 0
    # tiles of 1 KiB: 32 rows x 32 features, features padded to 128
    assert L.xq_bytes(8, 256) == 1 * 8 * 1024
    assert L.xq_bytes(33, 200) == 2 * 8 * 1024
    assert L.wq_bytes(12288, 49152) == 12288 * 49152
    assert L.wq_bytes(0, 5) == 0
    # scratch holds the slab-wise column maxima of the two absmax scans (2 bytes per column per slab)
    assert L.workspace_bytes(16, 12288, 49152, 32) >= max(12288, 49152) * 2
    assert L.workspace_bytes(0, 1, 1, 1) == 0


def test_argument_checks_need_no_gpu(lib):
    assert lib.llmint8_matmul(*([None] * 5), 4, *([None] * 3), 1, 1, 1, None, None, None, 0, None) == 1
    assert lib.llmint8_quantize_weight(None, 4, 4, None, None, None, 0, None) == 1
    assert lib.llmint8_status_string(0) == b"ok"
    assert b"workspace" in lib.llmint8_status_string(3)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2208_07339_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in txt and "from oracle" not in txt and "liboracle" not in txt, f


def test_missing_library_fails_loudly(monkeypatch):
    """No fallback: without the built HIP library the binding raises instead of computing anything."""
    from paper_2208_07339_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libllmint8.so"))
    with pytest.raises(binding.Llmint8Error, match="no fallback"):
        binding.lib()


def test_argument_checks_of_the_variants_need_no_gpu(lib):
    assert lib.llmint8_zp_quantize_weight(None, 4, 4, None, None, None, 0, None) == 1
    assert lib.llmint8_zp_linear(*([None] * 1), 4, 4, C.c_float(6.0), None, None, None, 4, None, 4, None, None,
                                 None, None, None, None, None, 0, None) == 1
    assert lib.llmint8_quantize_weight_granular(None, 4, 4, 0, None, None, None, 0, None) == 1
    assert lib.llmint8_dequantize_rows(None, None, 4, 4, None, None, 4, None, None) == 1
    assert lib.llmint8_debug_prefill_tile(99) == 1 and lib.llmint8_debug_prefill_tile(-1) == 0
    assert lib.llmint8_debug_decode_shape(99) == 1 and lib.llmint8_debug_decode_shape(-1) == 0
    assert lib.llmint8_debug_decode_shape(0) == 0 and lib.llmint8_debug_decode_shape(-1) == 0
    assert lib.llmint8_debug_decode_shape(-2) == 1 and lib.llmint8_debug_decode_shape(6) == 1
    # the entry point on the static scratch: sizes are checked before anything touches a device
    f = C.c_float(6.0)
    assert lib.llmint8_linear_static(None, 0, 4, f, None, None, None, 4, None, 4, *([None] * 7)) == 1
    assert lib.llmint8_linear_static(None, 4, 133145, f, None, None, None, 4, None, 4, *([None] * 7)) == 2
    assert lib.llmint8_linear_static(None, 64, 64, f, None, None, None, 1 << 20, None, 32, *([None] * 7)) == 5
    assert b"static" in lib.llmint8_status_string(5)


def test_tile_choice_of_the_prefill_gemm(lib):
    """Host logic: the workgroup tile chosen from the shape (llmint8_debug_prefill_tile_for needs no GPU).
    0 = 256 x 256, 1 = 192 x 256, 2 = 128 x 256, 3 = 128 x 128, 4 = 192 x 128, 5 = 192 x 64 (columns x tokens)."""
    f = lib.llmint8_debug_prefill_tile_for
    f.restype, f.argtypes = C.c_int, [C.c_int] * 3
    # the three prefill workloads of the benchmark keep the shapes their figures were measured with
    assert f(4096, 5120, 20480) == 0      # 13B FFN: 1 280 tiles = 5 full passes of 256 x 256
    assert f(2048, 49152, 12288) == 1     # 175B FFN down: 512 tiles of 192 x 256 = 2 full passes (256 x 256: 1.5)
    assert f(2048, 4096, 4096) == 2       # 6.7B attention: one 128 x 256 tile per compute unit
    # short X against a wide W: one 192-column tile per compute unit, token tile as small as covers X
    assert f(64, 12288, 49152) == 5 and f(33, 12288, 49152) == 5
    assert f(128, 12288, 49152) == 4 and f(96, 12288, 49152) == 4
    assert f(256, 12288, 49152) == 1
    # every answer is a valid tile, whatever the shape; nonsense is refused
    for s, h, o in [(33, 1, 1), (33, 133144, 7), (100000, 64, 8), (4096, 4096, 1 << 20), (257, 129, 65)]:
        assert 0 <= f(s, h, o) < 6
    assert f(0, 4, 4) == -1 and f(4, 4, -1) == -1


def test_benchmark_shapes_fit_the_static_scratch(lib):
    import paper_2208_07339_amd as L
    from paper_2208_07339_amd import workloads as wl
    for c in wl.CONFIGS.values():
        assert L.workspace_bytes(c["s"], c["h"], c["o"], 32) <= L.STATIC_SCRATCH_BYTES


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "single-GPU" in r.stderr


def test_header_is_plain_c(tmp_path):
    """include/llmint8.h is a C header: a C99 translation unit that includes it and links against the
    library builds with no warning, and its size functions agree with the Python binding's."""
    import subprocess

    import paper_2208_07339_amd as L
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include <stdio.h>\n#include "llmint8.h"\n'
        "int main(void) {\n"
        '    printf("%d %zu %zu %zu %s\\n", llmint8_opad(20), llmint8_wq_bytes(300, 70), llmint8_xq_bytes(33, 300),\n'
        "           llmint8_workspace_bytes(33, 300, 70, 20), llmint8_status_string(LLMINT8_WORKSPACE));\n"
        "    return llmint8_quantize_rows(0, 1, 1, 0, 0, 1, 0, 0, 0, 0) == LLMINT8_INVALID_ARG ? 0 : 1;\n"
        "}\n")
    exe = tmp_path / "use_header"
    lib_dir = os.path.dirname(L.LIB_PATH)
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
           "-o", str(exe), "-L", lib_dir, "-lllmint8", "-Wl,-rpath," + lib_dir]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(None, 4)
    assert int(out[0]) == L.opad(20) and int(out[1]) == L.wq_bytes(300, 70) and int(out[2]) == L.xq_bytes(33, 300)
    assert int(out[3]) == L.workspace_bytes(33, 300, 70, 20) and out[4].strip()
