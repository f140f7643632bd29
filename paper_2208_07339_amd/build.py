"""Compile the HIP sources under csrc/ for gfx950 into libllmint8.so (in-tree).

    python -m paper_2208_07339_amd.build
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllmint8.so")
LIB_STAMPS = os.path.join(HERE, "libllmint8_stamps.so")  # measurement build: see build(stamps=True)
SOURCES = ["api.hip", "prepass.hip", "gemm.hip", "decode.hip", "zeropoint.hip", "ceiling.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose=False, stamps=False):
    """Always recompiles; raises on failure.  Returns the library path.
    stamps=True builds libllmint8_stamps.so instead: the same sources with -DLLMINT8_GEMM_STAMPS, in which the
    prefill GEMM records the shader clock at its phase boundaries (paper_2208_07339_amd/phase_clocks.py reads
    them).  It is a measurement build and never the library the binding loads by default."""
    bdir = os.path.join(HERE, "_build_stamps" if stamps else "_build")
    os.makedirs(bdir, exist_ok=True)
    flags = FLAGS + (["-DLLMINT8_GEMM_STAMPS"] if stamps else [])
    lib = LIB_STAMPS if stamps else LIB

    def cc(src):
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        cmd = ["hipcc", *flags, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err)
        return obj

    with ThreadPoolExecutor(6) as ex:
        objs = list(ex.map(cc, SOURCES))
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib])
    return lib


if __name__ == "__main__":
    import sys
    print(build(verbose=True, stamps="--stamps" in sys.argv))
