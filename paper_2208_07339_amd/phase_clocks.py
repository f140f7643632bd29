"""Shader-clock stamps at the phase boundaries of one tile of the prefill GEMM.

    python -m paper_2208_07339_amd.build --stamps        # builds libllmint8_stamps.so (measurement build)
    LLMINT8_LIB=paper_2208_07339_amd/libllmint8_stamps.so python -m paper_2208_07339_amd.phase_clocks [workload [tile]]

Runs 300 back-to-back calls of llmint8_linear on the workload (default ffn13b), then prints, for the waves
of one workgroup (eight at 256 x 256 and 128 x 256, else four), the clocks spent in each phase of that
workgroup's second tile (its only tile where the workload gives it one: attn6p7b; then nothing is requested
for a next tile), and the K loop's clocks per stage (its MFMAs alone need 32 clocks per v_mfma_i32_32x32x32_i8: 1024 per stage of a 256 x 256
tile, 768 at 192 x 256, 512 at 128 x 256).
"""
import ctypes as C
import sys

import numpy as np


PHASES = [(0, 1, "wait for the first stage"), (1, 2, "K loop"), (2, 3, "wait for the epilogue operands"),
          (3, 4, "request the next tile's first two stages"), (4, 5, "row constants, outlier columns of X"),
          (5, 20, "dequantize + outlier product + store")]


def main():
    import torch

    import paper_2208_07339_amd as L
    from paper_2208_07339_amd import workloads as wl
    if not hasattr(L.lib(), "llmint8_debug_read_stamps"):
        sys.exit("this library has no clock stamps: build with `python -m paper_2208_07339_amd.build --stamps` and "
                 "set LLMINT8_LIB to libllmint8_stamps.so")
    name = sys.argv[1] if len(sys.argv) > 1 else "ffn13b"
    if len(sys.argv) > 2:
        L.debug_prefill_tile(int(sys.argv[2]))  # optional: force a workgroup tile (llmint8_debug_prefill_tile)
    d = wl.make(name)
    s, h, o = d["s"], d["h"], d["o"]
    X = torch.from_numpy(d["X"].view(np.int16)).cuda().view(torch.float16)
    W = torch.from_numpy(d["W"].view(np.int16)).cuda().view(torch.float16)
    ws = L.Workspace.allocate(s, h, o, 32)
    qw = L.quantize_weight(W, ws)
    outl = L.find_outliers(X, d["alpha"], 32, ws)
    rows = L.quantize_rows(X, outl)
    out = torch.empty((s, o), dtype=torch.float16, device="cuda")
    for _ in range(300):
        L.linear(X, qw, d["alpha"], outl, rows, ws, out)
    torch.cuda.synchronize()
    buf = (C.c_longlong * 256)()
    fn = L.lib().llmint8_debug_read_stamps
    fn.argtypes = [C.c_void_p]
    assert fn(buf) == 0
    t = np.array(list(buf), dtype=np.int64).reshape(8, 32)
    nw = 8 if t[4:, 20].all() else 4  # rows 4-7 stay zero where the workgroup has four waves
    t = t[:nw]
    if not t[:, 20].all():
        sys.exit(f"{name}: workgroup 9 has no tile, nothing was stamped")
    stages = 2 * ((h + 127) // 128)
    print(f"{name}: s={s} h={h} o={o}, {stages} K stages per tile; clocks of one tile of workgroup 9, waves 0-{nw - 1}")
    for a, b, what in PHASES:
        print(f"  {what:62s} " + " ".join(f"{int(t[w, b] - t[w, a]):7d}" for w in range(nw)))
    total = t[:, 20] - t[:, 0]
    kloop = t[:, 2] - t[:, 1]
    print(f"  {'whole tile':62s} " + " ".join(f"{int(v):7d}" for v in total))
    print(f"  {'start of the tile relative to wave 0':62s} " + " ".join(f"{int(t[w, 0] - t[0, 0]):7d}" for w in range(nw)))
    if (t[:, 0] > t[:, 21]).all() and int((t[:, 0] - t[:, 21]).max()) < 60000:  # the stamped tile is the workgroup's first
        print(f"  {'kernel entry to the start of the tile':62s} " + " ".join(f"{int(t[w, 0] - t[w, 21]):7d}" for w in range(nw)))
    ticks = (t[:, 23] - t[:, 22]).astype(np.float64)  # 100 MHz counter over the same tile
    if (ticks > 0).all():
        print(f"  shader clock inside the tile: {float((total / ticks).mean()) * 0.1:.2f} GHz "
              f"({float(ticks.mean()) / 100:.1f} us per tile)")
    print(f"  K loop per stage: {kloop.mean() / stages:.0f} clocks; share of the tile outside the K loop: "
          f"{100 * (1 - kloop.mean() / total.mean()):.1f} %")


if __name__ == "__main__":
    main()
