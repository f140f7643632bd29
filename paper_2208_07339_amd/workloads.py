"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws random numbers and plants structure; it holds none of
the method's arithmetic and is the one piece shared by the GPU tests, the
bench and the CPU oracle's tests.

Recipe (statistics from the paper's outlier analysis, Section 4 and the
outlier table of Appendix C): hidden states are N(0,1) rounded to fp16; a
handful of feature columns carry large one-signed values of magnitude
U(lo, hi) in 75% of the rows; weights are N(0, 0.02) rounded to fp16.  Layer
shapes follow the GPT-3 family sizes of the matmul benchmark table in
Appendix D.1 (hidden = 4 x model dimension).
"""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ALPHA = 6.0

# name -> s, h, o, planted columns (count or explicit list), magnitude range,
#         fraction of rows carrying the outlier, seed base
CONFIGS = {
    "tiny":        dict(s=8,    h=256,   o=512,   cols=[17, 200], lo=8.0,  hi=20.0, frac=1.0,  seed=0),
    "decode":      dict(s=16,   h=12288, o=49152, cols=7,         lo=10.0, hi=60.0, frac=0.75, seed=1000),
    "attn6p7b":    dict(s=2048, h=4096,  o=4096,  cols=6,         lo=10.0, hi=60.0, frac=0.75, seed=2000),
    "ffn13b":      dict(s=4096, h=5120,  o=20480, cols=8,         lo=10.0, hi=60.0, frac=0.75, seed=3000),
    "ffn175b_down": dict(s=2048, h=49152, o=12288, cols=20,       lo=10.0, hi=60.0, frac=0.75, seed=4000),
}

_BLOCK = 1 << 22  # elements per independently seeded block


def _workers():
    return max(1, min(8, os.cpu_count() or 1))


def normal_f16(rows, cols, std, seed):
    """[rows x cols] fp16 samples of N(0, std), reproducible for a given seed
    whatever the number of worker threads: row blocks have their own stream."""
    out = np.empty((rows, cols), dtype=np.float16)
    rows_per_block = max(1, _BLOCK // max(cols, 1))
    starts = list(range(0, rows, rows_per_block))

    def fill(b):
        r0 = starts[b]
        r1 = min(rows, r0 + rows_per_block)
        rng = np.random.default_rng([seed, b])
        blk = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        if std != 1.0:
            blk *= np.float32(std)
        out[r0:r1] = blk  # float32 -> float16, round to nearest even

    if len(starts) <= 1:
        for b in range(len(starts)):
            fill(b)
    else:
        with ThreadPoolExecutor(_workers()) as ex:
            list(ex.map(fill, range(len(starts))))
    return out


def make_x(s, h, cols, lo, hi, frac, seed):
    """Hidden states with planted outlier feature columns.
    Returns (X fp16 [s x h], planted column indices ascending)."""
    X = normal_f16(s, h, 1.0, seed)
    rng = np.random.default_rng([seed, 2])
    if isinstance(cols, int):
        planted = np.sort(rng.choice(h, size=cols, replace=False)).astype(np.int32)
    else:
        planted = np.asarray(sorted(cols), dtype=np.int32)
    n_rows = int(round(frac * s))
    for j in planted:
        sign = 1.0 if rng.random() < 0.5 else -1.0
        rows = rng.permutation(s)[:n_rows]
        mag = rng.uniform(lo, hi, size=n_rows).astype(np.float32)
        X[rows, j] = (sign * mag).astype(np.float16)
    return X, planted


def make_w(h, o, seed, std=0.02):
    return normal_f16(h, o, std, seed + 1)


def make(name, with_w=True):
    """Inputs of one named configuration: dict with X, W, alpha, planted, s, h, o."""
    c = CONFIGS[name]
    X, planted = make_x(c["s"], c["h"], c["cols"], c["lo"], c["hi"], c["frac"], c["seed"])
    W = make_w(c["h"], c["o"], c["seed"]) if with_w else None
    return dict(name=name, X=X, W=W, alpha=ALPHA, planted=planted, s=c["s"], h=c["h"], o=c["o"])


def make_custom(s, h, o, n_cols, seed, lo=10.0, hi=60.0, frac=0.75, std_w=0.02):
    """Same recipe at an arbitrary shape (ragged-shape parity cases)."""
    X, planted = make_x(s, h, min(n_cols, h), lo, hi, frac, seed)
    W = make_w(h, o, seed, std_w)
    return dict(name=f"custom_{s}x{h}x{o}", X=X, W=W, alpha=ALPHA, planted=planted, s=s, h=h, o=o)
