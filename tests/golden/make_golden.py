"""Writes tests/golden/tiny_oracle.txt: digests of every stage of the CPU oracle
on the Tiny configuration.  Calls only oracle/ and the input generator.  A
change of the oracle's arithmetic shows up as a diff of the stored file and
has to be justified from the paper in the commit that makes it.

    python tests/golden/make_golden.py
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

import oracle  # noqa: E402
from paper_2208_07339_amd import workloads as wl  # noqa: E402


def digest(a):
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def lines():
    d = wl.make("tiny")
    r = oracle.linear(d["X"], d["W"], d["alpha"])
    yield "# Tiny configuration (X 8x256 fp16, W 256x512 fp16, alpha 6.0, seed 0): oracle stage digests"
    yield "X_f16 sha256 " + digest(d["X"].view(np.uint16))
    yield "W_f16 sha256 " + digest(d["W"].view(np.uint16))
    yield "O " + " ".join(str(int(v)) for v in r["idx"])
    yield "c_x bits " + " ".join("%04x" % v for v in r["cx"].view(np.uint16))
    yield "c_w sha256 " + digest(r["cw"].view(np.uint16))
    yield "X_i8 sha256 " + digest(r["Xq"])
    yield "W_i8 sha256 " + digest(r["Wq"])
    yield "C_i32 sha256 " + digest(r["C"])
    yield "C_i32 row0 first8 " + " ".join(str(int(v)) for v in r["C"][0, :8])
    yield "Out_f16 sha256 " + digest(r["Out"].view(np.uint16))
    yield "Out_f16 row0 first8 bits " + " ".join("%04x" % v for v in r["Out"].view(np.uint16)[0, :8])


if __name__ == "__main__":
    with open(os.path.join(HERE, "tiny_oracle.txt"), "w") as f:
        f.write("\n".join(lines()) + "\n")
    print(open(os.path.join(HERE, "tiny_oracle.txt")).read())
