"""HIP path vs CPU oracle at the full benchmark sizes.  The oracle cannot
multiply these matrices in full within a test, so: the outlier set, every row
constant, every column constant and both int8 tensors are compared in full;
the int32 accumulators and fp16 outputs are compared on whole rows at tile
edges and on random samples the oracle computes one by one from the
definition.  Two runs per size: the staged calls with the accumulator export
(which runs the prefill GEMM's instantiation with the guarded epilogue), and
llmint8_linear exactly as bench.py calls it (automatic tile shape, no export:
the instantiation whose epilogue is fed from LDS), whose outputs and intermediate
buffers are held to the same comparisons."""
import numpy as np
import pytest

import oracle
from paper_2208_07339_amd import workloads as wl
from gpu_util import assert_out_close, bits, hip_weight_i8, oracle_rows, run_hip

pytestmark = pytest.mark.gpu


def check_config(name, edge_rows, nsample=1500):
    d = wl.make(name)
    X, W = d["X"], d["W"]
    s, h, o = d["s"], d["h"], d["o"]
    g = run_hip(X, W, d["alpha"], cap=32)
    idx = oracle.find_outliers(X, d["alpha"])
    assert g["status"] == 0 and g["idx"].tolist() == idx.tolist()
    assert set(d["planted"].tolist()) <= set(idx.tolist())
    Wq, cw = oracle.quantize_weight(W)
    assert np.array_equal(bits(g["cw"]), bits(cw))
    assert np.array_equal(hip_weight_i8(g["qw"]), Wq)
    Xq, cx = oracle.quantize_rows(X, idx)
    assert np.array_equal(bits(g["cx"]), bits(cx))
    assert np.array_equal(g["Xq"], Xq)
    assert np.all(cx.astype(np.float64) < d["alpha"])
    # whole rows at tile and block edges
    rows = sorted(set(r for r in edge_rows if r < s))
    ref = oracle_rows(X, W, idx, rows, Wq, cw)
    assert np.array_equal(g["C"][rows], ref["C"])
    scale = float(np.abs(ref["Out"].astype(np.float64)).max())
    assert_out_close(g["Out"][rows], ref["Out"], scale)
    # random single outputs from the definition
    rng = np.random.default_rng(123)
    ri = rng.integers(0, s, nsample)
    ci = rng.integers(0, o, nsample)
    Cs, Os = oracle.sampled(X, W, idx, ri, ci)
    assert np.array_equal(g["C"][ri, ci], Cs)
    assert_out_close(g["Out"][ri, ci], Os, scale)
    # property that holds at any size: outputs are finite and not all zero
    assert np.isfinite(g["Out"].astype(np.float32)).all() and g["Out"].any()

    # ---- the one-call path in the configuration bench.py times, into fresh buffers
    import torch

    import paper_2208_07339_amd as L
    cap = 32
    outl = L.Outliers(torch.full((cap,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda"),
                      torch.full((1,), -7, dtype=torch.int32, device="cuda"), cap)
    qrows = L.QuantizedRows(torch.full((L.xq_bytes(s, h),), 99, dtype=torch.int8, device="cuda"),
                            torch.full((s,), 7.0, dtype=torch.float16, device="cuda"),
                            torch.full((s, L.opad(cap)), 7.0, dtype=torch.float16, device="cuda"), s, h)
    out = torch.full((s, o), 7.0, dtype=torch.float16, device="cuda")
    for _ in range(2):
        L.linear(g["Xd"], g["qw"], d["alpha"], outl, qrows, g["ws"], out=out)
    torch.cuda.synchronize()
    n = int(outl.count.item())
    assert int(outl.status.item()) == 0 and outl.idx[:n].cpu().numpy().tolist() == idx.tolist()
    assert np.array_equal(bits(qrows.cx.cpu().numpy()), bits(cx))
    assert np.array_equal(L.export_rows(qrows).cpu().numpy(), Xq)
    Xo = qrows.Xo.cpu().numpy()
    assert np.array_equal(bits(Xo[:, :n]), bits(X[:, idx])) and not bits(Xo[:, n:]).any()
    lin = out.cpu().numpy()
    assert_out_close(lin[rows], ref["Out"], scale)
    assert_out_close(lin[ri, ci], Os, scale)
    # every output of the one-call path against the staged path's (the same arithmetic in another
    # epilogue: they may differ in the order of the fp32 sums of the outlier product only)
    assert_out_close(lin, g["Out"], scale)
    assert np.isfinite(lin.astype(np.float32)).all()


def test_decode_175b_ffn_up():
    check_config("decode", edge_rows=[0, 7, 15])


def test_prefill_6p7b_attention_projection():
    check_config("attn6p7b", edge_rows=[0, 31, 32, 127, 128, 255, 256, 2047])


def test_prefill_13b_ffn_up():
    check_config("ffn13b", edge_rows=[0, 255, 256, 1023, 4095])


def test_prefill_175b_ffn_down():
    check_config("ffn175b_down", edge_rows=[0, 255, 256, 2047], nsample=600)
