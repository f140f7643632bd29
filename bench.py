#!/usr/bin/env python3
"""Throughput of the LLM.int8() matmul hot path on one MI355X.

A step is one pass of the whole per-call path -- outlier scan, row quantize +
outlier gather, int8 GEMM with fused dequantization and fp16 outlier product
-- over one batch of synthetic hidden states already resident in HBM; the
weights were converted to int8 once, before the timed region (as the method
prescribes).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Workloads (paper_2208_07339_amd/workloads.py): ffn13b (default headline,
effective int8 TOPS), decode (HBM GB/s, reported in the same line under
"decode"), attn6p7b, ffn175b_down.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5033.0   # 256 CU x 8192 int8 op/clk/CU x 2.4 GHz, dense
HBM_PEAK_GBS = 8000.0
CAP = 32                       # capacity of the outlier index list
COPY_PROBE_BYTES = 256 << 20   # size of the calibration copies of --copy-probe

# HBM bytes per launch of the dominant kernel.  NOT read in this run (counters need their own rocprofv3
# --pmc passes): copied from the committed summary named in TRAFFIC_SOURCE, which gives the commands;
# None for workloads without such a summary.
TRAFFIC_SOURCE = "profiles/bench_default_ffn13b_decode_hbm_traffic.txt"
MEASURED_TRAFFIC = {
    # FETCH_SIZE / 0.5001 + WRITE_SIZE / 1.0 (KiB -> bytes; factors from the copy probe of the same runs)
    "ffn13b": 633.80e6 + 167.81e6,   # gemm_prefill_kernel<4,2,4,false,false>: operand panels re-fetched per XCD and round + Out
    "decode": 607.39e6 + 1.57e6,     # gemm_decode_kernel<1,1,8>
}


def traffic_fields(workload):
    t = MEASURED_TRAFFIC.get(workload)
    return {"traffic": t, "traffic_source": (TRAFFIC_SOURCE + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an "
                                             "earlier run of this command, not read in this run)") if t else None}


WARM_MS = 60.0  # least duration of the untimed warm-up (see run_workload)


def algorithmic_bytes_decode(s, h, o, n_out):
    """W_i8 + c_w + Out + outlier rows of W_f16 + X_i8 tile + Xo, per launch of the decode kernel."""
    return h * o + 2 * o + 2 * s * o + n_out * o * 2 + 32 * h + s * 32 * 2


def to_dev(a):
    import torch
    return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)


def run_workload(name, steps, warmup, copies=1, int8_rows=False, granularity="vectorwise", alpha=None, ceilings=True,
                 hold=None):
    import torch

    import paper_2208_07339_amd as L
    from paper_2208_07339_amd import workloads as wl

    d = wl.make(name)
    if alpha is not None:
        d["alpha"] = alpha
    s, h, o = d["s"], d["h"], d["o"]
    Xd = to_dev(d["X"])
    Wd = to_dev(d["W"])
    ws = L.Workspace.allocate(s, h, o, CAP)
    t0 = time.perf_counter()
    qws = [L.quantize_weight(Wd, ws, granularity=granularity)]
    torch.cuda.synchronize()
    t_wq = time.perf_counter() - t0
    if int8_rows:  # variant that keeps no fp16 weights: the outlier rows are rebuilt from the codes
        qws[0].W = None
    for _ in range(copies - 1):  # rotate weight copies so that no last-level cache flatters a streaming read
        q = qws[0]
        qws.append(L.QuantizedWeight(q.Wq.clone(), q.cw.clone(), q.W, q.h, q.o))
    outl = L.find_outliers(Xd, d["alpha"], CAP, ws)
    rows = L.quantize_rows(Xd, outl, granularity=granularity)
    out = torch.empty((s, o), dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    n_out = int(outl.count.item())

    def step(i):
        L.linear(Xd, qws[i % len(qws)], d["alpha"], outl, rows, ws, out, granularity=granularity)

    # Warm-up: W steps, and more of them until WARM_MS of back-to-back work have passed.  From idle the chip
    # needs some 30 ms of load to settle at its sustained clocks (measured: the first 10 ms run 15 % slow),
    # which is more than W steps of a 0.1 ms call.
    t0 = time.perf_counter()
    n_warm = 0
    while n_warm < warmup or (time.perf_counter() - t0) * 1e3 < WARM_MS:
        step(n_warm)
        n_warm += 1
        if n_warm % 16 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        step(i)
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps

    # The same steps again, now with HIP events recorded by the library on its launch stream around
    # the dominant kernel (llmint8_matmul is one launch): same back-to-back sequence, same thermal
    # state as the timed region above.
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    for e3 in evs:
        for e in e3:
            e.record()  # creates the handles
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        evs[i][0].record()
        L.linear(Xd, qws[i % len(qws)], d["alpha"], outl, rows, ws, out, events=(evs[i][1], evs[i][2]),
                 granularity=granularity)
    torch.cuda.synchronize()
    ms_step_events = (time.perf_counter() - t0) * 1e3 / steps
    ms_pre = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    mm = np.array([e[1].elapsed_time(e[2]) for e in evs])
    # whole steps from the events: start of step i to start of step i + 1 (the last one to its own end)
    st = np.array([evs[i][0].elapsed_time(evs[i + 1][0]) for i in range(steps - 1)] + [evs[-1][0].elapsed_time(evs[-1][2])])
    ceil = measured_ceiling(L, torch, name, qws, rows) if ceilings else None
    if hold:  # keep this load on the GPU for an outside power / clock sampler
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        zeros = torch.zeros(1 << 20, dtype=torch.int8, device="cuda")
        t_end, n = time.perf_counter() + hold[1], 0
        while time.perf_counter() < t_end:
            for _ in range(64):
                if hold[0] == "steps":
                    step(n)
                elif hold[0] == "probe":
                    L.probe_mfma(qws[0].Wq, rows.Xq, 400, sink)
                else:
                    L.probe_mfma(zeros, zeros, 400, sink)
                n += 1
            torch.cuda.synchronize()
    return dict(name=name, s=s, h=h, o=o, n_out=n_out, planted=len(d["planted"]), ms_step=ms_step,
                ms_prepass=ms_pre, ms_matmul=float(mm.mean()), ms_matmul_median=float(np.median(mm)),
                ms_matmul_min=float(mm.min()), ms_step_median=float(np.median(st)), ms_step_min=float(st.min()),
                ms_step_events=ms_step_events, warmup_steps_run=n_warm,
                weight_quantize_ms=t_wq * 1e3, ceiling=ceil,
                inputs=d)


def _timed_launches(torch, fn, n_warm, n_timed):
    """n_warm untimed launches of fn(i), then n_timed back to back between two events: ms per launch."""
    for i in range(n_warm):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(n_timed):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n_timed


def measured_ceiling(L, torch, name, qws, rows):
    """What this machine sustains, measured right after the timed steps (same warm state).
    Prefill: the register-only int8 MFMA issue loop (llmint8_probe_mfma) on this workload's own tiled codes,
    and on zeros.  Decode: a read-only stream (llmint8_probe_read) over the int8 weights, rotating the same
    two copies as the timed steps."""
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    if name == "decode":
        nbytes = qws[0].Wq.numel()
        ms = _timed_launches(torch, lambda i: L.probe_read(qws[i % len(qws)].Wq, sink), 200, 200)
        return {"kind": "read-only stream over the int8 weights (llmint8_probe_read)", "unit": "GB/s",
                "value": nbytes / (ms * 1e-3) / 1e9, "ms_per_launch": ms}
    iters = 400
    ops = []
    zeros = torch.zeros(1 << 20, dtype=torch.int8, device="cuda")
    out = {}
    for key, (A, B) in (("workload_operands", (qws[0].Wq, rows.Xq)), ("zero_operands", (zeros, zeros))):
        ms = _timed_launches(torch, lambda i: ops.append(L.probe_mfma(A, B, iters, sink)), 150, 100)
        out[key] = ops[-1] / (ms * 1e-3) / 1e12
        out[key + "_ms_per_launch"] = ms
    return {"kind": "register-only v_mfma_i32_32x32x32_i8 issue loop, 4 waves per CU, 64 MFMAs per iteration "
                    "(llmint8_probe_mfma): on this workload's tiled codes / on zeros", "unit": "TOP/s",
            "value": out["workload_operands"], "zero_operands": out["zero_operands"],
            "ms_per_launch": out["workload_operands_ms_per_launch"]}


def run_zeropoint(name, steps, warmup, alpha):
    """The zeropoint variant (Eq. 1-5) on the same inputs: whole call, and its matmul part alone."""
    import torch

    import paper_2208_07339_amd as L
    from paper_2208_07339_amd import workloads as wl

    d = wl.make(name)
    s, h, o = d["s"], d["h"], d["o"]
    Xd, Wd = to_dev(d["X"]), to_dev(d["W"])
    ws = L.Workspace.allocate(s, h, o, CAP)
    t0 = time.perf_counter()
    qw = L.zp_quantize_weight(Wd, ws)
    torch.cuda.synchronize()
    t_wq = time.perf_counter() - t0
    outl = L.find_outliers(Xd, alpha, CAP, ws)
    rows = L.zp_quantize_rows(Xd, outl)
    out = torch.empty((s, o), dtype=torch.float16, device="cuda")
    torch.cuda.synchronize()
    times = []
    for fn in (lambda: L.zp_linear(Xd, qw, alpha, outl, rows, ws, out), lambda: L.zp_matmul(rows, outl, qw, ws, out)):
        t0, n_warm = time.perf_counter(), 0
        while n_warm < warmup or (time.perf_counter() - t0) * 1e3 < WARM_MS:  # as in run_workload
            fn()
            n_warm += 1
            if n_warm % 16 == 0:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        times.append((time.perf_counter() - t0) * 1e3 / steps)
    return dict(name=name, s=s, h=h, o=o, n_out=int(outl.count.item()), planted=len(d["planted"]), ms_step=times[0],
                ms_matmul_calls=times[1], weight_quantize_ms=t_wq * 1e3)


def roofline_block(res):
    """The dominant kernel against its nominal peak and against what this box sustained in this run."""
    s, h, o = res["s"], res["h"], res["o"]
    if res["name"] == "decode":
        work, scale, peak = algorithmic_bytes_decode(s, h, o, res["n_out"]), 1e9, HBM_PEAK_GBS
        blk = {"bound": "hbm", "kernel": "gemm_decode_kernel", "unit": "GB/s"}
    else:
        work, scale, peak = 2.0 * s * h * o, 1e12, INT8_MFMA_PEAK_TOPS
        blk = {"bound": "mfma", "kernel": "gemm_prefill_kernel", "unit": "TOP/s"}
    ach = work / (res["ms_matmul"] * 1e-3) / scale
    blk.update({"achieved": ach, "peak": peak, "frac": ach / peak,
                "achieved_median": work / (res["ms_matmul_median"] * 1e-3) / scale,
                "achieved_best": work / (res["ms_matmul_min"] * 1e-3) / scale})
    c = res.get("ceiling")
    if c:
        blk.update({"measured_peak": c["value"], "frac_of_measured": ach / c["value"], "measured_peak_kind": c["kind"]})
        if "zero_operands" in c:
            blk["measured_peak_zero_operands"] = c["zero_operands"]
    blk.update(traffic_fields(res["name"]))
    return blk


def cpu_baseline(res, target_seconds=12.0, weights=None):
    """The CPU oracle, as it stands, on a bounded sample: the per-call steps (outlier scan, row
    quantization, integer product, dequantization + outlier product) on the first r rows of X
    against the full weight matrix, which is quantized beforehand and not timed."""
    import oracle
    d = res["inputs"]
    X, W = d["X"], d["W"]
    s, h, o = res["s"], res["h"], res["o"]
    Wq, cw = weights if weights is not None else oracle.quantize_weight(W)
    # calibrate the sample size on a couple of rows
    r = min(s, 2)
    t0 = time.perf_counter()
    _cpu_rows(oracle, X[:r], W, Wq, cw, d["alpha"])
    per_row = (time.perf_counter() - t0) / r
    cores = oracle.num_threads()
    # two rows under-use the cores: calibrate again on one row per core
    r = min(s, cores)
    t0 = time.perf_counter()
    _cpu_rows(oracle, X[:r], W, Wq, cw, d["alpha"])
    per_row = min(per_row, (time.perf_counter() - t0) / r)
    r = int(max(1, min(s, target_seconds / max(per_row, 1e-9))))
    r = max(min(s, cores), r - r % cores) if r >= cores else r
    t0 = time.perf_counter()
    _cpu_rows(oracle, X[:r], W, Wq, cw, d["alpha"])
    t = time.perf_counter() - t0
    return r, t, cores


def _cpu_rows(oracle, Xs, W, Wq, cw, alpha):
    Xs = np.ascontiguousarray(Xs)
    idx = oracle.find_outliers(Xs, alpha)
    Xq, cx = oracle.quantize_rows(Xs, idx)
    Cm = oracle.igemm(Xq, Wq)
    return oracle.output(Cm, cx, cw, Xs, W, idx)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="ffn13b", choices=["ffn13b", "decode", "attn6p7b", "ffn175b_down"])
    ap.add_argument("--no-decode", action="store_true", help="skip the secondary decode measurement")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the measured-ceiling leg (MFMA issue loop / read-only stream after the timed steps)")
    ap.add_argument("--outlier-rows", default="fp16", choices=["fp16", "int8"],
                    help="fp16: outlier product with the original weight rows (Eq. 8 as printed); int8: rows "
                         "rebuilt from the int8 codes, no fp16 weights kept (measured separately, not the headline)")
    ap.add_argument("--granularity", default="vectorwise", choices=["vectorwise", "rowwise", "tensorwise"],
                    help="absmax constants: vectorwise is the method (Section 3.1); rowwise / tensorwise are the "
                         "baselines of Table 1 (measured separately, not the headline)")
    ap.add_argument("--alpha", type=float, default=6.0,
                    help="outlier threshold; inf switches the decomposition off (the baselines without it)")
    ap.add_argument("--quantizer", default="absmax", choices=["absmax", "zeropoint"],
                    help="zeropoint: the asymmetric quantization of Eq. 1-5 per row of X / column of W (Table 1's "
                         "zeropoint rows; measured separately, not the headline)")
    ap.add_argument("--hold", default=None, choices=["steps", "probe", "probe-zeros"],
                    help="after the measurement keep the GPU busy for --hold-seconds with back-to-back steps of the "
                         "workload, or launches of the MFMA issue loop on its codes / on zeros, so that an outside "
                         "sampler (amd-smi metric --power --clock) can read socket power and clocks under that load")
    ap.add_argument("--hold-seconds", type=float, default=8.0)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run three device-to-device copies of 256 MiB first: under rocprofv3 --pmc their "
                         "FETCH_SIZE / WRITE_SIZE readings calibrate the counters (paper_2208_07339_amd/pmc_summary.py)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1. "
                 "value is one MI355X's throughput.")
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback.")

    if a.copy_probe:
        src = torch.ones(COPY_PROBE_BYTES, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if a.quantizer == "zeropoint":
        r = run_zeropoint(a.workload, a.steps, a.warmup, a.alpha)
        ops = 2.0 * r["s"] * r["h"] * r["o"]
        nbytes = algorithmic_bytes_decode(r["s"], r["h"], r["o"], r["n_out"])
        dec = a.workload == "decode"
        print(json.dumps({
            "metric": "zeropoint variant of the matmul per call (outlier scan + zeropoint row quantize + int8 GEMM "
                      "with the Eq. 5 corrections in the epilogue), 1 MI355X",
            "value": nbytes / (r["ms_step"] * 1e-3) / 1e9 if dec else ops / (r["ms_step"] * 1e-3) / 1e12,
            "unit": "GB/s" if dec else "TOPS", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
            "ms_per_step": r["ms_step"], "ms_matmul_calls": r["ms_matmul_calls"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
            "config": {"workload": a.workload, "s": r["s"], "h": r["h"], "o": r["o"],
                       "alpha": a.alpha if np.isfinite(a.alpha) else "inf", "quantizer": "zeropoint",
                       "outlier_columns_found": r["n_out"]},
            "weight_quantize_ms_once": r["weight_quantize_ms"]}))
        return
    i8 = a.outlier_rows == "int8"
    res = run_workload(a.workload, a.steps, a.warmup, copies=2 if a.workload == "decode" else 1, int8_rows=i8,
                       granularity=a.granularity, alpha=a.alpha, ceilings=not a.no_ceilings,
                       hold=(a.hold, a.hold_seconds) if a.hold else None)
    s, h, o = res["s"], res["h"], res["o"]
    ops = 2.0 * s * h * o
    line = {
        "metric": "effective int8 TOPS of the LLM.int8() matmul per call (outlier scan + row quantize + "
                  "int8 GEMM with fused dequant/outlier epilogue), 1 MI355X",
        "value": ops / (res["ms_step"] * 1e-3) / 1e12,
        "unit": "TOPS",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": res["ms_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": a.workload, "s": s, "h": h, "o": o, "alpha": a.alpha if np.isfinite(a.alpha) else "inf", "granularity": a.granularity,
                   "outlier_columns_planted": res["planted"], "outlier_columns_found": res["n_out"],
                   "outlier_capacity": CAP, "outlier_rows": a.outlier_rows},
        "ms_per_step_median": res["ms_step_median"], "ms_per_step_min": res["ms_step_min"],
        "ms_prepass": res["ms_prepass"], "ms_matmul_kernel": res["ms_matmul"],
        "ms_matmul_kernel_median": res["ms_matmul_median"], "ms_matmul_kernel_min": res["ms_matmul_min"],
        "ms_per_step_with_events": res["ms_step_events"], "warmup_steps_run": res["warmup_steps_run"],
        "weight_quantize_ms_once": res["weight_quantize_ms"],
    }
    if a.workload == "decode":
        line["metric"] = ("achieved HBM GB/s of the LLM.int8() matmul per call at decode size "
                          "(algorithmic bytes / step time), 1 MI355X")
        line["value"] = algorithmic_bytes_decode(s, h, o, res["n_out"]) / (res["ms_step"] * 1e-3) / 1e9
        line["unit"] = "GB/s"
    line["roofline"] = roofline_block(res)

    if not a.no_cpu_baseline and a.granularity == "vectorwise":  # the oracle leg times the method itself
        import oracle
        wts = oracle.quantize_weight(res["inputs"]["W"])
        r, t, cores = cpu_baseline(res, weights=wts)
        # the same oracle on one thread, on a smaller sample of the same rows
        oracle.set_num_threads(1)
        r1, t1, _ = cpu_baseline(res, target_seconds=5.0, weights=wts)
        oracle.set_num_threads(cores)
        if a.workload == "decode":
            # the oracle reads fp16 weights; quote it in the metric's unit on the same algorithmic bytes
            v = algorithmic_bytes_decode(r, h, o, res["n_out"]) / t / 1e9
            v1 = algorithmic_bytes_decode(r1, h, o, res["n_out"]) / t1 / 1e9
            unit = "GB/s"
        else:
            v = 2.0 * r * h * o / t / 1e12
            v1 = 2.0 * r1 * h * o / t1 / 1e12
            unit = "TOPS"
        line["cpu_baseline"] = {"value": v, "unit": unit, "cores": cores, "kind": "oracle",
                                "sample": f"per-call steps on the first {r} of {s} rows of X against the full "
                                          f"{h}x{o} weights (quantized beforehand, untimed); {t:.1f} s",
                                "single_thread": {"value": v1, "unit": unit, "cores": 1,
                                                  "sample": f"the first {r1} of {s} rows; {t1:.1f} s"}}
    del res["inputs"]

    if a.workload != "decode" and not a.no_decode:
        dres = run_workload("decode", a.steps, a.warmup, copies=2, int8_rows=i8, granularity=a.granularity,
                            alpha=a.alpha, ceilings=not a.no_ceilings)
        nbytes = algorithmic_bytes_decode(dres["s"], dres["h"], dres["o"], dres["n_out"])
        line["decode"] = {
            "workload": "decode", "s": dres["s"], "h": dres["h"], "o": dres["o"],
            "ms_per_step": dres["ms_step"], "ms_per_step_median": dres["ms_step_median"],
            "ms_per_step_min": dres["ms_step_min"], "ms_prepass": dres["ms_prepass"],
            "ms_matmul_kernel": dres["ms_matmul"], "ms_matmul_kernel_median": dres["ms_matmul_median"],
            "ms_matmul_kernel_min": dres["ms_matmul_min"],
            "value": nbytes / (dres["ms_step"] * 1e-3) / 1e9, "unit": "GB/s",
            "roofline": roofline_block(dres),
        }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
