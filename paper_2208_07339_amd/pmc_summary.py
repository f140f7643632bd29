"""Summarise rocprofv3 counter / kernel-trace CSVs of a bench.py run as short text.

    python -m paper_2208_07339_amd.pmc_summary counters <counter_collection.csv> [...]
    python -m paper_2208_07339_amd.pmc_summary trace <kernel_trace.csv>

`counters`: per kernel, the mean of each counter over its dispatches.  FETCH_SIZE / WRITE_SIZE are
reported by rocprofv3 in KiB per dispatch; the device-to-device copies that `bench.py --copy-probe`
runs first (256 MiB each: the first three dispatches of __amd_rocclr_copyBuffer) give the factor by
which the counter over- or under-reads, and every other kernel's reading is divided by it.
`trace`: per kernel, calls and mean / min / max duration, and the mean over the last `tail` dispatches
(optional third argument, default the last third): bench.py's own kernel figure comes from its last,
event-instrumented loop, after the warm-up and the timed loop, so that is the part to compare it with.
"""
import collections
import csv
import re
import sys

COPY_KIB = 256 * 1024  # bench.py COPY_PROBE_BYTES in KiB
COPY_KERNEL = "__amd_rocclr_copyBuffer"


def short(name):
    # rocprofv3 leaves names with _Float16 parameters mangled: spell the template arguments out
    m = re.match(r"_ZN7llmint8\d+(\w+?)I((?:L[ib]-?\d+E)+)E", name)
    if m:
        args = [("true" if v == "1" else "false") if k == "b" else v for k, v in re.findall(r"L([ib])(-?\d+)E", m.group(2))]
        return f"{m.group(1)}<{', '.join(args)}>"[:48]
    name = name.replace("llmint8::", "").replace("void ", "")
    return name.split("(")[0][:48]


def counters(paths):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    probes = collections.defaultdict(list)
    for p in paths:
        rows = sorted(csv.DictReader(open(p)), key=lambda r: int(r["Dispatch_Id"]))
        for r in rows:
            agg[r["Counter_Name"]][r["Kernel_Name"]].append(float(r["Counter_Value"]))
            if COPY_KERNEL in r["Kernel_Name"] and len(probes[r["Counter_Name"]]) < 3:
                probes[r["Counter_Name"]].append(float(r["Counter_Value"]))
    for cname, per_kernel in agg.items():
        factor = None
        probe = probes[cname]
        if cname in ("FETCH_SIZE", "WRITE_SIZE") and probe:
            factor = (sum(probe) / len(probe)) / COPY_KIB
            print(f"{cname}: 256 MiB copy reads {sum(probe) / len(probe):.0f} KiB over {len(probe)} dispatches "
                  f"-> factor {factor:.4f}")
        for k, vals in sorted(per_kernel.items(), key=lambda kv: -sum(kv[1])):
            mean = sum(vals) / len(vals)
            line = f"  {short(k):50s} n={len(vals):4d}  mean {mean:14.1f}"
            if factor:
                line += f"  -> {mean / factor * 1024 / 1e6:10.2f} MB per dispatch"
            print(line)


def trace(path, tail=None):
    agg = collections.defaultdict(list)
    for r in sorted(csv.DictReader(open(path)), key=lambda r: int(r["Start_Timestamp"])):
        agg[r["Kernel_Name"]].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in agg.values())
    print(f"{'kernel':50s} {'calls':>6s} {'mean us':>10s} {'min us':>10s} {'max us':>10s} {'share':>7s} {'last-n mean':>14s}")
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        n = min(len(v), tail) if tail else max(1, len(v) // 3)
        last = v[-n:]
        print(f"{short(k):50s} {len(v):6d} {sum(v) / len(v):10.1f} {min(v):10.1f} {max(v):10.1f} "
              f"{100 * sum(v) / total:6.1f}% {sum(last) / len(last):9.1f} ({n})")


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("counters", "trace"):
        sys.exit(__doc__)
    if sys.argv[1] == "counters":
        counters(sys.argv[2:])
    else:
        trace(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else None)
