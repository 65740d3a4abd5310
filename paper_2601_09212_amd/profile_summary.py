"""Collect and summarise the rocprofv3 evidence for one benchmark workload.

    python3 -m paper_2601_09212_amd.profile_summary --workload cfg5 --raw DIR --out FILE.md [--sq] [-- bench flags]

runs, each as a child process of its own and from /tmp (rocprofv3 writes temporary files beside
itself), with `python3 bench.py ...` directly after rocprofv3's `--`:

  1. `rocprofv3 --kernel-trace --stats`   over `bench.py --launch direct` (one library call per step)
  2. `rocprofv3 --pmc FETCH_SIZE`         over `bench.py --counter-run`
  3. `rocprofv3 --pmc WRITE_SIZE`         over `bench.py --counter-run`
  4. with --sq: `rocprofv3 --pmc <eight SQ counters>` over `bench.py --counter-run` (instruction mix,
     VALU / LDS busy cycles and LDS bank conflicts of every kernel)

and writes a short text summary: per-kernel launch statistics, HBM bytes per launch of every library
kernel, and the line

    traffic_bytes_per_launch: <dominant kernel> <bytes>

which bench.py reads back as `roofline.traffic`.  A counter-run first launches five reference
copies (`dst = src * 1`, 2^30 B in and 2^30 B out); FETCH_SIZE and WRITE_SIZE readings are turned
into bytes with what the same counter read for those copies in the same run, so no unit is assumed.
`--no-collect` only re-writes the summary from raw files that are already there.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SQ_COUNTERS = ["SQ_WAVES", "SQ_BUSY_CU_CYCLES", "SQ_WAVE_CYCLES", "SQ_INSTS_VALU", "SQ_ACTIVE_INST_VALU", "SQ_INSTS_LDS",
               "SQ_ACTIVE_INST_LDS", "SQ_LDS_BANK_CONFLICT"]
COPY_BYTES = 1 << 30
COUNTER_STEPS = 20          # library calls in a counter run


def commands(workload, raw, flags, sq, trace_only=False):
    bench = ["python3", os.path.join(ROOT, "bench.py"), "--no-others", "--workload", workload]
    prof = ["rocprofv3", "--output-format", "csv"]
    trace = prof + ["--kernel-trace", "--stats", "-d", os.path.join(raw, "trace"), "-o", "t", "--"] + bench + \
        ["--launch", "direct", "--steps", "300", "--warmup", "30", "--no-cpu-baseline"] + flags
    out = [("trace", trace, 240)]
    if trace_only:
        return out
    passes = [("fetch", ["FETCH_SIZE"]), ("write", ["WRITE_SIZE"])] + ([("sq", SQ_COUNTERS)] if sq else [])
    for name, counters in passes:
        out.append((name, prof + ["--pmc"] + counters + ["-d", os.path.join(raw, name), "-o", name[0], "--"] + bench +
                    ["--counter-run", "--steps", str(COUNTER_STEPS)] + flags, 150))
    return out


def collect(workload, raw, flags, sq, trace_only=False):
    env = dict(os.environ, TMPDIR="/tmp")
    for name, cmd, limit in commands(workload, raw, flags, sq, trace_only):
        print("[profile_summary]", name, flush=True)
        with open(os.path.join(raw, name + ".log"), "w") as log:
            try:
                rc = subprocess.run(cmd, cwd="/tmp", env=env, stdout=log, stderr=subprocess.STDOUT, timeout=limit).returncode
            except subprocess.TimeoutExpired:
                sys.exit("profile_summary: the %s pass did not finish in %d s; nothing further is run" % (name, limit))
        if rc != 0:
            sys.exit("profile_summary: the %s pass failed with status %d (see %s.log)" % (name, rc, name))
    for f in glob.glob(os.path.join(raw, "trace", "**", "*_kernel_trace.csv"), recursive=True):
        os.remove(f)     # one line per launch: large, and the statistics file holds what is used


def short(name):
    return re.sub(r"\(.*$", "", name).replace("void ", "")[:92]


def ours(name):
    return "csd::" in name


def one(pattern):
    files = glob.glob(pattern, recursive=True)
    if not files:
        sys.exit("profile_summary: no file matches " + pattern)
    return files[0]


def kernel_stats(raw):
    rows = [r for r in csv.DictReader(open(one(os.path.join(raw, "trace", "**", "*kernel_stats.csv")))) if ours(r["Name"])]
    return [(short(r["Name"]), int(r["Calls"]), float(r["AverageNs"]) / 1e3, float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
             float(r["TotalDurationNs"]) / 1e3) for r in rows]


def counter_rows(raw, sub):
    rows = list(csv.DictReader(open(one(os.path.join(raw, sub, "**", "*counter_collection.csv")))))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    return rows


def byte_counter(raw, sub, counter):
    """-> ({kernel: (launches, mean reading)}, mean reading of the reference copies, bytes per unit)"""
    rows = [r for r in counter_rows(raw, sub) if r["Counter_Name"] == counter]
    first = next(i for i, r in enumerate(rows) if ours(r["Kernel_Name"]) and "zero_words" not in r["Kernel_Name"])
    # the reference copies: the last five elementwise launches before the first library kernel
    ref = [float(r["Counter_Value"]) for r in rows[:first] if "elementwise" in r["Kernel_Name"]][-5:]
    if len(ref) != 5:
        sys.exit("profile_summary: reference copies not found in the %s run" % sub)
    refv = sum(ref) / 5
    acc = collections.OrderedDict()
    for r in rows:
        if ours(r["Kernel_Name"]):
            acc.setdefault(short(r["Kernel_Name"]), []).append(float(r["Counter_Value"]))
    return {k: (len(v), sum(v) / len(v)) for k, v in acc.items()}, refv, COPY_BYTES / refv


def sq_counters(raw):
    acc = collections.OrderedDict()
    for r in counter_rows(raw, "sq"):
        if ours(r["Kernel_Name"]):
            acc.setdefault(short(r["Kernel_Name"]), collections.defaultdict(list))[r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in acc.items()}


def bench_line(raw):
    for ln in open(os.path.join(raw, "trace.log")):
        if ln.startswith("{"):
            d = json.loads(ln)
            keys = ("bound", "achieved", "peak", "unit", "frac", "kernel", "us_per_launch", "whole_call_us", "whole_call_frac",
                    "graph_step_us", "direct_call_us")
            return {"value": d["value"], "ms_per_step": d["ms_per_step"], "config": d["config"],
                    "roofline": {k: d["roofline"].get(k) for k in keys}}
    return None


def summary(workload, raw, flags, sq, trace_only=False):
    lines = []
    stats = kernel_stats(raw)
    lines.append("== kernel trace (rocprofv3 --kernel-trace --stats), library kernels, times in us")
    for n, calls, avg, lo, hi, _ in stats:
        lines.append("%-92s calls=%5d avg=%9.2f min=%9.2f max=%9.2f" % (n, calls, avg, lo, hi))
    timed = [s for s in stats if "read_probe" not in s[0]]
    dominant = max(timed, key=lambda s: s[5])[0]
    total, per_call = {}, 0.0
    for counter, sub in (() if trace_only else (("FETCH_SIZE", "fetch"), ("WRITE_SIZE", "write"))):
        per_kernel, refv, per_unit = byte_counter(raw, sub, counter)
        lines.append("== %s: mean reading per launch -> bytes (bytes per unit from the reference copy: %.1f)" % (counter, per_unit))
        for k, (n, m) in per_kernel.items():
            lines.append("%-92s n=%3d reading=%12.1f -> %14.0f B" % (k, n, m, m * per_unit))
            total[k] = total.get(k, 0.0) + m * per_unit
            if "zero_words" not in k and "read_probe" not in k:
                per_call += n * m * per_unit / COUNTER_STEPS
        lines.append("%-92s n=%3d reading=%12.1f -> %14.0f B" % ("reference copy (2^30 B each way)", 5, refv, refv * per_unit))
    if sq:
        lines.append("== SQ counters: mean per launch, summed over the chip (cycles are per-SIMD / per-CU cycle counts as the counter defines them)")
        for k, d in sq_counters(raw).items():
            lines.append(k)
            lines.append("    " + "  ".join("%s=%.4g" % (c, d[c]) for c in SQ_COUNTERS if c in d))
            if d.get("SQ_BUSY_CU_CYCLES") and d.get("SQ_WAVES"):
                lines.append("    per wave: VALU instructions %.0f, LDS instructions %.0f; VALU-active / CU-busy cycles %.3f, "
                             "LDS-active / CU-busy %.3f, bank-conflict / LDS-active cycles %.3f" %
                             (d["SQ_INSTS_VALU"] / d["SQ_WAVES"], d["SQ_INSTS_LDS"] / d["SQ_WAVES"],
                              d["SQ_ACTIVE_INST_VALU"] / d["SQ_BUSY_CU_CYCLES"], d["SQ_ACTIVE_INST_LDS"] / d["SQ_BUSY_CU_CYCLES"],
                              d["SQ_LDS_BANK_CONFLICT"] / max(d["SQ_ACTIVE_INST_LDS"], 1.0)))
    if not trace_only and dominant not in total:
        sys.exit("profile_summary: no counter reading for " + dominant)
    traffic = "(trace only: no counter passes)" if trace_only else (
        "HBM bytes (FETCH_SIZE + WRITE_SIZE) per launch of the kernel with the largest share of the time:\n\n"
        "traffic_bytes_per_launch: %s %.0f" % (dominant.split("<")[0], total[dominant]))
    if not trace_only and not any(f in flags for f in ("--lantern", "--diagnostics")):
        # (runs with those flags also make calls of other entry points: no per-call figure)
        traffic += ("\n\nand of all launches of one cool_sd_verify call (the counter runs make %d calls):\n\n"
                    "traffic_bytes_per_call: %.0f" % (COUNTER_STEPS, per_call))
    cmds = "\n".join("    (cd /tmp; TMPDIR=/tmp " + " ".join(
        c.replace(raw, "RAW").replace(ROOT + "/", "") for c in cmd) + ")" for _, cmd, _ in commands(workload, raw, flags, sq, trace_only))
    bl = bench_line(raw)
    text = """# rocprofv3 summary: bench.py --workload %s%s

MI355X (gfx950), ROCm 7.2.0, one GPU.  Written by

    python3 -m paper_2601_09212_amd.profile_summary --workload %s --raw RAW --out THIS_FILE%s%s

which runs

%s

and reads RAW/trace/**/t_kernel_stats.csv and the per-dispatch counter files.  The trace covers every
launch of the run (warm-up, timed steps, the instrumented passes; the statistics kernel is also
launched alone, hence its higher count).  Kernel names carry their template arguments:
row_stats_kernel<dtype (1 = bf16), logit transform, load mode (2 = 16-byte nontemporal), tiles per
chunk, 3-D grid, neighbour aggregation appended>; row_stats_topk_kernel<dtype, load mode, threads
per row, guidance, 3-D grid>; sequence_*_kernel<dtype, logit transform, aligned rows, ...>.

```
%s
```

%s

bench.py's JSON line in the traced run (slower than an untraced run; compare the trace's average
for the dominant kernel with `roofline.us_per_launch` of an untraced run):

```
%s
```
""" % (workload, (" " + " ".join(flags)) if flags else "", workload, (" --sq" if sq else "") + (" --trace-only" if trace_only else ""),
       (" -- " + " ".join(flags)) if flags else "", cmds, "\n".join(lines), traffic, json.dumps(bl, indent=1))
    return text


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", required=True)
    ap.add_argument("--raw", required=True, help="folder for rocprofv3's output (created)")
    ap.add_argument("--out", required=True, help="the summary to write")
    ap.add_argument("--sq", action="store_true", help="also collect the SQ instruction / LDS counters")
    ap.add_argument("--trace-only", action="store_true", help="kernel trace only, no counter passes (no traffic line)")
    ap.add_argument("--no-collect", action="store_true", help="raw files are already there: only write the summary")
    ap.add_argument("flags", nargs="*", help="after --: further flags for bench.py (--early-exit, --lantern, ...)")
    a = ap.parse_args()
    raw = os.path.abspath(a.raw)
    os.makedirs(raw, exist_ok=True)
    if not a.no_collect:
        collect(a.workload, raw, a.flags, a.sq, a.trace_only)
    text = summary(a.workload, raw, a.flags, a.sq, a.trace_only)
    with open(a.out, "w") as f:
        f.write(text)
    print("[profile_summary] wrote", a.out, flush=True)


if __name__ == "__main__":
    main()
