"""Turn rocprofv3 csv output and bench.py JSON lines into the short text summaries kept under profiles/.

    python -m paper_1804_08066_amd.rocprof_summary <subcommand> ...

Subcommands (each writes one markdown file; the commands that produced the inputs are passed in and
printed at the top of the summary, so a reader can repeat the measurement):

  stats      per-kernel call count / average / min / max from `rocprofv3 --kernel-trace --stats`
  sweep      one row per (bits, bucket, workers) point, from one stats run + bench.py JSON per point
  traffic    HBM bytes per launch from two `--pmc` runs (FETCH_SIZE, WRITE_SIZE), scaled by a copy of
             known size; ends with the `traffic_json:` line that bench.py reads
  counters   mean SQ counter values per dispatch and the derived vector-ALU operations per element
  transient  bench.py --transient: per-step launch times after input generation / idle / settled
  machine    bench.py --machine-state: rocm-smi clock levels
"""
import argparse
import collections
import csv
import json
import os
import subprocess
import sys

# matched as substrings, first hit wins: a name that contains another comes before it
KERNELS = ("requantize_wave_kernel", "requantize_pack_kernel", "requantize_minmax_tensor_kernel", "requantize_minmax_kernel",
           "sum_range_minmax_tensor_kernel", "aggregate_update_rows_kernel", "aggregate_update_lds_kernel",
           "aggregate_update_minmax_tensors_kernel", "aggregate_update_minmax_kernel", "aggregate_update_tensors_kernel",
           "aggregate_mean_kernel", "tensor_range_batch_kernel", "tensor_range_kernel", "sum_squares_partial_kernel",
           "sum_squares_finish_kernel", "sum_squares_kernel", "quantize_minmax_tensors_wave_kernel",
           "quantize_minmax_tensors_kernel", "quantize_minmax_wave_kernel", "quantize_minmax_kernel",
           "quantize_tensors_wave_kernel", "quantize_tensors_cells_kernel", "quantize_tensors_kernel", "quantize_wave_kernel",
           "quantize_cells_kernel", "quantize_pack_kernel", "stream_quantize_kernel", "stream_update_kernel", "range_",
           "clear_", "finish_")


def short(name):
    """Library kernel name without template arguments; torch's copy kernel as 'plain copy'; else None."""
    for k in KERNELS:
        if k in name:
            return name.split("(anonymous namespace)::")[-1].split("<")[0].split("(")[0] if k.endswith("_") else k
    if "copybuffer" in name.lower():   # the runtime's device-to-device copy kernel, which torch's copy_ runs
        return "plain copy (torch copy_)"
    return None


_measured_at = None   # --measured-at: the commit the measurement ran on, when the summary is written later


def commit():
    if _measured_at:
        return _measured_at
    try:
        root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        h = subprocess.run(["git", "rev-parse", "--short", "HEAD"], cwd=root, capture_output=True, text=True).stdout.strip()
        dirty = subprocess.run(["git", "status", "--porcelain", "--untracked-files=no", "--", ".", ":!profiles"], cwd=root,
                               capture_output=True, text=True).stdout.strip()   # the summaries themselves do not count
        return h + ("+changes" if dirty else "")
    except OSError:
        return "unknown"


def last_json(path):
    lines = [ln for ln in open(path).read().strip().split("\n") if ln.startswith("{")]
    return json.loads(lines[-1])


def kernel_stats(path):
    """{short name: (calls, average ns, min ns, max ns)} merged over template instances."""
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        s = short(r["Name"])
        if not s:
            continue
        c, a = int(r["Calls"]), float(r["AverageNs"])
        if s in agg:
            o = agg[s]
            agg[s] = (o[0] + c, (o[1] * o[0] + a * c) / (o[0] + c), min(o[2], int(r["MinNs"])), max(o[3], int(r["MaxNs"])))
        else:
            agg[s] = (c, a, int(r["MinNs"]), int(r["MaxNs"]))
    return agg


def write(path, lines):
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    print("wrote", path)


def head(title, cmds):
    out = ["# " + title, "", "Measured at commit %s.  Command%s (from the repository root on an MI355X box):" %
           (commit(), "s" if len(cmds) > 1 else ""), ""]
    out += ["    " + c for c in cmds]
    out.append("")
    return out


def cmd_stats(a):
    out = head(a.title, a.cmd)
    out += ["| kernel | calls | average ns | min ns | max ns |", "|---|---|---|---|---|"]
    for k, v in kernel_stats(a.csv).items():
        if "copy" not in k:
            out.append("| %s | %d | %.0f | %d | %d |" % (k, v[0], v[1], v[2], v[3]))
    out.append("")
    if a.bench_json:
        d = last_json(a.bench_json)
        out.append("Same run, bench.py's HIP-event averages over its timed region: quantize %.2f us per launch, "
                   "aggregate_update %.2f us per launch, %.3f ms per step (value %.0f GB/s).  The rocprofv3 averages also "
                   "cover the cold region, the conditioning steps and the warm-up." %
                   (d["roofline"]["avg_launch_us"], d["roofline_aggregate"]["avg_launch_us"], d["ms_per_step"], d["value"]))
    for n in a.note or []:
        out.append(n)
    write(a.out, out)


def cmd_sweep(a):
    out = head(a.title, a.cmd)
    out += ["| bits | bucket | workers | code stores | quantize kernel | calls | avg us (rocprofv3) | avg us (HIP events) | % of 8 TB/s | "
            "streaming ceiling us | server kernel | calls | avg us (rocprofv3) | avg us (HIP events) | % of 8 TB/s | "
            "streaming ceiling us |",
            "|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|---|"]
    for spec in a.run:
        point, sdir, jpath = spec.split(":")
        b, B, W = (int(x) for x in point.split(","))
        ks = kernel_stats(os.path.join(sdir, "stats_kernel_stats.csv"))
        d = last_json(jpath)
        qk = next((k for k in ks if k.startswith("quantize")), None)
        sk = next((k for k in ks if k.startswith("aggregate")), None)
        r, ra = d["roofline"], d["roofline_aggregate"]
        ce = d.get("stream_ceiling") or {}
        cq = "%.1f" % ce["quantize_mix"]["us"] if ce else "-"
        cu = "%.1f" % ce["update_mix"]["us"] if ce else "-"
        policy = (d.get("config", {}).get("code_stores") or {}).get("chosen", "cached")
        out.append("| %d | %d | %d | %s | %s | %d | %.1f | %.1f | %.1f | %s | %s | %d | %.1f | %.1f | %.1f | %s |" %
                   (b, B, W, policy, qk, ks[qk][0], ks[qk][1] / 1e3, r["avg_launch_us"], 100 * r["frac"], cq,
                    sk, ks[sk][0], ks[sk][1] / 1e3, ra["avg_launch_us"], 100 * ra["frac"], cu))
    out.append("")
    out.append("The HIP-event columns are bench.py's averages over its timed region (after the conditioning steps); the "
               "rocprofv3 columns average every launch of the process, the cold region and the warm-up included.  "
               "Percentages: algorithmic bytes per launch / HIP-event time / 8 TB/s.  Streaming ceiling: the time of "
               "bench.py's streaming kernel for that kernel's read/write mix in the same run (same loads and stores, no "
               "arithmetic; HIP events).  Code stores: the cache policy of the quantizer's code words that bench.py's untimed "
               "probe chose for the point (mqg_quantize_to: kept cached for the update, or streamed to memory).")
    write(a.out, out)


def cmd_traffic(a):
    vals = {}
    for name, f in (("FETCH_SIZE", a.fetch), ("WRITE_SIZE", a.write)):
        acc = collections.defaultdict(list)
        for r in csv.DictReader(open(f)):
            s = short(r["Kernel_Name"])
            if s and r["Counter_Name"] == name:
                acc[s].append(float(r["Counter_Value"]))
        for k, v in acc.items():
            vals[(k, name)] = (len(v), sum(v) / len(v))
    copy = "plain copy (torch copy_)"
    kib = 4.0 * a.n / 1024.0
    fs, ws = kib / vals[(copy, "FETCH_SIZE")][1], kib / vals[(copy, "WRITE_SIZE")][1]
    out = head(a.title, a.cmd)
    out.append("`--calibrate-copy` adds three plain device copies of one gradient buffer (torch copy_, %d bytes read and "
               "written = %.0f KiB each way): the kernel of known size that the counters are scaled by." % (4 * a.n, kib))
    out += ["", "| kernel | dispatches | FETCH_SIZE mean (KiB) | WRITE_SIZE mean (KiB) |", "|---|---|---|---|"]
    kernels = [k for k in ("quantize_wave_kernel", "quantize_pack_kernel", "aggregate_update_rows_kernel",
                           "aggregate_update_lds_kernel") if (k, "FETCH_SIZE") in vals]
    for k in [copy] + kernels:
        out.append("| %s | %d | %.1f | %.1f |" % (k, vals[(k, "FETCH_SIZE")][0], vals[(k, "FETCH_SIZE")][1], vals[(k, "WRITE_SIZE")][1]))
    out += ["", "Scale factors from the copy (true KiB / counter KiB): FETCH_SIZE x %.4f, WRITE_SIZE x %.4f." % (fs, ws), "",
            "| kernel | HBM read (MB) | HBM written (MB) | total (MB) | algorithmic bytes (MB) | traffic / algorithmic |",
            "|---|---|---|---|---|---|"]
    nb = (a.n + a.bucket - 1) // a.bucket
    alg = {"quantize": 4 * a.n + a.n * a.bits / 8 + 4 * nb, "aggregate": a.workers * (a.n * a.bits / 8 + 4 * nb) + 8 * a.n}
    res = {"workload": {"n": a.n, "workers": a.workers, "bits": a.bits, "bucket": a.bucket}, "commit": commit()}
    for k in kernels:
        rd = vals[(k, "FETCH_SIZE")][1] * fs * 1024 / 1e6
        wr = vals[(k, "WRITE_SIZE")][1] * ws * 1024 / 1e6
        al = alg["quantize" if "quantize" in k else "aggregate"]
        out.append("| %s | %.1f | %.1f | %.1f | %.1f | %.3f |" % (k, rd, wr, rd + wr, al / 1e6, (rd + wr) / (al / 1e6)))
        res[k] = round((rd + wr) * 1e6)
    out += ["", "Reads of the server kernel below its algorithmic bytes are code words that the quantize launches of the same "
            "step left in the last-level cache.", "", "traffic_json: " + json.dumps(res)]
    write(a.out, out)


def cmd_counters(a):
    vals = collections.defaultdict(lambda: collections.defaultdict(list))
    for f in a.csv:
        for r in csv.DictReader(open(f)):
            k = short(r["Kernel_Name"])
            if k in a.kernel:
                vals[k][r["Counter_Name"]].append(float(r["Counter_Value"]))
    names = []
    for k in a.kernel:
        for c in vals[k]:
            if c not in names:
                names.append(c)
    mean = lambda k, c: (sum(vals[k][c]) / len(vals[k][c])) if vals[k][c] else float("nan")
    out = head(a.title, a.cmd)
    out += ["Mean counter value per dispatch (as rocprofv3 reports it, summed over the chip):", "",
            "| counter | " + " | ".join(a.kernel) + " |", "|---|" + "---|" * len(a.kernel)]
    for c in names:
        out.append("| %s | " % c + " | ".join("%.4g" % mean(k, c) for k in a.kernel) + " |")
    out += ["", "Derived (n = %d elements per dispatch; a wave instruction covers 64 lanes):" % a.n, ""]
    for k in a.kernel:
        line = "* %s: %.1f vector-ALU lane-operations per element (SQ_INSTS_VALU x 64 / n)" % (k, mean(k, "SQ_INSTS_VALU") * 64 / a.n)
        if vals[k]["SQ_ACTIVE_INST_VALU"] and vals[k]["SQ_BUSY_CYCLES"]:
            line += "; SQ_ACTIVE_INST_VALU x 4 / SQ_WAVE_CYCLES = %.3f" % (4 * mean(k, "SQ_ACTIVE_INST_VALU") / mean(k, "SQ_WAVE_CYCLES")) \
                if vals[k]["SQ_WAVE_CYCLES"] else ""
        if vals[k]["SQ_LDS_BANK_CONFLICT"] and mean(k, "SQ_ACTIVE_INST_LDS") > 0:
            line += "; LDS bank-conflict cycles / LDS-active cycles = %.3f" % (mean(k, "SQ_LDS_BANK_CONFLICT") / mean(k, "SQ_ACTIVE_INST_LDS"))
        out.append(line + ".")
    for n in a.note or []:
        out += ["", n]
    write(a.out, out)


def cmd_transient(a):
    d = last_json(a.bench_json)
    out = head(a.title, a.cmd)
    out.append("Per-step launch times (HIP events on the launch stream; one step = %d quantize launches + 1 aggregate_update; "
               "quantize figures are per launch), b = %d, bucket = %d.  rocm-smi is read after each series." %
               (d["config"]["workers"], d["config"]["bits"], d["config"]["bucket"]))
    for s in d["transient"]:
        q, ag = s["quantize_us"], s["aggregate_us"]
        out += ["", "## " + s["start"], "",
                "clock levels after the series: %s" % json.dumps(s["clocks_after"]), "",
                "| steps | quantize us (mean) | aggregate us (mean) |", "|---|---|---|"]
        for lo, hi in ((0, 1), (1, 3), (3, 8), (8, 16), (16, 24), (24, 40), (40, 80), (80, len(q))):
            if lo < len(q):
                hi = min(hi, len(q))
                out.append("| %d..%d | %.1f | %.1f |" % (lo, hi - 1, sum(q[lo:hi]) / (hi - lo), sum(ag[lo:hi]) / (hi - lo)))
        out += ["", "quantize, every step: " + " ".join("%.0f" % v for v in q)]
    for n in a.note or []:
        out += ["", n]
    write(a.out, out)


def cmd_machine(a):
    d = last_json(a.bench_json)
    ms = d["machine_state"]
    out = head(a.title, a.cmd)
    out += ["`bench.py --machine-state` starts `rocm-smi --showclocks --showperflevel --showpower` as a child process once "
            "right after the timed region and once while `mqg_quantize` runs back to back for two seconds.", "",
            "| state | sclk MHz | mclk MHz | performance level | power W |", "|---|---|---|---|---|"]
    for k, label in (("idle", "right after the timed region"), ("under_load", "under load")):
        v = ms.get(k, {})
        out.append("| %s | %s | %s | %s | %s |" % (label, v.get("sclk_mhz", "n/a"), v.get("mclk_mhz", "n/a"),
                                                  v.get("performance_level", "n/a"), v.get("power_w", "not reported to this user")))
    out += ["", "Load: %s.  Vector-ALU peaks are stated at 2.4 GHz and at the engine clock read here under load." % ms.get("load", "")]
    write(a.out, out)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="sub", required=True)

    def common(p):
        p.add_argument("--title", required=True)
        p.add_argument("--cmd", action="append", required=True, help="command that produced the input (repeatable)")
        p.add_argument("--out", required=True)
        p.add_argument("--note", action="append")
        p.add_argument("--measured-at", help="commit the measurement ran on (default: the work tree's HEAD, "
                                             "'+changes' if tracked files other than the summaries differ from it)")

    p = sub.add_parser("stats"); common(p)
    p.add_argument("--csv", required=True); p.add_argument("--bench-json")
    p = sub.add_parser("sweep"); common(p)
    p.add_argument("--run", action="append", required=True, help="bits,bucket,workers:<rocprofv3 output dir>:<bench json>")
    p = sub.add_parser("traffic"); common(p)
    p.add_argument("--fetch", required=True); p.add_argument("--write", required=True)
    p.add_argument("--n", type=int, default=100_000_000); p.add_argument("--workers", type=int, default=8)
    p.add_argument("--bits", type=int, default=4); p.add_argument("--bucket", type=int, default=1024)
    p = sub.add_parser("counters"); common(p)
    p.add_argument("--csv", action="append", required=True); p.add_argument("--kernel", action="append", required=True)
    p.add_argument("--n", type=int, default=100_000_000)
    p = sub.add_parser("transient"); common(p); p.add_argument("--bench-json", required=True)
    p = sub.add_parser("machine"); common(p); p.add_argument("--bench-json", required=True)
    a = ap.parse_args()
    global _measured_at
    _measured_at = a.measured_at
    {"stats": cmd_stats, "sweep": cmd_sweep, "traffic": cmd_traffic, "counters": cmd_counters,
     "transient": cmd_transient, "machine": cmd_machine}[a.sub](a)


if __name__ == "__main__":
    sys.exit(main())
