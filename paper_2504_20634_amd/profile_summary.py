"""Turn rocprofv3's CSV output for `bench.py` into the short summaries kept under profiles/.

The runs this reads (each a run of its own: rocprofv3 does not split counters over passes), all of the same program,

    python3 bench.py --no-cpu-baseline --no-workloads [--copy-probe]

  --kernel-trace --stats --output-format csv           -> <kt>/..._kernel_stats.csv  and the program's JSON line
  --pmc FETCH_SIZE      (with --copy-probe)            -> <fetch>/..._counter_collection.csv
  --pmc WRITE_SIZE      (with --copy-probe)            -> <write>/..._counter_collection.csv
  --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_WAVES  -> <sq>/..._counter_collection.csv
  --pmc VALUBusy                                       -> <busy>/..._counter_collection.csv

and what it writes:

  profiles/bench_2p28_kernel_trace.md      per kernel: launches, mean / min / max duration, beside bench.py's own
                                           event timing of the same run
  profiles/kernels_2p28_hbm_traffic.md     fetched and written KiB per launch against the algorithmic bytes
  profiles/kernels_2p28_valu_counters.md   vector-ALU instructions per element, VALUBusy
  profiles/kernel_counters.json            the figures bench.py reports (traffic of the headline kernel, VALU per
                                           element and VALUBusy per path), with the sha256 of the kernel sources
                                           they belong to: bench.py leaves them out when the sources have changed

It holds none of the method's arithmetic and calls nothing on the GPU.
"""
import argparse
import csv
import glob
import json
import os
import sys
from collections import defaultdict

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def short_name(full):
    """'void fbsr::round_tiles<1, 1, 2>(float const*, ...)' -> 'fbsr::round_tiles<1, 1, 2>'."""
    s = full.strip()
    if s.startswith("void "):
        s = s[5:]
    depth = 0
    for i, ch in enumerate(s):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return s[:i]
    return s


def one_csv(folder, suffix):
    found = sorted(glob.glob(os.path.join(folder, "**", "*" + suffix), recursive=True))
    if not found:
        raise SystemExit("no *%s under %s" % (suffix, folder))
    return found[0]


def read_stats(folder, timed):
    """kernel -> launches and mean / min / max duration of its LAST timed[kernel] launches (all, for a kernel without
    an entry): bench.py warms every path up with launches of the same call, so a kernel's last launches are the ones
    it timed (where two of its lines share a kernel, those of the second and the end of its warm-up)."""
    spans = defaultdict(list)
    with open(one_csv(folder, "_kernel_trace.csv"), newline="") as fh:
        for row in csv.DictReader(fh):
            spans[short_name(row["Kernel_Name"])].append((int(row["Start_Timestamp"]), int(row["End_Timestamp"])))
    out = {}
    for k, rows in spans.items():
        rows.sort()
        last = rows[-timed[k]:] if timed.get(k) else rows
        d = [(e - s) / 1e3 for s, e in last]
        out[k] = {"calls": len(rows), "used": len(d), "avg_us": sum(d) / len(d), "min_us": min(d), "max_us": max(d)}
    return out


def read_counters(folder):
    """kernel -> counter -> (mean per dispatch, dispatches)."""
    sums = defaultdict(lambda: defaultdict(float))
    seen = defaultdict(lambda: defaultdict(int))
    with open(one_csv(folder, "_counter_collection.csv"), newline="") as fh:
        for row in csv.DictReader(fh):
            k = short_name(row["Kernel_Name"])
            sums[k][row["Counter_Name"]] += float(row["Counter_Value"])
            seen[k][row["Counter_Name"]] += 1
    return {k: {c: (sums[k][c] / seen[k][c], seen[k][c]) for c in sums[k]} for k in sums}


def bench_entries(bench):
    """kernel -> {"labels": [...], "ms": mean of bench.py's own timings, "elements", "bytes"} from the JSON line."""
    by_kernel = {}
    for group in ("per_launch", "paths"):
        for label, e in bench.get(group, {}).items():
            k = e.get("kernel")
            if not k:
                continue
            d = by_kernel.setdefault(k, {"labels": [], "ms": [], "elements": e["elements"], "bytes": e["gb_s"] * e["ms"] * 1e6, "launches": 0})
            d["labels"].append(label)
            d["ms"].append(e["ms"])
            d["launches"] += e.get("launches", bench["steps"])   # a headline kernel runs once per step
    for d in by_kernel.values():
        d["ms"] = sum(d["ms"]) / len(d["ms"])
    return by_kernel


COPY_KERNEL = "__amd_rocclr_copyBuffer"


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--bench-json", required=True, help="the JSON line bench.py printed under the kernel-trace run")
    ap.add_argument("--kt", required=True)
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--sq")
    ap.add_argument("--busy")
    ap.add_argument("--bench-args", default="--no-cpu-baseline --no-workloads")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles"))
    args = ap.parse_args()

    import bench as bench_module
    with open(args.bench_json) as fh:
        line = [l for l in fh if l.lstrip().startswith("{")][-1]
    bench = json.loads(line)
    entries = bench_entries(bench)
    n = bench["config"]["elements"]
    tag = "2p%d" % (n.bit_length() - 1)
    prog = "python3 bench.py " + args.bench_args
    pre = "TMPDIR=/tmp "          # the commands are run from the repository root
    out_dir = {k: os.path.relpath(getattr(args, k), ROOT) if getattr(args, k) else "<dir>" for k in ("kt", "fetch", "write", "sq", "busy")}
    os.makedirs(args.out, exist_ok=True)
    figures = {"sources_sha256": bench_module.kernel_sources_hash(), "program": prog, "elements": n}

    # ---- kernel trace
    stats = read_stats(args.kt, {k: e["launches"] for k, e in entries.items()})
    rows = []
    for k in sorted(stats, key=lambda k: (k not in entries, k)):
        if not k.startswith("fbsr::"):
            continue
        s, e = stats[k], entries.get(k)
        rows.append("| %s | %d | %d | %.1f | %.1f | %.1f | %s | %s | %s |" % (
            k.replace("fbsr::", ""), s["calls"], s["used"], s["avg_us"], s["min_us"], s["max_us"],
            "%.1f" % (e["ms"] * 1e3) if e else "", "%.0f" % (e["bytes"] / s["avg_us"] / 1e3) if e else "",
            ", ".join(e["labels"]) if e else ""))
    head = [k for k in entries if any(l in bench["per_launch"] for l in entries[k]["labels"])]
    head_avg = sum(stats[k]["avg_us"] for k in head if k in stats) / max(1, sum(1 for k in head if k in stats))
    with open(os.path.join(args.out, "bench_%s_kernel_trace.md" % tag), "w") as fh:
        fh.write("# rocprofv3 --kernel-trace --stats of bench.py, 2^%d elements (MI355X, gfx950)\n\nCommand:\n\n" % (n.bit_length() - 1))
        fh.write("    %srocprofv3 --kernel-trace --stats --output-format csv -d %s -o kt \\\n        -- %s\n\n" % (pre, out_dir["kt"], prog))
        fh.write("Durations in microseconds, over a kernel's last `timed` launches: bench.py first keeps the GPU busy with\n"
                 "launches of the same call for 40 ms (the clocks dip for some tens of milliseconds when load sets in) and then\n"
                 "times a dozen.  `bench us` is bench.py's own HIP-event timing of those launches in the same run (events\n"
                 "include the gap between launches, so they read a few us above the trace); GB/s = algorithmic bytes per\n"
                 "launch / the trace's mean duration.  Kernels with no bench line are helper launches.\n\n")
        fh.write("Headline (`roofline` of the JSON line): the 18 `round_tiles<fmt, variant, W>` kernels of a step, fmt 1|2, variant 1..3,\n"
                 "W 2|4|8: mean of their mean durations %.1f us = %.0f GB/s of 5 B/element (bench.py's events: %.1f us, %.0f GB/s).\n\n"
                 % (head_avg, 5.0 * n / head_avg / 1e3, bench["roofline"]["avg_launch_ms"] * 1e3, bench["roofline"]["achieved"]))
        fh.write("| kernel | launches | timed | mean | min | max | bench us | GB/s | bench.py line |\n|---|---|---|---|---|---|---|---|---|\n")
        fh.write("\n".join(rows) + "\n")
    figures["headline_trace_avg_us"] = round(head_avg, 2)

    # ---- HBM traffic
    if args.fetch and args.write:
        fetch, write = read_counters(args.fetch), read_counters(args.write)
        copy_kib = 4.0 * n / 1024
        f_scale = copy_kib / fetch[COPY_KERNEL]["FETCH_SIZE"][0]
        w_scale = copy_kib / write[COPY_KERNEL]["WRITE_SIZE"][0]
        rows, traffic = [], {}
        for k in sorted(fetch, key=lambda k: (k not in entries, k)):
            if not k.startswith("fbsr::") or k not in write or k not in entries:
                continue
            f = fetch[k]["FETCH_SIZE"][0] * f_scale
            w = write[k]["WRITE_SIZE"][0] * w_scale
            alg = entries[k]["bytes"] / 1024
            traffic[k] = (f + w) * 1024
            rows.append("| %s | %d | %.0f | %.0f | %.0f | %.5f |" % (k.replace("fbsr::", ""), fetch[k]["FETCH_SIZE"][1], f, w, alg, (f + w) / alg))
        headline = [traffic[k] for k in head if k in traffic]
        if headline:
            figures["headline_traffic_bytes_%s" % tag] = int(round(sum(headline) / len(headline)))
        figures["traffic_bytes"] = {l: int(round(traffic[k])) for k in traffic for l in entries[k]["labels"] if l in bench.get("paths", {})}
        with open(os.path.join(args.out, "kernels_%s_hbm_traffic.md" % tag), "w") as fh:
            fh.write("# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE: every kernel bench.py times, 2^%d elements (2^27 for the fused updates)\n\n" % (n.bit_length() - 1))
            fh.write("Commands (one counter per run):\n\n    %srocprofv3 --pmc FETCH_SIZE --output-format csv -d %s -o f \\\n        -- %s --copy-probe\n" % (pre, out_dir["fetch"], prog))
            fh.write("    ... the same with --pmc WRITE_SIZE -d %s -o w\n\n" % out_dir["write"])
            fh.write("Counters (KiB per dispatch) scaled by what they read for the plain 1 GiB device copy of the same run\n"
                     "(FETCH_SIZE x %.5f, WRITE_SIZE x %.5f), mean per launch.  Algorithmic KiB: inputs once, outputs once\n"
                     "(what bench.py's GB/s figures count).\n\n" % (f_scale, w_scale))
            if headline:
                fh.write("Headline kernels (mean of the 18): %d bytes per launch against %d algorithmic.\n\n" % (figures["headline_traffic_bytes_%s" % tag], 5 * n))
            fh.write("| kernel | launches | fetched KiB | written KiB | algorithmic KiB | traffic / algorithmic |\n|---|---|---|---|---|---|\n")
            fh.write("\n".join(rows) + "\n")

    # ---- vector-ALU counters
    if args.sq:
        sq = read_counters(args.sq)
        busy = read_counters(args.busy) if args.busy else {}
        rows = []
        figures["valu_per_elem"], figures["valu_busy_pct"] = {}, {}
        for k in sorted(sq, key=lambda k: (k not in entries, k)):
            if not k.startswith("fbsr::") or k not in entries:
                continue
            c, e = sq[k], entries[k]
            waves = c["SQ_WAVES"][0]
            valu = c["SQ_INSTS_VALU"][0]
            per_elem = valu * 64.0 / e["elements"]
            b = busy.get(k, {}).get("VALUBusy", (None,))[0]
            rate = per_elem * e["elements"] / (stats[k]["avg_us"] * 1e-6) if k in stats else None
            rows.append("| %s | %d | %.1f | %.1f | %.1f | %.1f | %s | %s |" % (
                k.replace("fbsr::", ""), waves, valu / waves, c["SQ_INSTS_SALU"][0] / waves, c["SQ_INSTS_LDS"][0] / waves, per_elem,
                "%.1f" % (rate / 1e12) if rate else "", "%.0f %%" % b if b is not None else ""))
            for l in e["labels"]:
                if l in bench.get("paths", {}):
                    figures["valu_per_elem"][l] = round(per_elem, 1)
                    if b is not None:
                        figures["valu_busy_pct"][l] = round(b, 1)
        with open(os.path.join(args.out, "kernels_%s_valu_counters.md" % tag), "w") as fh:
            fh.write("# rocprofv3 --pmc SQ instruction counters per kernel: bench.py, 2^%d elements (MI355X, gfx950)\n\nCommands:\n\n" % (n.bit_length() - 1))
            fh.write("    %srocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_WAVES --output-format csv -d %s -o sq \\\n        -- %s\n" % (pre, out_dir["sq"], prog))
            fh.write("    ... and, in a run of its own, --pmc VALUBusy -d %s -o b\n\n" % out_dir["busy"])
            fh.write("VALU/elem = SQ_INSTS_VALU x 64 lanes / elements per launch: one-lane vector operations per element, idle lanes of\n"
                     "an issued instruction included.  T lane-ops/s = VALU/elem x elements / the kernel-trace mean duration; the\n"
                     "ceiling bench.py prices it against is 78.6 T/s (the chip's 157.3 TFLOP/s of fp32 FMA at two flops each); plain\n"
                     "adds, logic ops and right shifts sustain 57..60 T/s here, left shifts, three-operand ops, converts and\n"
                     "multiplies 34 T/s, so an instruction mix decides how close a kernel can come.  VALUBusy is rocprofv3's derived\n"
                     "metric: the share of the kernel's time with vector-ALU work in flight.\n\n")
            fh.write("| kernel | waves | VALU/wave | SALU/wave | LDS/wave | VALU/elem | T lane-ops/s | VALUBusy |\n|---|---|---|---|---|---|---|---|\n")
            fh.write("\n".join(rows) + "\n")

    missing = [l for g in ("paths",) for l, e in bench.get(g, {}).items() if e.get("kernel") and e["kernel"] not in stats]
    if missing:
        print("bench lines whose kernel name is not in the trace: %s" % ", ".join(missing), file=sys.stderr)
    with open(os.path.join(args.out, "kernel_counters.json"), "w") as fh:
        json.dump(figures, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("wrote %s" % args.out)


if __name__ == "__main__":
    main()
