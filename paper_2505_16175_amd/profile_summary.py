"""Turns rocprofv3 CSV output of bench.py runs into the short text summaries kept under profiles/.

    python -m paper_2505_16175_amd.profile_summary --name cfg5_7b_hour_stack \\
        --kernel-trace prof/kt --fetch prof/fetch --write prof/write \\
        --bench-json prof/kt.json --command "<the bench.py arguments the three runs used>"

The three directories come from three runs of the SAME bench.py command (one counter per run; rocprofv3 does not
split counters over passes), from the repo root with TMPDIR=/tmp:

    rocprofv3 --kernel-trace --stats -d prof/kt    -o run --output-format csv -- python3 bench.py <args>
    rocprofv3 --pmc FETCH_SIZE       -d prof/fetch -o run --output-format csv -- python3 bench.py <args>
    rocprofv3 --pmc WRITE_SIZE       -d prof/write -o run --output-format csv -- python3 bench.py <args>

Writes profiles/<name>_kernel_trace.txt (per-kernel times beside bench.py's own figures of the same run),
profiles/<name>_hbm_traffic.txt (per-kernel HBM-side bytes) and the row of <name> in profiles/attend_hbm_traffic.txt,
the table bench.py reads for roofline.traffic. FETCH_SIZE / WRITE_SIZE are KiB per dispatch; each is scaled by what
the same counter reads for the plain 256 MiB device-to-device copy that bench.py issues at its end.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CAL_KIB = 262144.0     # the calibration copy reads and writes 256 MiB
TABLE = os.path.join(ROOT, "profiles", "attend_hbm_traffic.txt")
TABLE_HEADER = """# HBM-side bytes per launch of the group-attention kernel (attend_mfma_kernel), per config: rocprofv3 --pmc
# FETCH_SIZE and WRITE_SIZE (KiB per dispatch, one counter per run), averaged over the kernel's launches of the bench
# command and each scaled by the same counter's reading for a plain 256 MiB device-to-device copy. bench.py reads this
# table for roofline.traffic; rows are rewritten by `python -m paper_2505_16175_amd.profile_summary`.
# config | bytes per launch | read MB | written MB | launches | bench.py arguments of the counter runs
"""


def _one(pattern):
    hits = sorted(glob.glob(pattern, recursive=True))
    if not hits:
        raise SystemExit(f"no file matches {pattern}")
    return hits[-1]


def _short(name):
    return re.sub(r"^void ", "", name)[:90]


def kernel_times(directory):
    stats = collections.OrderedDict()
    for r in csv.DictReader(open(_one(os.path.join(directory, "**", "*kernel_trace.csv")))):
        stats.setdefault(r["Kernel_Name"], []).append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return stats


def counter(directory, name):
    per_kernel = collections.OrderedDict()
    for r in csv.DictReader(open(_one(os.path.join(directory, "**", "*counter_collection.csv")))):
        if r["Counter_Name"] == name:
            per_kernel.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return per_kernel


def calibration(fetch, write):
    """Readings of the two counters for the 256 MiB calibration copy. The run holds other plain copies (the input
    generator clones tensors of tens of MB to GB). WRITE_SIZE counts a plain copy's KiB one for one, so the
    calibration copy (and any other copy of exactly its size, which reads the same) is found there by value; the
    FETCH_SIZE run issued the same copies in the same order, so its reading is taken at the same positions."""
    wv = [x for k, v in write.items() if "copyBuffer" in k for x in v]
    fv = [x for k, v in fetch.items() if "copyBuffer" in k for x in v]
    at = [i for i, x in enumerate(wv) if abs(x - CAL_KIB) <= 0.005 * CAL_KIB]
    if not at or len(fv) != len(wv):
        raise SystemExit("the calibration copy is not in the counter output (or the two runs differ in their copies)")
    return sum(fv[i] for i in at) / len(at), sum(wv[i] for i in at) / len(at)


def main():
    csv.field_size_limit(10 ** 9)
    ap = argparse.ArgumentParser()
    ap.add_argument("--name", required=True, help="config name (row key of the traffic table, prefix of the summaries)")
    ap.add_argument("--kernel-trace")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--bench-json", help="the JSON line bench.py printed in the kernel-trace run")
    ap.add_argument("--command", default="", help="bench.py arguments of the runs")
    args = ap.parse_args()
    os.makedirs(os.path.join(ROOT, "profiles"), exist_ok=True)

    if args.kernel_trace:
        stats = kernel_times(args.kernel_trace)
        total = sum(sum(v) for v in stats.values())
        out = [f"rocprofv3 kernel-trace summary, workload {args.name}, MI355X",
               "command (from the repo root, TMPDIR=/tmp):",
               f"  rocprofv3 --kernel-trace --stats -d {args.kernel_trace} -o run --output-format csv -- python3 bench.py {args.command}"]
        if args.bench_json:
            line = [l for l in open(args.bench_json) if l.startswith('{"metric"')][-1]
            j = json.loads(line)
            rf = j["roofline"]
            out += ["bench.py's own figures in this same run:",
                    f"  ms_per_step {j['ms_per_step']:.3f}  value {j['value']:.4g} {j['unit']}  roofline.avg_launch_us "
                    f"{rf['avg_launch_us']:.1f}  achieved {rf['achieved']:.1f} TFLOP/s  frac {rf['frac']:.3f}  "
                    f"whole_step_frac {rf['whole_step_frac']:.3f}",
                    "  (roofline.avg_launch_us is taken with HIP events around the qp_group_attend calls of a serial replay. Where the",
                    "   timed steps alternate consecutive groups' attention launches over two streams (groups of under two rounds of",
                    "   workgroups: configs 2 and 3) the overlap stretches each launch's begin-to-end time in this trace and the --stats",
                    "   average below mixes both kinds of launches; where they run on one stream (configs 4 and 5) the two agree)"]
        out += ["", "kernel | calls | total ms | average us | min us | max us | % of GPU time"]
        for k, v in sorted(stats.items(), key=lambda kv: -sum(kv[1]))[:14]:
            out.append(f"{_short(k)} | {len(v)} | {sum(v) / 1e3:.3f} | {sum(v) / len(v):.2f} | {min(v):.2f} | {max(v):.2f} | "
                       f"{100 * sum(v) / total:.2f}")
        att = [v for k, v in stats.items() if "attend_mfma_kernel" in k]
        if att:
            v = sorted(att[0])
            out += ["", f"attend_mfma_kernel: {len(v)} launches, median {v[len(v) // 2]:.1f} us, average {sum(v) / len(v):.1f} us"]
        path = os.path.join(ROOT, "profiles", f"{args.name}_kernel_trace.txt")
        open(path, "w").write("\n".join(out) + "\n")
        print("wrote", path)

    if args.fetch and args.write:
        f, w = counter(args.fetch, "FETCH_SIZE"), counter(args.write, "WRITE_SIZE")
        cf, cw = calibration(f, w)
        sf, sw = CAL_KIB / cf, CAL_KIB / cw
        out = [f"rocprofv3 HBM-side counters per dispatch (KiB), workload {args.name}, MI355X",
               "commands (from the repo root, TMPDIR=/tmp), one counter per run:",
               f"  rocprofv3 --pmc FETCH_SIZE -d {args.fetch} -o run --output-format csv -- python3 bench.py {args.command}",
               f"  rocprofv3 --pmc WRITE_SIZE -d {args.write} -o run --output-format csv -- python3 bench.py {args.command}",
               "calibration: bench.py ends with one plain device-to-device copy of 256 MiB (= 262144 KiB read, 262144 KiB written):",
               f"  FETCH_SIZE of that copy  {cf:.1f} KiB  -> scale factor {sf:.3f}",
               f"  WRITE_SIZE of that copy  {cw:.1f} KiB  -> scale factor {sw:.3f}", "",
               "kernel | dispatches | FETCH_SIZE avg KiB (raw) | scaled MB read | WRITE_SIZE avg KiB (raw) | scaled MB written"]
        row = None
        for k, v in f.items():
            if "copyBuffer" in k or k not in w:
                continue
            fr, wr = sum(v) / len(v), sum(w[k]) / len(w[k])
            rd, wt = fr * sf * 1024 / 1e6, wr * sw * 1024 / 1e6
            out.append(f"{_short(k)} | {len(v)} | {fr:.1f} | {rd:.2f} | {wr:.1f} | {wt:.2f}")
            if "attend_mfma_kernel" in k:
                row = (rd, wt, len(v))
        path = os.path.join(ROOT, "profiles", f"{args.name}_hbm_traffic.txt")
        open(path, "w").write("\n".join(out) + "\n")
        print("wrote", path)
        if row is not None:
            rows = collections.OrderedDict()
            if os.path.exists(TABLE):
                for line in open(TABLE):
                    if not line.startswith("#") and "|" in line:
                        rows[line.split("|")[0].strip()] = line.rstrip("\n")
            rd, wt, n = row
            rows[args.name] = f"{args.name} | {(rd + wt) * 1e6:.0f} | {rd:.2f} | {wt:.2f} | {n} | {args.command}"
            open(TABLE, "w").write(TABLE_HEADER + "\n".join(rows.values()) + "\n")
            print("updated", TABLE)


if __name__ == "__main__":
    main()
