"""Turns rocprofv3 output into the short text summaries kept under profiles/.

    python -m paper_2503_06823_amd.profile_tools kernel-stats <dir> --command "<cmd>" --out profiles/x.md
            [--bench-json line.json] [--title "..."] [--note "..."]
    python -m paper_2503_06823_amd.profile_tools traffic <fetch_dir> <write_dir> --command "<cmd>" --out profiles/x.md
    python -m paper_2503_06823_amd.profile_tools counters <dir> [<dir> ...] --command "<cmd>" --out profiles/x.md
            [--kernels substring,substring]

<dir> is what `rocprofv3 -d <dir>` wrote (searched recursively for *_kernel_stats.csv or
*_counter_collection.csv).  `traffic` expects the profiled command to have run bench.py with
--copy-calibration: the library's copy kernel on 1 GiB in the same run give the factors by which FETCH_SIZE and
WRITE_SIZE (KiB per dispatch as the counters read them) are scaled to bytes; its summary ends in a
```json block that bench.py reads back for `roofline.traffic`.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

csv.field_size_limit(1 << 30)
CALIBRATION_BYTES = 1 << 30       # bench.py --copy-calibration copies 1 GiB device to device


def short_name(name: str) -> str:
    """Kernel name without namespaces, return type and argument list; template arguments kept."""
    name = name.replace("emoe::(anonymous namespace)::", "").replace("void ", "")
    depth, out = 0, []
    for ch in name:                      # cut at the first '(' that is not inside template brackets
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            break
        out.append(ch)
    s = "".join(out).strip()
    return s if len(s) <= 90 else s[:87] + "..."


def _find(directory: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {directory}")
    return hits[0]


def read_counters(directory: str):
    """{(short kernel name, counter): [value per dispatch]} from a counter_collection.csv."""
    agg = collections.defaultdict(list)
    with open(_find(directory, "counter_collection.csv"), newline="") as f:
        for r in csv.DictReader(f):
            agg[(short_name(r["Kernel_Name"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    return agg


def cmd_kernel_stats(a):
    rows = list(csv.DictReader(open(_find(a.dir, "kernel_stats.csv"), newline="")))
    with open(a.out, "w") as f:
        f.write(f"# {a.title or 'rocprofv3 kernel-trace summary'}\n\n")
        f.write("Command (run on the MI355X box from the repository root):\n\n```\n" + a.command + "\n```\n\n")
        f.write("Per-kernel statistics over the whole run (warm-up and timed steps):\n\n")
        f.write("| kernel | calls | total ms | average us | min us | max us | % of GPU time |\n|---|---|---|---|---|---|---|\n")
        for r in rows:
            if float(r["Percentage"]) < a.min_percent:
                continue
            f.write(f"| `{short_name(r['Name'])}` | {r['Calls']} | {int(r['TotalDurationNs']) / 1e6:.3f} | "
                    f"{float(r['AverageNs']) / 1e3:.1f} | {int(r['MinNs']) / 1e3:.1f} | {int(r['MaxNs']) / 1e3:.1f} | "
                    f"{float(r['Percentage']):.2f} |\n")
        if a.note:
            f.write("\n" + a.note + "\n")
        if a.bench_json:
            b = json.loads(open(a.bench_json).read().strip().splitlines()[-1])
            keep = {k: b[k] for k in ("value", "ms_per_step", "ms_per_step_eager", "launch", "roofline", "prefill_breakdown_ms",
                                      "breakdown_ms", "ceilings", "combine_fold_measurement", "layer_tflops",
                                      "layer_mfma_frac", "layer_weight_gbs", "layer_hbm_frac", "miss_rate") if k in b}
            for sub in ("decode", "c5", "c2"):
                if sub in b:
                    keep[sub] = {k: b[sub][k] for k in ("value", "ms_per_step", "roofline", "breakdown_ms") if k in b[sub]}
            f.write("\nThe same run's bench.py line (HIP-event times over the timed steps only), in part:\n\n```\n")
            f.write(json.dumps(keep, indent=1) + "\n```\n")
    print(a.out)


def cmd_traffic(a):
    fetch, write = read_counters(a.fetch_dir), read_counters(a.write_dir)
    def calib(agg, counter):
        v = [x for (k, c), vals in agg.items() if c == counter and k.startswith("copy_stream_kernel") for x in vals]
        if not v:
            raise SystemExit(f"no 1 GiB calibration copy found for {counter}: run bench.py with --copy-calibration")
        return (CALIBRATION_BYTES / 1024) / (sum(v) / len(v)), sum(v) / len(v), len(v)
    f_fac, f_read, f_n = calib(fetch, "FETCH_SIZE")
    w_fac, w_read, w_n = calib(write, "WRITE_SIZE")
    kernels = sorted({k for (k, c) in fetch if c == "FETCH_SIZE"})
    rows = []
    for k in kernels:
        fv, wv = fetch.get((k, "FETCH_SIZE"), []), write.get((k, "WRITE_SIZE"), [])
        if not fv or not wv:
            continue
        fk, wk = sum(fv) / len(fv), sum(wv) / len(wv)
        total = (fk * f_fac + wk * w_fac) * 1024
        if total < a.min_bytes:
            continue
        rows.append({"kernel": k, "dispatches": len(fv), "fetch_size_kib": fk, "write_size_kib": wk,
                     "hbm_bytes_per_launch": total})
    rows.sort(key=lambda r: -r["hbm_bytes_per_launch"] * r["dispatches"])
    with open(a.out, "w") as f:
        f.write(f"# {a.title or 'HBM traffic per launch (rocprofv3 hardware counters)'}\n\n")
        f.write("Two counter runs of the same command, one counter each (run on the MI355X box from the repository "
                "root), then\n`python -m paper_2503_06823_amd.profile_tools traffic <out1> <out2> ...` wrote this file:\n\n"
                "```\n" + a.command + "\n```\n\n")
        f.write("`--copy-calibration` makes bench.py run the library's plain copy kernel on 1 GiB three times before the "
                "workloads, so each run\nalso holds a kernel of known traffic:\n\n")
        f.write("| calibration kernel | known KiB | counter reads (KiB, average) | dispatches | factor (known / read) |\n|---|---|---|---|---|\n")
        f.write(f"| `copy_stream_kernel` on 1 GiB, FETCH_SIZE | 1 048 576 read | {f_read:,.1f} | {f_n} | {f_fac:.3f} |\n")
        f.write(f"| `copy_stream_kernel` on 1 GiB, WRITE_SIZE | 1 048 576 written | {w_read:,.1f} | {w_n} | {w_fac:.3f} |\n\n")
        f.write("Averages per dispatch (KiB as the counters read them) and the scaled HBM-side bytes per launch:\n\n")
        f.write("| kernel | dispatches | FETCH_SIZE | WRITE_SIZE | read + written = bytes per launch |\n|---|---|---|---|---|\n")
        for r in rows:
            rd, wr = r["fetch_size_kib"] * f_fac * 1024, r["write_size_kib"] * w_fac * 1024
            f.write(f"| `{r['kernel']}` | {r['dispatches']} | {r['fetch_size_kib']:,.0f} | {r['write_size_kib']:,.0f} | "
                    f"{rd / 1e9:.3f} GB + {wr / 1e9:.3f} GB = {r['hbm_bytes_per_launch'] / 1e9:.3f} GB |\n")
        if a.note:
            f.write("\n" + a.note + "\n")
        f.write("\nMachine-readable (bench.py reads `roofline.traffic` from here):\n\n```json\n")
        f.write(json.dumps({"fetch_factor": f_fac, "write_factor": w_fac, "kernels": rows}, indent=1) + "\n```\n")
    print(a.out)


def read_durations(directory: str):
    """{short kernel name: [dispatch duration in ns]} from the kernel_trace.csv of the same run."""
    dur = collections.defaultdict(list)
    with open(_find(directory, "kernel_trace.csv"), newline="") as f:
        for r in csv.DictReader(f):
            dur[short_name(r["Kernel_Name"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return dur


def cmd_counters(a):
    want = [s for s in (a.kernels or "").split(",") if s]
    table = collections.defaultdict(dict)     # kernel -> counter -> (mean, n)
    for d in a.dirs:
        for (k, c), v in read_counters(d).items():
            if want and not any(w in k for w in want):
                continue
            table[k][c] = (sum(v) / len(v), len(v))
        for k, v in read_durations(d).items():
            if k in table:
                table[k]["duration_us (dispatch timestamps, counters on)"] = (sum(v) / len(v) / 1e3, len(v))
    for k, t in table.items():                # derived figures of the matrix-core counter set
        if "SQ_BUSY_CU_CYCLES" in t and "SQ_VALU_MFMA_BUSY_CYCLES" in t:
            busy, mfma = t["SQ_BUSY_CU_CYCLES"][0], t["SQ_VALU_MFMA_BUSY_CYCLES"][0]
            t["matrix pipe busy = MFMA_BUSY / (4 SIMDs x BUSY_CU)"] = (mfma / (4 * busy), 0)
            dur = t.get("duration_us (dispatch timestamps, counters on)")
            if dur:
                t["sustained GHz = BUSY_CU / 256 CUs / duration"] = (busy / a.cus / (dur[0] * 1e3), 0)
        if "SQ_INSTS_VALU_MFMA_MOPS_BF16" in t:
            t["TFLOP executed = MOPS_BF16 x 512"] = (t["SQ_INSTS_VALU_MFMA_MOPS_BF16"][0] * 512 / 1e12, 0)
    counters = sorted({c for t in table.values() for c in t})
    with open(a.out, "w") as f:
        f.write(f"# {a.title or 'Hardware counters per dispatch (rocprofv3 --pmc)'}\n\n")
        f.write("Commands (one counter group per run, on the MI355X box from the repository root), then\n"
                "`python -m paper_2503_06823_amd.profile_tools counters <out dirs> ...` wrote this file:\n\n```\n" + a.command + "\n```\n\n")
        kernels = sorted(table, key=lambda k: -max(m for m, _ in table[k].values()))
        f.write("Average per dispatch (counters are sums over the chip):\n\n| counter | " + " | ".join(f"`{k}`" for k in kernels) + " |\n|---|" + "---|" * len(kernels) + "\n")
        f.write("| dispatches | " + " | ".join(str(max(n for _, n in table[k].values())) for k in kernels) + " |\n")
        for c in counters:
            f.write(f"| {c} | " + " | ".join(f"{table[k][c][0]:,.4g}" if c in table[k] else "" for k in kernels) + " |\n")
        if a.note:
            f.write("\n" + a.note + "\n")
    print(a.out)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    def common(p):
        p.add_argument("--command", required=True, help="the full profiled command, as it was run")
        p.add_argument("--out", required=True)
        p.add_argument("--title", default="")
        p.add_argument("--note", default="", help="free text appended to the summary (the reading of the figures)")
    p = sub.add_parser("kernel-stats"); p.add_argument("dir"); common(p)
    p.add_argument("--bench-json", default=""); p.add_argument("--min-percent", type=float, default=0.0)
    p.set_defaults(fn=cmd_kernel_stats)
    p = sub.add_parser("traffic"); p.add_argument("fetch_dir"); p.add_argument("write_dir"); common(p)
    p.add_argument("--min-bytes", type=float, default=16e6)
    p.set_defaults(fn=cmd_traffic)
    p = sub.add_parser("counters"); p.add_argument("dirs", nargs="+"); common(p); p.add_argument("--kernels", default="")
    p.add_argument("--cus", type=int, default=256, help="compute units the per-chip cycle counters are divided by")
    p.set_defaults(fn=cmd_counters)
    a = ap.parse_args(argv)
    a.fn(a)


if __name__ == "__main__":
    main()
