"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2404_19124_amd.profile_summary trace  <dir> --command "<cmd>" --out profiles/<name>.txt
    python -m paper_2404_19124_amd.profile_summary traffic --workload W --label L --match SUBSTR
           --fetch <dir> --write <dir> --fetch-cal <dir> --write-cal <dir> --command "<cmd>" --out profiles/<name>.txt

`trace` reads `*_kernel_trace.csv` of a `rocprofv3 --kernel-trace --stats --output-format csv`
run: per-kernel calls / total / average, and the timeline of the last step.

`traffic` reads `*_counter_collection.csv` of four `rocprofv3 --pmc` runs: FETCH_SIZE
and WRITE_SIZE (KiB per dispatch) of the benchmark, and the same two counters of
`bench.py --copy-probe`, whose launch moves a known number of bytes.  The factor
known / counted of the copy scales the benchmark's reading; the per-launch HBM
bytes of the kernels whose name contains SUBSTR are appended to
profiles/hbm_traffic.json under [workload][label], where bench.py looks them up.

Reads files only; runs nothing on the GPU.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _one(dirname: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(dirname, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, dirname))
    return hits[-1]


def _short(name: str) -> str:
    name = name.replace("specdraft::", "").replace("void ", "")
    cut = name.find("(")
    return (name if cut < 0 else name[:cut])[:64]


def cmd_trace(a) -> int:
    rows = list(csv.DictReader(open(_one(a.dir, "kernel_trace.csv"))))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    agg = collections.OrderedDict()
    total = 0.0
    for r in rows:
        us = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        d = agg.setdefault(_short(r["Kernel_Name"]), [0, 0.0, 1e30, 0.0])
        d[0] += 1
        d[1] += us
        d[2] = min(d[2], us)
        d[3] = max(d[3], us)
        total += us
    lines = ["# rocprofv3 --kernel-trace --stats summary (durations in microseconds)", "# command: " + a.command, "",
             "%-64s %7s %12s %9s %9s %9s %6s" % ("kernel", "calls", "total_us", "avg_us", "min_us", "max_us", "pct")]
    for name, (n, t, lo, hi) in sorted(agg.items(), key=lambda kv: -kv[1][1])[:a.top]:
        lines.append("%-64s %7d %12.1f %9.2f %9.2f %9.2f %6.2f" % (name, n, t, t / n, lo, hi, 100.0 * t / total))
    ends = [i for i, r in enumerate(rows) if a.step_end in r["Kernel_Name"]]
    if len(ends) >= 2:
        lo, hi = ends[-2], ends[-1]
        lines += ["", "# timeline of the last step (gap = idle time before the kernel, under the profiler)"]
        prev = int(rows[lo]["End_Timestamp"])
        for r in rows[lo + 1:hi + 1]:
            s, e = int(r["Start_Timestamp"]), int(r["End_Timestamp"])
            lines.append("%-64s grid %8s  dur %8.2f  gap %6.2f" % (_short(r["Kernel_Name"]), r.get("Grid_Size_X", "?"),
                                                                 (e - s) / 1e3, (s - prev) / 1e3))
            prev = e
        lines.append("# sum of kernel durations of that step: %.2f us" % sum(
            (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3 for r in rows[lo + 1:hi + 1]))
    text = "\n".join(lines) + "\n"
    open(a.out, "w").write(text)
    sys.stdout.write(text)
    return 0


def _counter(dirname: str, counter: str, match: str):
    """(mean counter value per dispatch, dispatches) over kernels whose name contains `match`."""
    vals = []
    for r in csv.DictReader(open(_one(dirname, "counter_collection.csv"))):
        if r["Counter_Name"] == counter and match in r["Kernel_Name"]:
            vals.append(float(r["Counter_Value"]))
    if not vals:
        raise SystemExit("no %s rows for kernels matching %r in %s" % (counter, match, dirname))
    return sum(vals) / len(vals), len(vals)


def cmd_traffic(a) -> int:
    kib = 1024.0
    f_cal, nfc = _counter(a.fetch_cal, "FETCH_SIZE", "copy_probe_kernel")
    w_cal, nwc = _counter(a.write_cal, "WRITE_SIZE", "copy_probe_kernel")
    k_fetch = a.cal_bytes / (f_cal * kib)
    k_write = a.cal_bytes / (w_cal * kib)
    f, nf = _counter(a.fetch, "FETCH_SIZE", a.match)
    w, nw = _counter(a.write, "WRITE_SIZE", a.match)
    fetch_b, write_b = f * kib * k_fetch, w * kib * k_write
    total = fetch_b + write_b
    lines = [
        "# HBM traffic per launch from rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE, KiB per dispatch)",
        "# commands: " + a.command,
        "workload %s, kernels matching %r (%d / %d dispatches averaged)" % (a.workload, a.match, nf, nw),
        "copy probe: %d bytes read and written per launch; FETCH_SIZE %.1f KiB (%d launches), WRITE_SIZE %.1f KiB (%d)"
        % (a.cal_bytes, f_cal, nfc, w_cal, nwc),
        "scale factors known/counted: fetch %.4f, write %.4f" % (k_fetch, k_write),
        "FETCH_SIZE %.1f KiB -> %.0f bytes read per launch" % (f, fetch_b),
        "WRITE_SIZE %.1f KiB -> %.0f bytes written per launch" % (w, write_b),
        "traffic %.0f bytes per launch" % total,
    ]
    if a.algorithmic_bytes:
        lines.append("algorithmic bytes per launch %.0f -> traffic / algorithmic = %.3f"
                     % (a.algorithmic_bytes, total / a.algorithmic_bytes))
    text = "\n".join(lines) + "\n"
    open(a.out, "w").write(text)
    sys.stdout.write(text)
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        table = json.load(open(path))
    except (OSError, ValueError):
        table = {}
    table.setdefault(a.workload, {})[a.label] = round(total)
    json.dump(table, open(path, "w"), indent=1, sort_keys=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("dir")
    t.add_argument("--command", required=True)
    t.add_argument("--out", required=True)
    t.add_argument("--top", type=int, default=14)
    t.add_argument("--step-end", default="accept_kernel", help="kernel that ends a step")
    t.set_defaults(fn=cmd_trace)
    h = sub.add_parser("traffic")
    for name in ("fetch", "write", "fetch-cal", "write-cal", "workload", "label", "match", "command", "out"):
        h.add_argument("--" + name, required=True)
    h.add_argument("--cal-bytes", type=int, required=True)
    h.add_argument("--algorithmic-bytes", type=float, default=0.0)
    h.set_defaults(fn=cmd_traffic)
    a = ap.parse_args()
    return a.fn(a)


if __name__ == "__main__":
    sys.exit(main())
