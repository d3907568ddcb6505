"""Turn rocprofv3 CSV output of ``bench.py`` into the short text summary kept under ``profiles/``.

Inputs are the files rocprofv3 writes with ``--output-format csv``:
  * ``--kernel-trace --stats``  ->  ``*_kernel_stats.csv`` and ``*_kernel_trace.csv``
  * ``--pmc FETCH_SIZE``        ->  ``*_counter_collection.csv``   (its own run)
  * ``--pmc WRITE_SIZE``        ->  ``*_counter_collection.csv``   (its own run)
  * optionally one more ``--pmc`` run (``--pmc-dir``) whose counters are tabulated as they are

FETCH_SIZE / WRITE_SIZE do not read in KiB on this chip, so both are scaled by what they read for
a streaming kernel whose traffic is known exactly: the quantiser that bench.py runs once per
shape reads 4 bytes and writes 0.53125 bytes per weight, and its grid size is weights / 8.

Usage:
  python -m paper_2602_02711_amd.rocprof_summary --trace-dir D1 --fetch-dir D2 --write-dir D3 \
      --command "..." --out-md profiles/x.md --out-json profiles/x.json
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os

def _one(directory, pattern):
    hits = glob.glob(os.path.join(directory, "**", pattern), recursive=True)
    if not hits:
        raise FileNotFoundError(f"no {pattern} under {directory}")
    return hits[0]


def short(name: str) -> str:
    if name.startswith("void "):
        name = name[5:]
    name = name.replace("dmr::(anonymous namespace)::", "").replace("dmr::", "")
    return name.split("(")[0]


def trace_stats(trace_dir):
    """Per (kernel, grid, workgroup): calls, mean / min / max duration in microseconds."""
    rows = collections.defaultdict(list)
    with open(_one(trace_dir, "*_kernel_trace.csv")) as fh:
        for r in csv.DictReader(fh):
            key = (short(r["Kernel_Name"]), int(r["Grid_Size_X"]), int(r["Workgroup_Size_X"]))
            rows[key].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    return {k: (len(v), sum(v) / len(v), min(v), max(v)) for k, v in rows.items()}


def trace_gaps(trace_dir, max_gap_us=20.0):
    """End-to-start gaps between consecutive kernels of the trace (sorted by start time), keyed by the pair
    (previous kernel, next kernel): count, median and mean gap, and the median start-to-start period, in
    microseconds.  Gaps above `max_gap_us` (host-side pauses between graph replays, set-up work) are left out."""
    rows = []
    with open(_one(trace_dir, "*_kernel_trace.csv")) as fh:
        for r in csv.DictReader(fh):
            rows.append((int(r["Start_Timestamp"]), int(r["End_Timestamp"]),
                         f'{short(r["Kernel_Name"])} [{int(r["Grid_Size_X"]) // max(int(r["Workgroup_Size_X"]), 1)} wg]'))
    rows.sort()
    pairs = collections.defaultdict(list)
    for (s0, e0, n0), (s1, e1, n1) in zip(rows, rows[1:]):
        gap = (s1 - e0) / 1e3
        if gap <= max_gap_us:
            pairs[(n0, n1)].append((gap, (s1 - s0) / 1e3, (e0 - s0) / 1e3))
    out = {}
    for key, v in pairs.items():
        gaps = sorted(g for g, _, _ in v)
        periods = sorted(p for _, p, _ in v)
        durs = sorted(d for _, _, d in v)
        out[key] = (len(v), gaps[len(gaps) // 2], sum(gaps) / len(gaps), periods[len(periods) // 2], durs[len(durs) // 2])
    return out


def counter_means(pmc_dir, counter):
    rows = collections.defaultdict(list)
    with open(_one(pmc_dir, "*_counter_collection.csv")) as fh:
        for r in csv.DictReader(fh):
            if r["Counter_Name"] != counter:
                continue
            key = (short(r["Kernel_Name"]), int(r["Grid_Size"]), int(r["Workgroup_Size"]))
            rows[key].append(float(r["Counter_Value"]))
    return {k: (len(v), sum(v) / len(v)) for k, v in rows.items()}


def calibration(means, bytes_per_weight):
    """Scale = known KiB / counter reading, from the quantiser dispatches (grid = weights / 8)."""
    num = den = 0.0
    for (name, grid, _), (n, mean) in means.items():
        if name == "quantize_kernel":
            num += n * grid * 8 * bytes_per_weight / 1024.0
            den += n * mean
    if den == 0:
        raise RuntimeError("no quantize_kernel dispatch to calibrate against")
    return num / den


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--trace-dir", required=True)
    ap.add_argument("--fetch-dir")
    ap.add_argument("--write-dir")
    ap.add_argument("--pmc-dir", help="a further --pmc run whose counters are tabulated as they are")
    ap.add_argument("--command", required=True, help="the full profiled command, for the record")
    ap.add_argument("--kernel", default="w4_gemv_kernel", help="substring naming the dominant kernel")
    ap.add_argument("--title", default="decode GEMV sweep (bench.py)", help="what was profiled, for the heading")
    ap.add_argument("--note", default="", help="where and when the counters were taken, stored as `source` in the json")
    ap.add_argument("--gaps", action="store_true", help="add the end-to-start gaps between consecutive kernels")
    ap.add_argument("--out-md", required=True)
    ap.add_argument("--out-json")
    args = ap.parse_args()

    stats = trace_stats(args.trace_dir)
    lines = [f"# rocprofv3 summary: {args.title}, MI355X", "",
             "Commands (each its own run, from /tmp with TMPDIR=/tmp):", "", "```", args.command, "```", "",
             "## Kernel durations (--kernel-trace), microseconds", "",
             "| kernel | grid | wg | calls | mean | min | max |", "|---|---|---|---|---|---|---|"]
    dom_calls = dom_total = 0.0
    for (name, grid, wg), (n, mean, lo, hi) in sorted(stats.items(), key=lambda kv: -kv[1][0] * kv[1][1]):
        if any(tag in name for tag in ("gemv", "skinny", "gemm", "mid_kernel", "stream", "panel", "wide", "splitk",
                                       "rmsnorm", "swiglu", "residual", "xfrag")):
            lines.append(f"| {name} | {grid} | {wg} | {n} | {mean:.2f} | {lo:.2f} | {hi:.2f} |")
        if args.kernel in name:
            dom_calls += n
            dom_total += n * mean
    dom_mean = dom_total / dom_calls if dom_calls else float("nan")
    lines += ["", f"Dominant kernel `{args.kernel}` (all instantiations, all shapes): {int(dom_calls)} launches, "
                  f"mean {dom_mean:.3f} us per launch.", ""]

    out = {"kernel": args.kernel, "mean_launch_us": dom_mean, "launches": int(dom_calls)}
    if args.gaps:
        lines += ["## End-to-start gaps between consecutive kernels (--kernel-trace timestamps), microseconds", "",
                  "Gap = start of the next kernel minus end of the previous one; period = start to start.  Pairs with "
                  "at least 50 occurrences; pauses above 20 us (between graph replays) left out.", "",
                  "| previous kernel | next kernel | pairs | median gap | mean gap | median duration of previous | median period |",
                  "|---|---|---|---|---|---|---|"]
        for (n0, n1), (n, med, mean, period, dur) in sorted(trace_gaps(args.trace_dir).items(), key=lambda kv: -kv[1][0]):
            if n >= 50:
                lines.append(f"| {n0} | {n1} | {n} | {med:.2f} | {mean:.2f} | {dur:.2f} | {period:.2f} |")
        lines.append("")
    if args.fetch_dir and args.write_dir:
        fetch = counter_means(args.fetch_dir, "FETCH_SIZE")
        write = counter_means(args.write_dir, "WRITE_SIZE")
        sf = calibration(fetch, 4.0)
        sw = calibration(write, 0.53125)
        lines += ["## HBM traffic (--pmc FETCH_SIZE, --pmc WRITE_SIZE), scaled", "",
                  f"Scale factors from the quantiser (reads 4 B, writes 0.53125 B per weight): "
                  f"FETCH_SIZE x {sf:.4f}, WRITE_SIZE x {sw:.4f} give KiB.", "",
                  "| kernel | grid | wg | launches | fetched MB | written MB |", "|---|---|---|---|---|---|"]
        tot_f = tot_w = tot_n = 0.0
        for key, (n, mean) in sorted(fetch.items()):
            name, grid, wg = key
            if "gemv" not in name and "skinny" not in name:
                continue
            w_mean = write.get(key, (0, 0.0))[1]
            fb, wb = mean * sf * 1024, w_mean * sw * 1024
            lines.append(f"| {name} | {grid} | {wg} | {n} | {fb / 1e6:.3f} | {wb / 1e6:.4f} |")
            if args.kernel in name:
                tot_f += n * fb
                tot_w += n * wb
                tot_n += n
        if tot_n:
            if args.note:
                out["source"] = args.note
            out.update({"fetch_bytes_per_launch": tot_f / tot_n, "write_bytes_per_launch": tot_w / tot_n,
                        "traffic": (tot_f + tot_w) / tot_n, "scale_fetch": sf, "scale_write": sw})
            lines += ["", f"`{args.kernel}`: {tot_f / tot_n / 1e6:.3f} MB fetched + {tot_w / tot_n / 1e6:.4f} MB "
                          f"written per launch on average (algorithmic: 29.002 MB per launch over the four shapes).", ""]
    if args.pmc_dir:
        # any other counters of one --pmc run: mean per launch of every counter, per kernel of interest
        table = collections.defaultdict(lambda: collections.defaultdict(list))
        with open(_one(args.pmc_dir, "*_counter_collection.csv")) as fh:
            for r in csv.DictReader(fh):
                key = (short(r["Kernel_Name"]), int(r["Grid_Size"]), int(r["Workgroup_Size"]))
                table[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
        names = sorted({c for cs in table.values() for c in cs})
        lines += ["## Counters (--pmc " + " ".join(names) + "), mean per launch", "",
                  "| kernel | grid | wg | launches | " + " | ".join(names) + " |", "|---|---|---|---|" + "---|" * len(names)]
        for key, cs in sorted(table.items()):
            name, grid, wg = key
            if args.kernel not in name:
                continue
            n = max(len(v) for v in cs.values())
            cells = [f"{sum(cs[c]) / len(cs[c]):.4g}" if c in cs else "" for c in names]
            lines.append(f"| {name} | {grid} | {wg} | {n} | " + " | ".join(cells) + " |")
        lines.append("")
    with open(args.out_md, "w") as fh:
        fh.write("\n".join(lines) + "\n")
    if args.out_json:
        with open(args.out_json, "w") as fh:
            json.dump(out, fh, indent=1)
            fh.write("\n")
    print("\n".join(lines))


if __name__ == "__main__":
    main()
