"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept under profiles/ and into
profiles/dominant_kernel_traffic.json, the file from which bench.py takes `roofline.traffic`.

Usage (from the repository root, after the rocprofv3 runs named in the summary's header):

  python3 -m paper_2412_20386_amd.profile_summary --kernel-trace out/prof/kt --fetch out/prof/fetch \
      --write out/prof/write --bench-json out/prof/bench_kt.json --config 3 \
      --dominant linear_mfma_wreg --out profiles/bench_vim_b_stack_kernel_trace_and_traffic.txt

Every input is optional; what is missing is left out of the summary.  HBM traffic of a kernel = the counter's
median over its dispatches (KiB) times the factor that makes the same counter read 262144 KiB for the 256 MiB
device-to-device copy that bench.py issues in the same run.
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import json
import os
import re
import statistics
import sys

OURS = ("linear_", "pts_linear", "quantize_", "fold_smoothing", "weight_rowsum", "count_bad_scales", "sum_bad_scales")
BASES = ("linear_e2m3_persistent", "linear_e2m3_generic", "quantize_pts_a4_e2m3_blocks", "quantize_pts_a4_e2m3_stream",
         "quantize_pts_a4_e2m3_generic", "fold_smoothing_w4_e2m3_rows", "linear_mfma_wreg", "linear_mfma_persistent", "linear_mfma_smallk", "linear_mfma_dma", "linear_mfma_generic",
         "linear_mfma_wres", "linear_stream_smallk", "pts_linear_wres", "pts_linear_generic", "quantize_pts_a4_stream",
         "quantize_pts_stream", "quantize_pts_generic", "quantize_dynamic_rows", "fold_smoothing_w4_rows",
         "fold_smoothing_rows", "weight_rowsum_rows", "count_bad_scales", "sum_bad_scales")
COPY_KIB = 262144.0  # bench.py's calibration copy


def short(name: str) -> str:
    base = next((b for b in BASES if b in name), None)
    if base is None:
        return name[:40]
    tag = ""
    for t, label in (("Int8OffsetPath", "<int8+offset>"), ("Int4Path", "<int4>"), ("Int8Path", "<int8>"),
                     ("Half16Path", "<fp16>")):
        if t in name:
            tag = label
            break
    def flags(mangled, demangled):  # boolean template arguments, in order
        m = re.search(mangled, name)
        if m:
            return [g == "1" for g in m.groups()]
        m = re.search(demangled, name)
        return [g == "true" for g in m.groups()] if m else None
    if base == "linear_stream_smallk":  # <k-steps, fused quantizer, two alignments, packed 4-bit operands, zero offset>
        f = flags(r"smallkILi\d+ELb([01])ELi\d+ELi\d+ELb([01])ELb([01])E",
                  r"smallk<\d+, (true|false), \d+, \d+, (true|false), (true|false)>") or [False, False, False]
        fused, packed, offset = f
        tag = "<" + ("fused " if fused else "") + ("int4" if packed else ("int8+offset" if offset else "int8")) + ">"
        if tag == "<fused int8>":
            tag = "<fused>"
    if base == "pts_linear_wres":  # <channel blocks, depth, parity aids, 4-bit, zero offset>
        f = flags(r"wresILi\d+ELi\d+ELb[01]ELb([01])ELb([01])E", r"wres<\d+, \d+, (?:true|false), (true|false), (true|false)>") or [False, False]
        tag = "<int4>" if f[0] else ("<int8+offset>" if f[1] else "")
    if base == "linear_mfma_wreg":
        tag = "<K=768>" if ("ILi12E" in name or "<12," in name) else "<K=384>"
    return base + tag


def first(pattern: str):
    hits = sorted(glob.glob(pattern))
    return hits[0] if hits else None


def split_bimodal(values):
    """Two problem shapes on one grid: split where the durations span more than 1.5x."""
    if len(values) > 8 and max(values) > 1.5 * min(values):
        cut = (max(values) * min(values)) ** 0.5
        return [(" [short]", [v for v in values if v < cut]), (" [long]", [v for v in values if v >= cut])]
    return [("", values)]


def kernel_trace_lines(directory: str, out: list) -> None:
    kt = first(os.path.join(directory, "**", "*kernel_trace.csv")) or first(os.path.join(directory, "*kernel_trace.csv"))
    if kt:
        groups = collections.defaultdict(list)
        for r in csv.DictReader(open(kt)):
            if any(k in r["Kernel_Name"] for k in OURS):
                dur = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
                groups[(short(r["Kernel_Name"]), r["Grid_Size_X"], r["LDS_Block_Size"])].append(dur)
        out.append("per-dispatch kernel durations from rocprofv3 --kernel-trace (us), grouped by kernel / grid size / LDS bytes;")
        out.append("a group whose durations span more than 1.5x is split at the geometric mean of its extremes (two problem shapes on one grid):")
        for tag, d in sorted(groups.items()):
            for suffix, dd in split_bimodal(d):
                if dd:
                    label = f"{tag[0]}{suffix} grid {tag[1]} lds {tag[2]}"
                    out.append(f"  {label:70s} calls {len(dd):5d}  avg {statistics.mean(dd):8.2f}  median "
                               f"{statistics.median(dd):8.2f}  min {min(dd):8.2f}  max {max(dd):8.2f}")
    ks = first(os.path.join(directory, "**", "*kernel_stats.csv")) or first(os.path.join(directory, "*kernel_stats.csv"))
    if ks:
        out.append("rocprofv3 --stats (kernel_stats.csv), this library's kernels:")
        for r in csv.DictReader(open(ks)):
            if any(k in r["Name"] for k in OURS):
                out.append(f"  {short(r['Name']):40s} calls {r['Calls']:>6s} avg_ns {float(r['AverageNs']):12.1f} "
                           f"min_ns {r['MinNs']:>10s} max_ns {r['MaxNs']:>10s} pct {r['Percentage']}")


def counter_groups(directory: str):
    f = first(os.path.join(directory, "**", "*counter_collection.csv")) or first(os.path.join(directory, "*counter_collection.csv"))
    agg = collections.defaultdict(list)
    if f:
        per_dispatch = collections.defaultdict(float)
        meta = {}
        for r in csv.DictReader(open(f)):
            key = (r["Dispatch_Id"], r["Counter_Name"])
            per_dispatch[key] += float(r["Counter_Value"])
            meta[key] = (short(r["Kernel_Name"]) if any(k in r["Kernel_Name"] for k in OURS) else r["Kernel_Name"][:40],
                         r["Grid_Size"], r["LDS_Block_Size"], r["Counter_Name"])
        for key, v in per_dispatch.items():
            agg[meta[key]].append(v)
    return agg


def counter_lines(name: str, agg, out: list):
    out.append(f"rocprofv3 --pmc {name} (KiB per dispatch), grouped by kernel / grid / LDS:")
    copy_reading = None
    for k, v in sorted(agg.items()):
        ours = any(o in k[0] for o in OURS)
        if "copyBuffer" in k[0]:
            if max(v) < 1000:
                continue
            copy_reading = max(v)
        elif not ours:
            continue
        for suffix, vv in split_bimodal(v):
            if vv:
                out.append(f"  {k[0] + suffix:45s} grid {k[1]:>9s} lds {k[2]:>7s} {k[3]}: n {len(vv):4d} median "
                           f"{statistics.median(vv):14.1f} min {min(vv):14.1f} max {max(vv):14.1f}")
    return copy_reading


def dominant_median(agg, substr: str):
    """Median counter reading over the dispatches of the dominant kernel (its long cluster, if it has two)."""
    values = [x for k, v in agg.items() if substr in k[0] for x in v]
    if not values:
        return None
    parts = split_bimodal(values)
    return statistics.median(parts[-1][1])


def counter_table(directories, kernels, out: list) -> None:
    """Per kernel (short name) the median over dispatches of every counter found in the given
    rocprofv3 --pmc output directories (values of one dispatch are summed over its rows: one per XCD / SE)."""
    for directory in directories:
        f = first(os.path.join(directory, "**", "*counter_collection.csv")) or first(os.path.join(directory, "*counter_collection.csv"))
        if not f:
            continue
        per_dispatch = collections.defaultdict(lambda: collections.defaultdict(float))
        names = {}
        for r in csv.DictReader(open(f)):
            if any(k in r["Kernel_Name"] for k in OURS):
                per_dispatch[r["Dispatch_Id"]][r["Counter_Name"]] += float(r["Counter_Value"])
                names[r["Dispatch_Id"]] = short(r["Kernel_Name"])
        out.append(f"counters of {directory} (median per dispatch, summed over the device):")
        for want in kernels:
            rows = [c for d, c in per_dispatch.items() if want == names[d]]
            if not rows:
                continue
            # a kernel used for two problem shapes: keep the cluster with the larger first counter
            key = sorted(rows[0])[0]
            vals = [r[key] for r in rows]
            if len(vals) > 8 and max(vals) > 1.5 * min(vals):
                cut = (max(vals) * min(vals)) ** 0.5
                rows = [r for r in rows if r[key] >= cut]
            out.append(f"  {want}: {len(rows)} dispatches")
            for k in sorted(rows[0]):
                out.append(f"     {k:34s} {statistics.median(r[k] for r in rows):18.0f}")


def main() -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--kernel-trace", help="output directory of the rocprofv3 --kernel-trace --stats run")
    ap.add_argument("--fetch", help="output directory of the rocprofv3 --pmc FETCH_SIZE run")
    ap.add_argument("--write", help="output directory of the rocprofv3 --pmc WRITE_SIZE run")
    ap.add_argument("--bench-json", help="stdout of bench.py under the kernel-trace run")
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--dominant", default="linear_mfma_wreg<K=768>", help="short name (substring) of the dominant kernel")
    ap.add_argument("--counters", nargs="*", default=[], help="output directories of further rocprofv3 --pmc runs (SQ_* ...)")
    ap.add_argument("--kernels", default="linear_mfma_wreg<K=768>,linear_mfma_persistent<int8>,pts_linear_wres,linear_stream_smallk<fused>,quantize_pts_stream",
                    help="comma-separated short-name substrings for the --counters table")
    ap.add_argument("--header", help="text file whose content is put in front of the summary (workload, commands)")
    ap.add_argument("--out", help="summary text file to write (default: stdout only)")
    ap.add_argument("--traffic-json", default=os.path.join("profiles", "dominant_kernel_traffic.json"))
    args = ap.parse_args()

    out = []
    if args.header:
        out.append(open(args.header).read().rstrip("\n"))
    if args.bench_json:
        line = open(args.bench_json).read().strip().splitlines()[-1]
        bj = json.loads(line)
        out.append(f"bench.py under the profiler: ms_per_step {bj['ms_per_step']}, roofline {bj['roofline']}")
    if args.kernel_trace:
        kernel_trace_lines(args.kernel_trace, out)
    if args.counters:
        counter_table(args.counters, [k for k in args.kernels.split(",") if k], out)
    traffic = {}
    for name, directory in (("FETCH_SIZE", args.fetch), ("WRITE_SIZE", args.write)):
        if not directory:
            continue
        agg = counter_groups(directory)
        copy_reading = counter_lines(name, agg, out)
        dom = dominant_median(agg, args.dominant)
        if copy_reading and dom is not None:
            factor = COPY_KIB / copy_reading
            traffic[name] = dict(median_kib=dom, copy_reading_kib=copy_reading, factor=round(factor, 4),
                                 bytes=dom * factor * 1024.0)
            out.append(f"  -> {args.dominant}: median {dom:.1f} KiB x factor {factor:.3f} (the 256 MiB copy reads "
                       f"{copy_reading:.1f} KiB) = {dom * factor * 1024.0 / 1e6:.1f} MB per launch")
    if "FETCH_SIZE" in traffic and "WRITE_SIZE" in traffic:
        rec = dict(config=args.config, kernel=args.dominant, fetch_bytes=round(traffic["FETCH_SIZE"]["bytes"]),
                   write_bytes=round(traffic["WRITE_SIZE"]["bytes"]),
                   traffic_bytes=round(traffic["FETCH_SIZE"]["bytes"] + traffic["WRITE_SIZE"]["bytes"]),
                   fetch_factor=traffic["FETCH_SIZE"]["factor"], write_factor=traffic["WRITE_SIZE"]["factor"],
                   source="rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py, medians over the kernel's dispatches, "
                          "scaled by the 256 MiB copy of the same run")
        with open(args.traffic_json, "w") as f:
            json.dump(rec, f, indent=1)
            f.write("\n")
        out.append(f"wrote {args.traffic_json}: {rec['traffic_bytes'] / 1e6:.1f} MB per launch")
    text = "\n".join(out) + "\n"
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    sys.stdout.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
