"""Condenses rocprofv3 CSV output of a run of this library into a short text summary and a
per-kernel HBM-traffic table.

Usage (after three runs of the same command, e.g. `python3 bench.py --single --no-cpu-baseline`):

    rocprofv3 --kernel-trace --stats --output-format csv -d OUT/trace -o t -- python3 bench.py ...
    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d OUT/fetch -o p -- python3 bench.py ...
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d OUT/write -o p -- python3 bench.py ...
    python3 rocprof_summary.py OUT --txt summary.txt --json traffic.json [--extra DIR ...]

    (optional) rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES --kernel-trace ... -d OUT/mfma ...  and  --extra OUT/mfma

With both MFMA counters in an --extra directory the summary derives, per kernel,
mfma_busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES): the share of the busy compute units' SIMD
cycles (4 SIMDs per CU) in which the matrix pipe was working.

FETCH_SIZE / WRITE_SIZE are scaled by what the same counters read for the library's own 1 GiB
`calibration_copy_kernel` (which every bench.py run launches first): factor = 2^20 KiB / reading.
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

CALIB_KIB = float(1 << 20)  # the calibration copy reads 1 GiB and writes 1 GiB


def short_name(full: str) -> str:
    """'void heta::agg_wave_kernel<float, 4, 32, 1>(heta::AggParams)' -> 'agg_wave_kernel<float, 4, 32, 1>'"""
    n = full.replace("(anonymous namespace)::", "")
    n = n.split("(")[0].replace("void ", "").replace("heta::", "").strip()
    return n


def family(name: str) -> str:
    """Kernel family as the library's own profiler names it."""
    base = name.split("<")[0]
    if base in ("gemm_kernel", "gemm_direct_kernel"):
        args = [a.strip() for a in name[name.index("<") + 1:name.rindex(">")].split(",")]
        ct = "f32" if args[0] == "float" else "bf16"
        if base == "gemm_direct_kernel" and args[1] == "float" and args[4] == "float":
            ct = "f32"  # fp32 operands on the bf16 MFMA as six terms per product: the library times it as an fp32 projection
        # both operands r-contiguous = the weight gradient (contraction over graph rows)
        wgrad = (args[2] == "true" and args[4] == "true") if base == "gemm_kernel" else (args[2] == "true" and args[5] == "true")
        return f"gemm_wgrad_{ct}" if wgrad else f"gemm_{ct}"
    if base.endswith("_multi_kernel"):  # several relations per launch: timed under the single-relation kernel's name
        base = base[:-len("_multi_kernel")] + "_kernel"
    if base == "agg_wave_split_kernel":  # the long rows of a small launch, four wavefronts per row
        return "agg_wave_kernel"
    if base == "agg_pair_kernel":  # both row classes of a small launch in one grid: timed as its short-row part
        return "agg_batch_kernel"
    return base


def read_counter(dirname: str):
    """{counter: {kernel: [n, sum]}} from every *counter_collection.csv below dirname."""
    agg = collections.defaultdict(lambda: collections.defaultdict(lambda: [0, 0.0]))
    for f in glob.glob(os.path.join(dirname, "**", "*counter_collection.csv"), recursive=True):
        with open(f) as fh:
            for r in csv.DictReader(fh):
                a = agg[r["Counter_Name"]][short_name(r["Kernel_Name"])]
                a[0] += 1
                a[1] += float(r["Counter_Value"])
    return agg


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("out", help="directory holding trace/, fetch/, write/ (any of them may be missing)")
    ap.add_argument("--extra", nargs="*", default=[], help="more counter-run directories to list")
    ap.add_argument("--txt")
    ap.add_argument("--json")
    ap.add_argument("--command", default="", help="the profiled command, recorded in the summary")
    args = ap.parse_args()
    lines = []
    if args.command:
        lines.append(f"command: {args.command}")
    durations = {}
    for f in glob.glob(os.path.join(args.out, "trace", "**", "*kernel_stats.csv"), recursive=True):
        lines.append("")
        lines.append("kernel-trace --stats (durations over the whole run, incl. warm-up):")
        lines.append(f"{'kernel':100s} {'calls':>6s} {'total_ms':>10s} {'avg_us':>10s} {'pct':>6s}")
        with open(f) as fh:
            for r in list(csv.DictReader(fh))[:16]:
                n = short_name(r["Name"])
                durations[n] = float(r["AverageNs"]) / 1e3
                lines.append(f"{n[:100]:100s} {r['Calls']:>6s} {float(r['TotalDurationNs']) / 1e6:10.3f} "
                             f"{float(r['AverageNs']) / 1e3:10.1f} {float(r['Percentage']):6.2f}")
    fetch = read_counter(os.path.join(args.out, "fetch")).get("FETCH_SIZE", {})
    write = read_counter(os.path.join(args.out, "write")).get("WRITE_SIZE", {})
    traffic = {}
    if fetch and write:
        cf = fetch.get("calibration_copy_kernel")
        cw = write.get("calibration_copy_kernel")
        if not cf or not cw or cf[1] <= 0 or cw[1] <= 0:
            print("no calibration_copy_kernel in the counter runs", file=sys.stderr)
            return 1
        f_fetch = CALIB_KIB / (cf[1] / cf[0])
        f_write = CALIB_KIB / (cw[1] / cw[0])
        lines.append("")
        lines.append(f"HBM traffic per launch (KiB counters x calibration factor: FETCH_SIZE x {f_fetch:.3f}, "
                     f"WRITE_SIZE x {f_write:.3f}; factors from the 1 GiB calibration copy):")
        lines.append(f"{'kernel':100s} {'launches':>8s} {'read_MB':>10s} {'write_MB':>10s} {'GB/s':>8s}")
        fam = collections.defaultdict(lambda: [0, 0.0])
        for k in sorted(set(fetch) | set(write), key=lambda k: -(fetch.get(k, [0, 0])[1])):
            if k.startswith("at::") or "rocclr" in k:
                continue
            nf, sf = fetch.get(k, [0, 0.0])
            nw, sw = write.get(k, [0, 0.0])
            n = max(nf, nw)
            rd = sf / max(nf, 1) * f_fetch * 1024.0
            wr = sw / max(nw, 1) * f_write * 1024.0
            rate = (rd + wr) / (durations[k] * 1e-6) / 1e9 if k in durations else float("nan")
            lines.append(f"{k[:100]:100s} {n:8d} {rd / 1e6:10.1f} {wr / 1e6:10.1f} {rate:8.0f}")
            a = fam[family(k)]
            a[0] += n
            a[1] += (rd + wr) * n
        traffic = {k: {"launches": n, "hbm_bytes_per_launch": tot / n} for k, (n, tot) in fam.items() if n}
    for d in args.extra:
        counters = read_counter(d)
        busy, cu = counters.get("SQ_VALU_MFMA_BUSY_CYCLES"), counters.get("SQ_BUSY_CU_CYCLES")
        if busy and cu:
            lines.append("")
            lines.append("MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES), per kernel (launch-weighted):")
            fam_busy = collections.defaultdict(lambda: [0.0, 0.0])
            for k, (n, v) in sorted(busy.items(), key=lambda kv: -kv[1][1]):
                if k.startswith("at::") or "rocclr" in k or k not in cu or cu[k][1] <= 0 or v <= 0:
                    continue
                lines.append(f"{k[:100]:100s} n={n:6d} mfma_busy={v / (4.0 * cu[k][1]):6.3f}")
                fb = fam_busy[family(k)]
                fb[0] += v
                fb[1] += 4.0 * cu[k][1]
            for k, (num, den) in fam_busy.items():
                traffic.setdefault(k, {})["mfma_busy"] = num / den
        for cname, ks in counters.items():
            lines.append("")
            lines.append(f"counter {cname} (average per launch):")
            for k, (n, v) in sorted(ks.items(), key=lambda kv: -kv[1][1])[:10]:
                if k.startswith("at::") or "rocclr" in k:
                    continue
                lines.append(f"{k[:100]:100s} n={n:6d} avg={v / n:16.1f}")
    text = "\n".join(lines) + "\n"
    if args.txt:
        with open(args.txt, "w") as fh:
            fh.write(text)
    else:
        sys.stdout.write(text)
    if args.json and traffic:
        with open(args.json, "w") as fh:
            json.dump(traffic, fh, indent=1, sort_keys=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
