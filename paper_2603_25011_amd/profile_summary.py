#!/usr/bin/env python3
"""Turns rocprofv3 output of `bench.py` runs into the short text summaries under profiles/ and into
profiles/traffic.json, which bench.py reads for the `traffic` fields of its roofline objects.

Expected input: one directory with a sub-directory per profiler run (each run made with
`--output-format csv`), any subset of

    kt/     rocprofv3 --kernel-trace --stats   -- python3 bench.py --no-cpu --no-extra --steps 20 --warmup 5
    fetch/  rocprofv3 --pmc FETCH_SIZE         -- python3 bench.py --no-cpu --no-extra --steps 3 --warmup 1 --calib-copy
    write/  rocprofv3 --pmc WRITE_SIZE         -- (same command)
    sq/     rocprofv3 --pmc <SQ_* and GRBM_GUI_ACTIVE counters of the forward kernel> -- (steps 3, no --calib-copy)
    l2/     rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum -- (steps 3)

FETCH_SIZE / WRITE_SIZE readings are scaled by what the same counters read for the 1 GiB plain copies
that `--calib-copy` appends (lsr::copy_probe_kernel: 1 048 576 KiB read and written per launch).

    python -m paper_2603_25011_amd.profile_summary gpurun_out/prof c5_large_fwdbwd

prints the summaries; with --write it stores them as profiles/<workload>_*.txt and updates
profiles/traffic.json.
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

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KIB = 1 << 20          # one calibration copy reads and writes 1 GiB


def short_name(name: str) -> str:
    m = re.search(r"lsr::(\w+)", name)
    return "lsr::" + m.group(1) if m else name.split("(")[0][:60]


def find_csv(run_dir: str, suffix: str):
    hits = glob.glob(os.path.join(run_dir, "**", "*" + suffix), recursive=True)
    return hits[0] if hits else None


def kernel_stats(run_dir: str):
    path = find_csv(run_dir, "kernel_stats.csv")
    rows = []
    if path:
        for r in csv.DictReader(open(path)):
            if "lsr::" in r["Name"]:
                rows.append((short_name(r["Name"]), r["Name"], int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]),
                             float(r["MaxNs"]), float(r["Percentage"])))
    return rows


def counters(run_dir: str):
    """{kernel short name: {counter: [values per dispatch]}}; template arguments are kept apart by full name."""
    path = find_csv(run_dir, "counter_collection.csv")
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    if path:
        for r in csv.DictReader(open(path)):
            if "lsr::" in r["Kernel_Name"]:
                acc[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return acc


def mean(v):
    return sum(v) / len(v) if v else 0.0


FWD_KERNELS = ("lsr::fwd_prep_kernel", "lsr::fwd_plan_kernel", "lsr::fwd_rows_kernel", "lsr::fwd_pack_kernel",
               "lsr::fwd_bf16_kernel", "lsr::fwd_merge_kernel")
BWD_KERNELS = ("lsr::bwd_count_kernel", "lsr::bwd_scan_kernel", "lsr::bwd_place_staged_kernel", "lsr::bwd_place_kernel",
               "lsr::bwd_chunk_bounds_kernel", "lsr::bwd_dh_sliced_kernel", "lsr::bwd_dw_sliced_kernel",
               "lsr::bwd_dw_tile_kernel", "lsr::bwd_dh_kernel", "lsr::bwd_dw_kernel")
GATHER_KERNELS = ("lsr::bwd_dh_sliced_kernel", "lsr::bwd_dw_sliced_kernel", "lsr::bwd_dw_tile_kernel")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("prof_dir")
    ap.add_argument("workload")
    ap.add_argument("--write", action="store_true", help="store the summaries under profiles/ and update traffic.json")
    args = ap.parse_args()
    d = args.prof_dir
    out = {}

    ks = kernel_stats(os.path.join(d, "kt"))
    if ks:
        lines = ["rocprofv3 --kernel-trace --stats, workload %s, MI355X, one GPU." % args.workload,
                 "Command (from the repository root):",
                 "  rocprofv3 --kernel-trace --stats -d gpurun_out/prof/kt -o kt --output-format csv -- \\",
                 "      python3 bench.py --no-cpu --no-extra --steps 20 --warmup 5", "",
                 "%-34s %6s %12s %12s %12s %7s" % ("kernel", "calls", "avg us", "min us", "max us", "% time")]
        for short, full, calls, avg, mn, mx, pct in sorted(ks, key=lambda r: -r[6]):
            tmpl = re.search(r"<(.*)>", full)
            label = short + ("<" + tmpl.group(1)[:18] + ">" if tmpl else "")
            lines.append("%-34s %6d %12.1f %12.1f %12.1f %7.2f" % (label[:34], calls, avg / 1e3, mn / 1e3, mx / 1e3, pct))
        out["kernel_trace"] = "\n".join(lines)

    traffic = {}
    fetch, write = counters(os.path.join(d, "fetch")), counters(os.path.join(d, "write"))
    if fetch and write:
        cf = mean(fetch.get("lsr::copy_probe_kernel", {}).get("FETCH_SIZE", []))
        cw = mean(write.get("lsr::copy_probe_kernel", {}).get("WRITE_SIZE", []))
        sf = COPY_KIB / cf if cf else float("nan")
        sw = COPY_KIB / cw if cw else float("nan")
        lines = ["rocprofv3 memory-traffic counters, workload %s, MI355X, one GPU." % args.workload,
                 "Two runs (one counter each), from the repository root:",
                 "  rocprofv3 --pmc FETCH_SIZE -d gpurun_out/prof/fetch -o fetch --output-format csv -- \\",
                 "      python3 bench.py --no-cpu --no-extra --steps 3 --warmup 1 --calib-copy",
                 "  rocprofv3 --pmc WRITE_SIZE -d gpurun_out/prof/write -o write --output-format csv -- (same command)", "",
                 "Calibration: lsr::copy_probe_kernel copies 1 GiB (1 048 576 KiB read, 1 048 576 KiB written) per launch and reads",
                 "  FETCH_SIZE %.0f -> scale %.3f;  WRITE_SIZE %.0f -> scale %.3f." % (cf, sf, cw, sw), "",
                 "Mean per dispatch (counter units are KiB as printed), and GB per forward / backward call after scaling",
                 "(launches per call = dispatches of the kernel / dispatches of lsr::fwd_bf16_kernel resp. lsr::bwd_count_kernel):", "",
                 "%-32s %9s %14s %14s %10s %10s" % ("kernel", "launches", "FETCH_SIZE", "WRITE_SIZE", "read GB", "write GB")]
        tot = {"fwd": [0.0, 0.0], "bwd": [0.0, 0.0]}
        calls = {"fwd": float(len(fetch.get("lsr::fwd_bf16_kernel", {}).get("FETCH_SIZE", [])) or 1),
                 "bwd": float(len(fetch.get("lsr::bwd_count_kernel", {}).get("FETCH_SIZE", [])) or 1)}
        for k in FWD_KERNELS + BWD_KERNELS:
            f, w = fetch.get(k, {}).get("FETCH_SIZE", []), write.get(k, {}).get("WRITE_SIZE", [])
            if not f and not w:
                continue
            per_step = max(len(f), len(w)) / calls["fwd" if k in FWD_KERNELS else "bwd"]
            rgb = mean(f) * sf * 1024 * per_step / 1e9
            wgb = mean(w) * sw * 1024 * per_step / 1e9
            lines.append("%-32s %9.2f %14.0f %14.0f %10.3f %10.3f" % (k, per_step, mean(f), mean(w), rgb, wgb))
            side = "fwd" if k in FWD_KERNELS else "bwd"
            tot[side][0] += rgb
            tot[side][1] += wgb
            if k == "lsr::fwd_bf16_kernel":
                traffic["fwd_fused_kernel_bytes"] = int((rgb + wgb) * 1e9)
        lines += ["", "forward : %.3f GB read + %.3f GB written per call" % tuple(tot["fwd"]),
                  "backward: %.3f GB read + %.3f GB written per call" % tuple(tot["bwd"])]
        out["hbm_counters"] = "\n".join(lines)
        traffic["fwd_bytes"] = int((tot["fwd"][0] + tot["fwd"][1]) * 1e9)
        traffic["bwd_bytes"] = int((tot["bwd"][0] + tot["bwd"][1]) * 1e9)
        traffic["fetch_scale"], traffic["write_scale"] = sf, sw
        traffic["source"] = ("profiles/%s_hbm_counters.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a 1 GiB copy)"
                             % args.workload.split("_")[0])

    l2 = counters(os.path.join(d, "l2"))
    if l2:
        lines = ["rocprofv3 L2 (TCC) counters of the backward gathers, workload %s, MI355X, one GPU." % args.workload,
                 "  rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum -d gpurun_out/prof/l2 -o l2 --output-format csv -- \\",
                 "      python3 bench.py --no-cpu --no-extra --steps 3 --warmup 1", "",
                 "%-32s %10s %16s %16s %16s %9s" % ("kernel", "dispatches", "TCC_REQ", "TCC_HIT", "TCC_MISS", "hit rate")]
        l2_json = {}
        for k in FWD_KERNELS + BWD_KERNELS:
            c = l2.get(k)
            if not c:
                continue
            req, hit, miss = mean(c.get("TCC_REQ_sum", [])), mean(c.get("TCC_HIT_sum", [])), mean(c.get("TCC_MISS_sum", []))
            rate = hit / (hit + miss) if hit + miss > 0 else float("nan")
            lines.append("%-32s %10d %16.0f %16.0f %16.0f %9.3f" % (k, len(c.get("TCC_REQ_sum", [])), req, hit, miss, rate))
            if k in GATHER_KERNELS:
                l2_json[k] = {"req_per_dispatch": req, "hit_per_dispatch": hit, "miss_per_dispatch": miss, "hit_rate": rate}
        out["l2_counters"] = "\n".join(lines)
        traffic["bwd_l2"] = l2_json

    sq = counters(os.path.join(d, "sq"))
    if sq.get("lsr::fwd_bf16_kernel"):
        c = {k: mean(v) for k, v in sq["lsr::fwd_bf16_kernel"].items()}
        lines = ["rocprofv3 SQ counters of lsr::fwd_bf16_kernel, workload %s, MI355X, one GPU (mean per dispatch)." % args.workload,
                 "  rocprofv3 --pmc SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVES SQ_LDS_BANK_CONFLICT \\",
                 "      SQ_INSTS_LDS SQ_WAVE_CYCLES SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE -d gpurun_out/prof/sq -o sq --output-format csv -- \\",
                 "      python3 bench.py --no-cpu --no-extra --steps 3 --warmup 1", ""]
        for k in sorted(c):
            lines.append("%-34s %18.4g" % (k, c[k]))
        if c.get("GRBM_GUI_ACTIVE") and c.get("SQ_VALU_MFMA_BUSY_CYCLES"):
            # GRBM_GUI_ACTIVE is summed over the 8 XCDs; busy cycles over all SIMDs of 256 CUs
            cycles_per_xcd = c["GRBM_GUI_ACTIVE"] / 8.0
            busy = c["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * 256.0 * cycles_per_xcd)
            lines += ["", "cycles per XCD (GRBM_GUI_ACTIVE / 8)          %.4g" % cycles_per_xcd,
                      "matrix-core busy = MFMA_BUSY / (4 SIMDs x 256 CUs x cycles)   %.3f" % busy]
            if c.get("SQ_INSTS_VALU_MFMA_MOPS_BF16"):
                lines.append("flops issued = MOPS_BF16 x 512                 %.4g" % (c["SQ_INSTS_VALU_MFMA_MOPS_BF16"] * 512.0))
        out["fwd_bf16_kernel_sq_counters"] = "\n".join(lines)

    sqb = counters(os.path.join(d, "sqb"))
    if any(sqb.get(k) for k in GATHER_KERNELS):
        lines = ["rocprofv3 SQ counters of the backward's gather kernels, workload %s, MI355X, one GPU (mean per dispatch)." % args.workload,
                 "  rocprofv3 --pmc SQ_INSTS_VALU SQ_INSTS_LDS SQ_INSTS_VMEM_RD SQ_ACTIVE_INST_VALU SQ_WAVE_CYCLES SQ_BUSY_CYCLES \\",
                 "      SQ_LDS_BANK_CONFLICT SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE -d gpurun_out/prof/sqb -o sqb --output-format csv -- \\",
                 "      python3 bench.py --no-cpu --no-extra --steps 3 --warmup 1", "",
                 "VALU issue share = SQ_INSTS_VALU x 4 cycles / (4 SIMDs x 256 CUs x cycles): a wave-wide fp32 or integer",
                 "instruction occupies its SIMD's 16 lanes for 4 cycles (packed fp32 is not used)."]
        sq_json = {}
        for k in GATHER_KERNELS:
            if not sqb.get(k):
                continue
            c = {n: mean(v) for n, v in sqb[k].items()}
            lines += ["", k]
            for n in sorted(c):
                lines.append("  %-32s %18.4g" % (n, c[n]))
            if c.get("GRBM_GUI_ACTIVE") and c.get("SQ_INSTS_VALU"):
                cyc = c["GRBM_GUI_ACTIVE"] / 8.0
                share = c["SQ_INSTS_VALU"] * 4.0 / (4.0 * 256.0 * cyc)
                lines += ["  cycles per XCD (GRBM_GUI_ACTIVE / 8)  %.4g" % cyc, "  VALU issue share                      %.3f" % share]
                sq_json[k] = {"valu_insts_per_dispatch": c["SQ_INSTS_VALU"], "cycles_per_dispatch": cyc, "valu_issue_share": share}
        out["bwd_gather_sq_counters"] = "\n".join(lines)
        traffic["bwd_sq"] = sq_json

    for tag, text in out.items():
        print("=" * 20, tag)
        print(text)
    if args.write:
        pdir = os.path.join(ROOT, "profiles")
        os.makedirs(pdir, exist_ok=True)
        for tag, text in out.items():
            with open(os.path.join(pdir, "%s_%s.txt" % (args.workload.split("_")[0], tag)), "w") as f:
                f.write(text + "\n")
        if traffic:
            tpath = os.path.join(pdir, "traffic.json")
            try:
                doc = json.load(open(tpath))
            except (OSError, ValueError):
                doc = {"workloads": {}}
            doc.setdefault("workloads", {}).setdefault(args.workload, {}).update(traffic)
            with open(tpath, "w") as f:
                json.dump(doc, f, indent=1, sort_keys=True)
                f.write("\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
