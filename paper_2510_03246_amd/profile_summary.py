"""Turn rocprofv3 output of bench.py runs into the short summaries kept under profiles/.

    python -m paper_2510_03246_amd.profile_summary --workload opt6.7b --launches OUT/launches.json \
        --stats OUT/prof_bench --fetch OUT/pmc_fetch --write OUT/pmc_write \
        [--mfma OUT/pmc_mfma] [--clock OUT/pmc_clock] --out profiles

Inputs: the output directories of
    rocprofv3 --kernel-trace --stats -d <stats> -o bench --output-format csv -- python3 bench.py <ARGS>
    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <fetch> -o pmc --output-format csv -- python3 bench.py <ARGS> --copy-calibration
    rocprofv3 --pmc WRITE_SIZE ...                                                 (same)
    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY ... (optional, --mfma)
    rocprofv3 --pmc GRBM_GUI_ACTIVE ...                                            (optional, --clock)
with ARGS = --steps 2 --warmup 1 --no-cpu-baseline --no-mfma-ceiling, and the file that one of these runs wrote with
--dump-launches: the library's own records of the timed region, one per launch, in enqueue order.  rocprofv3 names
a GEMM launch by its kernel template only; the records give the kernel class (planes per operand and epilogue), and
the two lists are matched from the end of the process backwards, GEMM launch by GEMM launch.

Outputs: <out>/bench_<workload>_admm_step_kernel_stats.md (kernel statistics, traffic per launch, matrix-core
counters per launch) and <out>/traffic_<workload>.json (HBM bytes per launch and class, stamped with the hash of the
kernel sources, read by bench.py for roofline.traffic).
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import hashlib
import json
import os

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")

# kernels whose every launch belongs to one class of the library's records
KERNEL_CLASS = {"pruned_rows_kernel": "pruned_rows", "cojob_drain_kernel": "pruned_rows_drain", "split_t_kernel": "split_act", "split_c_kernel": "split_act",
                "row_sums_kernel": "row_sums", "plane_c_to_t_kernel": "plane_c_to_t", "splitk_reduce_kernel": "splitk_reduce"}


# how the counters accumulate over the chip: SQ_BUSY_CYCLES once per shader engine, SQ_VALU_MFMA_BUSY_CYCLES once per
# SIMD, GRBM_GUI_ACTIVE once per XCD (8 XCDs x 4 shader engines; 256 CUs x 4 SIMDs)
N_XCD, N_SE, N_SIMD = 8, 32, 1024


def sources_hash() -> str:
    """sha256 over the HIP sources and headers of libstrp.so (sorted by name; the benchmark helper library's one file is
    no part of it): changes whenever a kernel does."""
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(CSRC, "*"))):
        if path.endswith((".hip", ".h")) and os.path.basename(path) != "bench_probe.hip":
            h.update(os.path.basename(path).encode())
            h.update(open(path, "rb").read())
    return h.hexdigest()


def short_name(kernel_name: str) -> str:
    return kernel_name.replace("void ", "").split("(")[0]


def load_counters(directory: str):
    """Dispatches of a --pmc run in order: [{name, wg, ms, counters{}}]."""
    files = glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise FileNotFoundError(f"no *counter_collection.csv under {directory}")
    disp = collections.OrderedDict()
    with open(files[0], newline="") as f:
        for r in csv.DictReader(f):
            d = disp.setdefault(int(r["Dispatch_Id"]), dict(name=short_name(r["Kernel_Name"]), full=r["Kernel_Name"],
                                                            wg=int(r["Grid_Size"]) // max(int(r["Workgroup_Size"]), 1),
                                                            ms=(int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6,
                                                            counters=collections.defaultdict(float)))
            d["counters"][r["Counter_Name"]] += float(r["Counter_Value"])
    return [disp[k] for k in sorted(disp)]


def is_gemm(name: str) -> bool:
    return "strp::gemm_dma_kernel" in name or "strp::gemm_kernel" in name


def classify(dispatches, launches):
    """Attach `cls` to the dispatches of the timed region (the tail of the process); returns the index where it starts."""
    gemm_records = [n for n in launches if n.startswith("gemm_")]
    gemm_idx = [i for i, d in enumerate(dispatches) if is_gemm(d["name"])]
    if len(gemm_idx) < len(gemm_records):
        raise ValueError(f"{len(gemm_idx)} GEMM dispatches in the trace, {len(gemm_records)} in the records")
    tail = gemm_idx[len(gemm_idx) - len(gemm_records):]
    for i, cls in zip(tail, gemm_records):
        dispatches[i]["cls"] = cls
    # the timed region starts at the selection ahead of its first GEMM (scores, then top-k, then the plane writer)
    start = tail[0] if tail else len(dispatches)
    for i in range(start, max(start - 12, -1), -1):
        if "unit_scores_kernel" in dispatches[i]["name"]:
            start = i
            break
    for d in dispatches[start:]:
        if "cls" in d or "strp::" not in d["name"]:
            continue
        for kern, cls in KERNEL_CLASS.items():
            if kern in d["name"]:
                # the record's full name carries a suffix (row_sums_wanda, pruned_rows_az): take it from the records
                full = [n for n in launches if n.startswith(cls)]
                d["cls"] = full[0] if full else cls
    return start


def traffic_tables(fetch_dir, write_dir, launches):
    F, W = load_counters(fetch_dir), load_counters(write_dir)
    if len(F) != len(W):
        raise ValueError(f"the two counter runs differ in their dispatch count: {len(F)} vs {len(W)}")
    cal = [i for i, d in enumerate(F) if "vectorized_elementwise_kernel" in d["name"] and "MulFunctor" in d["full"] and d["wg"] >= 1 << 17]
    if not cal:
        raise ValueError("no copy-calibration kernel in the trace (run bench.py with --copy-calibration)")
    c = cal[-1]
    fcal, wcal = F[c]["counters"]["FETCH_SIZE"], W[c]["counters"]["WRITE_SIZE"]
    fs, ws = (1 << 20) / fcal, (1 << 20) / wcal            # the kernel reads 2^30 and writes 2^30 bytes = 2^20 KiB each
    start = classify(F, launches)
    rows = []
    per_class = collections.defaultdict(lambda: dict(launches=0, fetch_gb=0.0, write_gb=0.0, ms=0.0))
    short = collections.defaultdict(lambda: dict(launches=0, fetch_gb=0.0, write_gb=0.0, ms=0.0))
    for i in range(len(F)):
        d = F[i]
        if "strp::" not in d["name"]:
            continue
        fg = d["counters"]["FETCH_SIZE"] * fs * 1024 / 1e9
        wg = W[i]["counters"]["WRITE_SIZE"] * ws * 1024 / 1e9
        if d["ms"] >= 0.3:
            rows.append((d["name"], d.get("cls", "" if i >= start else "(before the timed region)"), d["wg"], d["ms"], fg, wg))
        elif i >= start:
            sh = short[d["name"]]
            sh["launches"] += 1
            sh["fetch_gb"] += fg
            sh["write_gb"] += wg
            sh["ms"] += d["ms"]
        if i >= start and "cls" in d:
            pc = per_class[d["cls"]]
            pc["launches"] += 1
            pc["fetch_gb"] += fg
            pc["write_gb"] += wg
            pc["ms"] += d["ms"]
    cal_note = (f"Calibration: the elementwise copy kernel of `--copy-calibration` (2^30 bytes in, 2^30 bytes out) reads "
                f"FETCH_SIZE = {fcal:.0f} KiB and WRITE_SIZE = {wcal:.0f} KiB, so FETCH_SIZE is scaled by {fs:.2f} and "
                f"WRITE_SIZE by {ws:.2f}.")
    return rows, per_class, cal_note, dict(fetch_scale=fs, write_scale=ws), short


def mfma_table(mfma_dir, clock_dir, launches):
    M = load_counters(mfma_dir)
    classify(M, launches)
    C = None
    if clock_dir:
        C = load_counters(clock_dir)
        classify(C, launches)
    out = []
    for i, d in enumerate(M):
        if not is_gemm(d["name"]) or "cls" not in d:
            continue
        c = d["counters"]
        busy = c.get("SQ_BUSY_CYCLES", 0.0)
        row = dict(cls=d["cls"], wg=d["wg"], ms=d["ms"],
                   mfma_busy=c.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / busy * (N_SE / N_SIMD) if busy else float("nan"),
                   wait_any=c.get("SQ_WAIT_INST_ANY", 0.0) / c["SQ_WAVE_CYCLES"] if c.get("SQ_WAVE_CYCLES") else float("nan"))
        if C is not None and i < len(C) and C[i]["name"] == d["name"]:
            row["ghz"] = C[i]["counters"].get("GRBM_GUI_ACTIVE", 0.0) / N_XCD / (C[i]["ms"] * 1e6) if C[i]["ms"] > 0 else float("nan")
        out.append(row)
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--workload", default="opt6.7b")
    ap.add_argument("--launches", required=True)
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--mfma")
    ap.add_argument("--clock")
    ap.add_argument("--bench-args", default="--steps 2 --warmup 1 --no-cpu-baseline --no-mfma-ceiling")
    ap.add_argument("--out", default=os.path.join(os.path.dirname(HERE), "profiles"))
    args = ap.parse_args()
    launches = json.load(open(args.launches))["launches"]
    os.makedirs(args.out, exist_ok=True)
    md = [f"# bench.py, {args.workload}-shaped FFN module: kernel statistics, HBM traffic and matrix-core counters per launch", "",
          "Every run below is started on the MI355X box from /tmp with TMPDIR=/tmp; `R` = the repository's root, `OUT` = a scratch directory, "
          "`ARGS` = `" + args.bench_args + "`; the first run also carries `--dump-launches OUT/launches.json` "
          "(the library's own launch records, which name the class of every GEMM launch).",
          "This file and `traffic_" + args.workload + ".json` are then written from the runs' CSV output by", "",
          "    python3 -m paper_2510_03246_amd.profile_summary --workload " + args.workload + " --launches OUT/launches.json "
          "--stats OUT/prof_bench --fetch OUT/pmc_fetch --write OUT/pmc_write --mfma OUT/pmc_mfma "
          "--clock OUT/pmc_clock --out profiles", "",
          f"Kernel sources: sha256 {sources_hash()[:16]} (over csrc/*.hip, *.h of libstrp.so).", ""]
    if args.stats:
        files = glob.glob(os.path.join(args.stats, "**", "*kernel_stats.csv"), recursive=True)
        md += ["## Kernel statistics", "",
               "    rocprofv3 --kernel-trace --stats -d OUT/prof_bench -o bench --output-format csv -- python3 R/bench.py ARGS", "",
               "Library kernels only (torch's input-generation kernels omitted); module initialisation, warm-up and the timed iterations.", "",
               "| kernel | calls | total ms | avg ms | min ms | max ms | % |", "|---|---|---|---|---|---|---|"]
        with open(files[0], newline="") as f:
            for r in csv.DictReader(f):
                if "strp::" not in r["Name"]:
                    continue
                md.append(f"| {short_name(r['Name'])} | {r['Calls']} | {float(r['TotalDurationNs']) / 1e6:.3f} | "
                          f"{float(r['AverageNs']) / 1e6:.4f} | {float(r['MinNs']) / 1e6:.4f} | {float(r['MaxNs']) / 1e6:.4f} | "
                          f"{float(r['Percentage']):.2f} |")
        md.append("")
    if args.fetch and args.write:
        rows, per_class, cal_note, scales, short = traffic_tables(args.fetch, args.write, launches)
        md += ["## HBM-side traffic per launch", "",
               "    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d OUT/pmc_fetch -o pmc --output-format csv -- python3 R/bench.py ARGS --copy-calibration",
               "    rocprofv3 --pmc WRITE_SIZE --kernel-trace -d OUT/pmc_write -o pmc --output-format csv -- python3 R/bench.py ARGS --copy-calibration", "",
               cal_note, "Launches of 0.3 ms and more in dispatch order; `class` is the library's record of that launch.", "",
               "| kernel | class | workgroups | ms | fetch GB | write GB |", "|---|---|---|---|---|---|"]
        md += [f"| {n} | {c} | {wg} | {ms:.2f} | {fg:.2f} | {wgb:.2f} |" for n, c, wg, ms, fg, wgb in rows]
        md += ["", "Per class, averaged over its launches in the timed region:", "",
               "| class | launches | avg ms | fetch GB | write GB | fetch + write GB |", "|---|---|---|---|---|---|"]
        classes = {}
        for cls, pc in sorted(per_class.items(), key=lambda kv: -kv[1]["ms"]):
            n = pc["launches"]
            md.append(f"| {cls} | {n} | {pc['ms'] / n:.3f} | {pc['fetch_gb'] / n:.2f} | {pc['write_gb'] / n:.2f} | "
                      f"{(pc['fetch_gb'] + pc['write_gb']) / n:.2f} |")
            classes[cls] = dict(launches=n, fetch_gb=pc["fetch_gb"] / n, write_gb=pc["write_gb"] / n,
                                traffic_gb=(pc["fetch_gb"] + pc["write_gb"]) / n, avg_ms_under_counters=pc["ms"] / n)
        md += ["", "Launches shorter than 0.3 ms of the timed region, summed per kernel (the factorisation chains' panel and update "
               "launches carry the units of the pruned rows' pass: its 12 GB in and 24 GB out per iteration show up here):", "",
               "| kernel | launches | total ms | fetch GB | write GB |", "|---|---|---|---|---|"]
        for name, sh in sorted(short.items(), key=lambda kv: -(kv[1]["fetch_gb"] + kv[1]["write_gb"])):
            if sh["fetch_gb"] + sh["write_gb"] >= 0.05:
                md.append(f"| {name} | {sh['launches']} | {sh['ms']:.2f} | {sh['fetch_gb']:.2f} | {sh['write_gb']:.2f} |")
        md.append("")
        js = dict(workload=args.workload, sources_sha256=sources_hash(), unit="GB per launch (FETCH_SIZE + WRITE_SIZE, copy-calibrated)",
                  command="rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE --kernel-trace -- python3 bench.py " + args.bench_args + " --copy-calibration",
                  calibration=scales, classes=classes)
        with open(os.path.join(args.out, f"traffic_{args.workload}.json"), "w") as f:
            json.dump(js, f, indent=1, sort_keys=True)
            f.write("\n")
    if args.mfma:
        rows = mfma_table(args.mfma, args.clock, launches)
        md += ["## Matrix-core counters per GEMM launch of the timed region", "",
               "    rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_WAIT_INST_ANY --kernel-trace -d OUT/pmc_mfma -o pmc --output-format csv -- python3 R/bench.py ARGS"]
        if args.clock:
            md.append("    rocprofv3 --pmc GRBM_GUI_ACTIVE --kernel-trace -d OUT/pmc_clock -o pmc --output-format csv -- python3 R/bench.py ARGS")
        md += ["", "`MFMA busy` = (SQ_VALU_MFMA_BUSY_CYCLES / 1024 SIMDs) / (SQ_BUSY_CYCLES / 32 shader engines): the share of the kernel's cycles "
               "in which a SIMD's matrix core executes, averaged over the SIMDs; "
               "`waiting` = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES (share of the wavefront cycles spent waiting on any instruction); "
               "`clock` = GRBM_GUI_ACTIVE / 8 XCDs / launch duration (the clock the chip sustains while the kernel runs; 2.4 GHz nominal).", "",
               "| class | workgroups | ms | MFMA busy | waiting | clock GHz |", "|---|---|---|---|---|---|"]
        for r in rows:
            ghz = f"{r['ghz']:.2f}" if "ghz" in r else "-"
            md.append(f"| {r['cls']} | {r['wg']} | {r['ms']:.2f} | {r['mfma_busy']:.3f} | {r['wait_any']:.3f} | {ghz} |")
        md.append("")
        if args.clock:
            # the same clock figure for every library kernel: the chip holds 2.2-2.4 GHz on everything but the fp16 GEMMs
            agg = collections.defaultdict(lambda: [0.0, 0.0, 0])
            for d in load_counters(args.clock):
                if "strp::" in d["name"] and d["ms"] >= 0.2 and "GRBM_GUI_ACTIVE" in d["counters"]:
                    a = agg[d["name"]]
                    a[0] += d["counters"]["GRBM_GUI_ACTIVE"] / N_XCD
                    a[1] += d["ms"] * 1e6
                    a[2] += 1
            md += ["Sustained clock per kernel over its launches of 0.2 ms and more (whole run):", "",
                   "| kernel | launches | clock GHz |", "|---|---|---|"]
            for name, (cyc, ns, n) in sorted(agg.items(), key=lambda kv: -kv[1][1]):
                md.append(f"| {name} | {n} | {cyc / ns:.2f} |")
            md.append("")
    os.makedirs(args.out, exist_ok=True)
    path = os.path.join(args.out, f"bench_{args.workload}_admm_step_kernel_stats.md")
    with open(path, "w") as f:
        f.write("\n".join(md))
    print("wrote", path)


if __name__ == "__main__":
    main()
