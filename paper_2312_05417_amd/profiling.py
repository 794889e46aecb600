"""Turns rocprofv3 output of a bench.py run into the short text summaries kept under profiles/.

    python -m paper_2312_05417_amd.profiling kernel-trace --stats-csv DIR/NAME_kernel_stats.csv \\
        --trace-csv DIR/NAME_kernel_trace.csv --bench-json BENCH.json --workload c2 --command "rocprofv3 ..." --out profiles/NAME_kernel_trace.md
    python -m paper_2312_05417_amd.profiling pmc --fetch-csv DIR1/NAME_counter_collection.csv \\
        --write-csv DIR2/NAME_counter_collection.csv --bench-json BENCH.json --workload c2 \\
        --command "rocprofv3 --pmc FETCH_SIZE ..." --command "rocprofv3 --pmc WRITE_SIZE ..." --out profiles/NAME_pmc.md

BENCH.json is what bench.py printed in the profiled run (its roofline block names the dominant kernel and the
algorithmic bytes of one launch).  A pmc summary ends with one machine-readable line, `<!-- bench-traffic {...} -->`,
which bench.py matches against what it launches before it reports `roofline.traffic`.
Nothing here touches the GPU or the library: text in, text out.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import statistics
import subprocess
import sys


def short_name(kernel: str) -> str:
    """`void espn::kernel<...>(args)` -> `espn::kernel<...>`."""
    name = kernel.strip()
    if name.startswith("void "):
        name = name[5:]
    name = name.replace("(anonymous namespace)::", "")
    depth = 0
    for i, ch in enumerate(name):
        if ch == "<":
            depth += 1
        elif ch == ">":
            depth -= 1
        elif ch == "(" and depth == 0:
            return name[:i]
    return name


def pick(result: dict, workload: str | None) -> dict:
    """The entry of a bench.py line for `workload` (a key such as c2, or the start of a workload name)."""
    entries = [result] + list(result.get("configs", []))
    if workload is None:
        return entries[0]
    for e in entries:
        if e["config"]["workload"].startswith(workload):
            return e
    raise SystemExit("no entry for workload %r in the bench line (has: %s)" % (
        workload, ", ".join(e["config"]["workload"] for e in entries)))


def commit_id() -> str:
    try:
        return subprocess.check_output(["git", "rev-parse", "--short", "HEAD"], text=True).strip()
    except Exception:
        return "unknown"


def kernel_trace(args) -> None:
    rows = list(csv.DictReader(open(args.stats_csv)))
    entry = pick(json.load(open(args.bench_json)), args.workload)
    roof, cfg = entry["roofline"], entry["config"]
    want = roof["kernel"]
    mine = [r for r in rows if short_name(r["Name"]) == want]
    if not mine:
        raise SystemExit("kernel %s is not in %s" % (want, args.stats_csv))
    # The same instantiation may also run with fewer batches per launch in other legs of the run (one batch per
    # launch through espn_rerank): the launches of the timed path are the ones with the largest grid.
    spans = collections.defaultdict(list)
    for r in csv.DictReader(open(args.trace_csv)):
        if short_name(r["Kernel_Name"]) == want:
            spans[int(r["Grid_Size_X"])].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    grid = max(spans)
    avg_ns, n_dominant = statistics.mean(spans[grid]), len(spans[grid])
    per_launch = roof["algorithmic_bytes_per_launch"]
    with open(args.out, "w") as f:
        f.write("# rocprofv3 kernel trace: %s (N=%d docs, d=%d, B=%d, K=%d, k=%d, %s lists)\n\n" % (
            cfg["workload"], cfg["n_docs"], cfg["dim"], cfg["batch_queries"], cfg["candidates_per_query"], cfg["top_k"],
            cfg["candidate_law"]))
        f.write("Command (from /tmp with TMPDIR=/tmp, R = repository root):\n\n")
        for c in args.command:
            f.write("    %s\n" % c)
        if any("--kernels-only" in c for c in args.command):
            f.write("\n`--kernels-only`: every leg of bench.py runs on ONE stream, launches back to back (the timed region of the\n"
                    "queue entry point, whose launches overlap on three streams, is left out: overlapped launches would blur the\n"
                    "per-kernel averages).  Warm-up launches are included in the counts.\n")
        f.write("\n")
        f.write("| kernel | calls | total ns | average ns | % of GPU time | min ns | max ns | stddev |\n|---|---|---|---|---|---|---|---|\n")
        for r in rows[:6]:
            f.write("| `%s` | %s | %s | %.0f | %s | %s | %s | %.0f |\n" % (
                short_name(r["Name"])[:100], r["Calls"], r["TotalDurationNs"], float(r["AverageNs"]), r["Percentage"],
                r["MinNs"], r["MaxNs"], float(r["StdDev"])))
        f.write("\nDominant kernel of the timed path: `%s`, %d batch(es) of %d queries per launch, %.0f algorithmic bytes per launch.\n" % (
            want, roof.get("batches_per_launch", 1), cfg["batch_queries"], per_launch))
        if len(spans) > 1:
            f.write("Of its %d launches in the table above, the %d with the full grid (%d work-items) are those launches; the\n"
                    "others are the same instantiation taking one batch per launch in the other legs of the run (%s).\n" % (
                        sum(len(v) for v in spans.values()), n_dominant, grid,
                        ", ".join("%d launches of %d work-items, average %.1f us" % (len(v), g, statistics.mean(v) / 1e3)
                                  for g, v in sorted(spans.items()) if g != grid)))
        f.write("rocprofv3 average %.1f us per launch; bench.py in the same run (HIP events around back-to-back launches on the\n"
                "launch stream, dispatch gaps included): %.1f us.\n" % (avg_ns / 1e3, roof["kernel_ms_avg"] * 1e3))
        what = "8 TB/s HBM" if roof["bound"] == "hbm" else "%.0f GB/s %s" % (roof["peak"], roof["bound"].upper())
        f.write("-> %.1f GB/s = %.3f of the %s peak by the profiler's duration, %.1f GB/s = %.3f by bench.py's timing.\n" % (
            per_launch / avg_ns, per_launch / avg_ns / roof["peak"], what, roof["achieved"], roof["frac"]))
        one = roof.get("one_batch_per_launch")
        if one and roof.get("batches_per_launch", 1) > 1:
            f.write("One batch per launch (`%s`, espn_rerank): %.1f us by the events = %.3f of the peak.\n" % (
                one["kernels"][0], one["kernel_ms_avg"] * 1e3, one["frac"]))
        f.write("The other kernels in the list are the ranking kernels, bench.py's plain-read probe and torch's generators filling\n"
                "the synthetic table.\n")
        for note in args.note:
            f.write(note + "\n")
    print("wrote", args.out)


def pmc(args) -> None:
    entry = pick(json.load(open(args.bench_json)), args.workload)
    roof, cfg = entry["roofline"], entry["config"]
    want = roof["kernel"]
    by = {}
    for counter, path in (("FETCH_SIZE", args.fetch_csv), ("WRITE_SIZE", args.write_csv)):
        vals, grids = collections.defaultdict(list), collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            if r.get("Counter_Name", counter) == counter:
                vals[short_name(r["Kernel_Name"])].append(float(r["Counter_Value"]))
                grids[short_name(r["Kernel_Name"])].append(int(r["Grid_Size"]))
        # of the dominant kernel only the launches with the full grid count (the same instantiation may take one
        # batch per launch in other legs of the run)
        if want in vals:
            full = max(grids[want])
            vals[want] = [v for v, g in zip(vals[want], grids[want]) if g == full]
        by[counter] = vals
    cal = {}
    for counter in by:
        copies = [v for n, v in by[counter].items() if n.split("::")[-1] == "copy_kernel"]
        if not copies:
            raise SystemExit("no calibration copy in the %s run (bench.py --calibration-copy)" % counter)
        cal[counter] = 1048576.0 / statistics.mean(copies[0])
    if want not in by["FETCH_SIZE"] or want not in by["WRITE_SIZE"]:
        raise SystemExit("kernel %s is not in the counter files" % want)
    fetch, write = statistics.mean(by["FETCH_SIZE"][want]), statistics.mean(by["WRITE_SIZE"][want])
    traffic = (fetch * cal["FETCH_SIZE"] + write * cal["WRITE_SIZE"]) * 1024
    alg = roof["algorithmic_bytes_per_launch"]
    with open(args.out, "w") as f:
        f.write("# rocprofv3 hardware byte counters: %s (N=%d docs, d=%d, B=%d, K=%d, k=%d, %s lists)\n\n" % (
            cfg["workload"], cfg["n_docs"], cfg["dim"], cfg["batch_queries"], cfg["candidates_per_query"], cfg["top_k"],
            cfg["candidate_law"]))
        f.write("Two runs (one counter each), from /tmp with TMPDIR=/tmp, R = repository root:\n\n")
        for c in args.command:
            f.write("    %s\n" % c)
        f.write("\nCounter values are KiB per dispatch.  `--calibration-copy` adds one plain copy kernel (bench.py's own probe\n"
                "library) that reads exactly 2^30 bytes and writes 2^30 bytes (1048576 KiB each).\n\n")
        f.write("| kernel | counter | dispatches | mean KiB | min | max |\n|---|---|---|---|---|---|\n")
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            for name, v in by[counter].items():
                if "maxsim" in name or "topk" in name or name.split("::")[-1] == "copy_kernel":
                    f.write("| `%s` | %s | %d | %.2f | %.2f | %.2f |\n" % (name[:100], counter, len(v), statistics.mean(v), min(v), max(v)))
        f.write("\nCalibration: the 1 GiB copy reads as FETCH_SIZE x %.3f and WRITE_SIZE x %.3f.\n\n" % (cal["FETCH_SIZE"], cal["WRITE_SIZE"]))
        f.write("`%s` (%d batch(es) of %d queries per launch): traffic per launch = (%.2f x %.3f + %.2f x %.3f) KiB = %.1f MB;\n"
                "algorithmic bytes per launch = %.1f MB; ratio %.3f.\n" % (
                    want, roof.get("batches_per_launch", 1), cfg["batch_queries"], fetch, cal["FETCH_SIZE"], write,
                    cal["WRITE_SIZE"], traffic / 1e6, alg / 1e6, traffic / alg))
        f.write("These counters sit at the L2/fabric boundary: they cannot tell Infinity-Cache hits from HBM accesses.\n")
        for note in args.note:
            f.write(note + "\n")
        rec = {"workload": cfg["workload"], "kernel": want, "n_docs": cfg["n_docs"], "batch_queries": cfg["batch_queries"],
               "batches_per_launch": roof.get("batches_per_launch", 1), "scored_per_query": cfg["scored_per_query"],
               "query_tokens": cfg["query_tokens"], "candidate_law": cfg["candidate_law"], "seed": cfg["seed"],
               "fetch_size_kib": round(fetch, 2), "write_size_kib": round(write, 2),
               "fetch_factor": round(cal["FETCH_SIZE"], 3), "write_factor": round(cal["WRITE_SIZE"], 3),
               "commit": args.commit or commit_id()}
        f.write("\n<!-- bench-traffic %s -->\n" % json.dumps(rec))
    print("wrote %s: traffic %.1f MB, algorithmic %.1f MB, ratio %.3f" % (args.out, traffic / 1e6, alg / 1e6, traffic / alg))


def batch_threshold(args) -> None:
    """The batch-size sweep of a host-resident run (bench.py --sweep-batch) against Eq. 4's prediction."""
    entry = pick(json.load(open(args.bench_json)), args.workload)
    bt, cfg = entry["batch_threshold"], entry["config"]
    with open(args.out, "w") as f:
        f.write("# Batch threshold of the host-resident mode (Eq. 4 with PCIe in the SSD's place): %s\n\n" % cfg["workload"])
        f.write("Command:\n\n")
        for c in args.command:
            f.write("    %s\n" % c)
        f.write("\nTable: %d documents (%.1f GB, %s), K = %d candidates per query drawn %s, %d staging slots, engine: %s.\n\n" % (
            cfg["n_docs"], cfg["table_gb"], cfg["residency"], cfg["candidates_per_query"], cfg["candidate_law"],
            cfg["staging_slots"], cfg["prefetch_engine"]))
        f.write("Eq. 4: B_max = bandwidth x budget / (bytes per query) = %.1f GB/s x %.0f ms / %.2f MB = **%.1f queries** (a query's %d\n"
                "documents counted in full, as in the paper, where nothing is shared between queries).\n\n" % (
                    bt["bandwidth_gbs"], bt["budget_ms"], bt["bytes_per_query_mb"], bt["predicted_eq4"], cfg["candidates_per_query"]))
        f.write("Measured: the prefetch of the first B queries of a batch (the other slot holding the first B queries of the batch\n"
                "before, as in the running pipeline), best of three:\n\n")
        f.write("| B | transfer ms | MB over PCIe | MB if nothing were shared (Eq. 4's bytes) | GB/s |\n|---|---|---|---|---|\n")
        for b, v in sorted(bt["sweep"].items(), key=lambda kv: int(kv[0])):
            f.write("| %s | %.2f | %.0f | %.0f | %.1f |\n" % (b, v["transfer_ms"], v["pcie_mb"], v["logical_mb"],
                                                            v["pcie_mb"] / v["transfer_ms"]))
        f.write("\nThe transfer outgrows the %.0f ms budget at **B = %s** (interpolated).  The time is bytes moved / link rate at every\n"
                "batch size, so Eq. 4 holds with the bytes that actually move; a document that several queries list, or that the\n"
                "other slot still holds, crosses PCIe once, which is why the measured threshold is %.1f times the prediction made\n"
                "from the paper's no-sharing bytes (a lower bound).\n" % (
                    bt["budget_ms"], "%.0f" % bt["measured"] if bt["measured"] else "beyond the sweep",
                    (bt["measured"] or float("nan")) / bt["predicted_eq4"]))
    print("wrote", args.out)


def main(argv=None) -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("kernel-trace")
    a.add_argument("--stats-csv", required=True)
    a.add_argument("--trace-csv", required=True)
    b = sub.add_parser("pmc")
    b.add_argument("--fetch-csv", required=True)
    b.add_argument("--write-csv", required=True)
    b.add_argument("--commit", default=None, help="commit the run was taken at (default: HEAD)")
    c = sub.add_parser("batch-threshold")
    for p in (a, b, c):
        p.add_argument("--bench-json", required=True)
        p.add_argument("--workload", default=None)
        p.add_argument("--note", action="append", default=[], help="a line to append to the summary")
        p.add_argument("--command", action="append", default=[], help="the profiled command line(s), for the record")
        p.add_argument("--out", required=True)
    args = ap.parse_args(argv)
    {"kernel-trace": kernel_trace, "pmc": pmc, "batch-threshold": batch_threshold}[args.what](args)


if __name__ == "__main__":
    main(sys.argv[1:])
