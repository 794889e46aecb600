"""The text tooling around the benchmark (no GPU): rocprofv3 CSV + a bench.py line -> a summary under profiles/,
whose machine-readable line bench.py matches against what it launches before it reports counter traffic."""
import csv
import importlib.util
import json
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

KERNEL = "espn::maxsim_slice_kernel<32, 8, 4, 2, false, 2, true>"
FULL = "void " + KERNEL + "(espn::DocSource, espn::Batch, espn::BatchSet, unsigned int*, int, espn::RankOut)"
COPY = "void espn_bench::copy_kernel(unsigned int const*, unsigned int*, unsigned long)"


def bench_line(per_launch=16):
    cfg = {"workload": "c2-colberter-d32", "n_docs": 1000000, "dim": 32, "batch_queries": 64, "candidates_per_query": 1000,
           "scored_per_query": 1000, "query_tokens": 32, "top_k": 10, "candidate_law": "uniform", "seed": 20231205}
    roof = {"bound": "hbm", "kernel": KERNEL, "batches_per_launch": per_launch, "achieved": 6200.0, "peak": 8000.0,
            "frac": 0.775, "algorithmic_bytes_per_launch": 2.6e9, "kernel_ms_avg": 0.42}
    return {"config": cfg, "roofline": roof}


def counter_csv(path, counter, kib_full, kib_small, kib_copy):
    with open(path, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Dispatch_Id", "Grid_Size", "Kernel_Name", "Counter_Name", "Counter_Value"])
        for i in range(4):
            w.writerow([i, 4194304, FULL, counter, kib_full + i])          # the launches of 16 batches
        for i in range(7):
            w.writerow([10 + i, 262144, FULL, counter, kib_small])         # the same instantiation, fewer batches: ignored
        w.writerow([30, 524288, COPY, counter, kib_copy])


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_for_test", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_short_names():
    from paper_2312_05417_amd import profiling
    assert profiling.short_name(FULL) == KERNEL
    assert profiling.short_name(COPY) == "espn_bench::copy_kernel"
    assert profiling.short_name("void (anonymous namespace)::k<int>(int)") == "k<int>"
    assert profiling.short_name("plain_name") == "plain_name"


def test_pmc_summary_and_the_line_bench_matches(tmp_path, monkeypatch):
    from paper_2312_05417_amd import profiling
    fetch, write, line = tmp_path / "f.csv", tmp_path / "w.csv", tmp_path / "b.json"
    counter_csv(fetch, "FETCH_SIZE", 1400000.0, 88000.0, 524288.0)         # the copy reads 2^20 KiB: this counter shows half
    counter_csv(write, "WRITE_SIZE", 4300.0, 250.0, 1048576.0)
    line.write_text(json.dumps(bench_line()))
    prof_dir = tmp_path / "profiles"
    prof_dir.mkdir()
    out = prof_dir / "x_pmc.md"
    profiling.main(["pmc", "--fetch-csv", str(fetch), "--write-csv", str(write), "--bench-json", str(line),
                    "--command", "rocprofv3 --pmc FETCH_SIZE -- python3 bench.py", "--commit", "abc1234", "--out", str(out)])
    text = out.read_text()
    assert "FETCH_SIZE x 2.000" in text and "WRITE_SIZE x 1.000" in text
    rec = json.loads(text.split("<!-- bench-traffic ")[1].split(" -->")[0])
    assert rec["kernel"] == KERNEL and rec["batches_per_launch"] == 16 and rec["commit"] == "abc1234"
    assert abs(rec["fetch_size_kib"] - 1400001.5) < 1e-6                    # only the full-grid launches are averaged
    # bench.py finds it for the same kernel on the same workload, scaled to its own batches per launch ...
    bench = load_bench()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    sig = {"workload": "c2-colberter-d32", "kernel": KERNEL, "n_docs": 1000000, "batch_queries": 64,
           "scored_per_query": 1000, "query_tokens": 32, "candidate_law": "uniform", "seed": 20231205}
    traffic, source = bench.measured_traffic(sig, 10)
    want = (1400001.5 * 2.0 + 4301.5 * 1.0) * 1024 * 10 / 16
    assert abs(traffic - want) / want < 1e-9 and source["commit"] == "abc1234" and source["file"].endswith("x_pmc.md")
    # ... and refuses it for another kernel instantiation, another batch size or another seed
    for key, other in (("kernel", KERNEL.replace("8, 4", "16, 4")), ("batch_queries", 128), ("seed", 1)):
        traffic, why = bench.measured_traffic(dict(sig, **{key: other}), 10)
        assert traffic is None and isinstance(why, str)


def test_kernel_trace_summary_picks_the_full_grid_launches(tmp_path):
    from paper_2312_05417_amd import profiling
    stats, trace, line = tmp_path / "s.csv", tmp_path / "t.csv", tmp_path / "b.json"
    with open(stats, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"])
        w.writerow([FULL, 11, 2000000, 181818.2, 80.0, 30000, 430000, 1000.0])
    with open(trace, "w", newline="") as f:
        w = csv.writer(f)
        w.writerow(["Kernel_Name", "Start_Timestamp", "End_Timestamp", "Grid_Size_X"])
        for i in range(4):
            w.writerow([FULL, 1000, 1000 + 420000, 4194304])
        for i in range(7):
            w.writerow([FULL, 1000, 1000 + 32000, 262144])
    line.write_text(json.dumps(bench_line()))
    out = tmp_path / "x_kernel_trace.md"
    profiling.main(["kernel-trace", "--stats-csv", str(stats), "--trace-csv", str(trace), "--bench-json", str(line),
                    "--command", "rocprofv3 --kernel-trace --stats -- python3 bench.py --kernels-only", "--out", str(out)])
    text = out.read_text()
    assert "rocprofv3 average 420.0 us per launch" in text and "the 4 with the full grid" in text
    assert "7 launches of 262144 work-items, average 32.0 us" in text
