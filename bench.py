#!/usr/bin/env python3
"""Benchmark of the re-ranking hot path (candidate gather + MaxSim + ranked top-k) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c2|c3|c4|c1]

One step = one pass of the whole path (espn_rerank) over one batch of synthetic input that is
already resident in HBM.  Successive steps use different pre-drawn candidate sets and queries, so
that a batch is not simply served from the last-level cache.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
DEFAULT_STEPS = {"c1": 200, "c2": 400, "c3": 100, "c4": 12}
DEFAULT_SETS = {"c1": 16, "c2": 32, "c3": 8, "c4": 2}

# HBM bytes per score-kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (profiles/*.md give the commands and the copy-kernel calibration); None until measured.
MEASURED_TRAFFIC_BYTES = {
    # (FETCH_SIZE KiB x 2.0 calibration + WRITE_SIZE KiB x 1.0) x 1024, MaxSim kernel, per launch
    "c2": (86786.86 * 2.0 + 273.59) * 1024,       # profiles/maxsim_d32_c2_pmc.md
    "c3": (2251394.18 * 2.0 + 1147.58) * 1024,    # profiles/maxsim_d128_c3_pmc.md
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4"])
    ap.add_argument("--sets", type=int, default=None, help="distinct pre-drawn batches to rotate through")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-queries", type=int, default=None)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB read + 1 GiB write elementwise kernel (a known-size "
                         "reference for hardware byte counters when profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no cross-GPU step); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if int(os.environ.get("WORLD_SIZE", "1")) > 1:
        print("bench.py: launched with WORLD_SIZE > 1; only one rank on one GPU is supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2312_05417_amd import binding as espn, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = espn.lib()                       # fails loudly if the HIP library is not built

    w = synth.WORKLOADS[args.workload]
    seed = synth.DEFAULT_SEED if args.seed is None else args.seed
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[args.workload]
    warmup = args.warmup if args.warmup is not None else max(3, steps // 10)
    n_sets = args.sets if args.sets is not None else DEFAULT_SETS[args.workload]

    t_setup = time.time()
    emb, off = synth.table(w, seed, device=dev)
    counts = np.diff(off)
    table = espn.espn_table_load(emb, off)
    log("%s: table %d docs, %d rows x %d, %.2f GB in HBM (%.1f s)" % (
        w.name, w.n_docs, emb.shape[0], w.dim, emb.numel() * 2 / 1e9, time.time() - t_setup))
    cands_np = [synth.candidates(w, seed, s) for s in range(n_sets)]
    cands = [torch.from_numpy(c).to(dev) for c in cands_np]
    qs = [synth.queries(w, seed, s, device=dev) for s in range(n_sets)]
    out_ids = [torch.empty((w.B, w.k), dtype=torch.int64, device=dev) for _ in range(n_sets)]
    out_sc = [torch.empty((w.B, w.k), dtype=torch.float32, device=dev) for _ in range(n_sets)]
    ws_bytes = espn.espn_workspace_bytes(w.B, w.K)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    scores_view = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K)
    log("inputs ready: %d sets of %d x %d candidates (%.1f s)" % (n_sets, w.B, w.K, time.time() - t_setup))

    # algorithmic bytes of one score-kernel launch: per pair the document's rows, its offset pair,
    # its id and its score; per query its matrix once
    pair_bytes = [float((2 * w.dim * counts[c]).sum()) + 28.0 * c.size for c in cands_np]
    launch_bytes = float(np.mean(pair_bytes)) + w.B * w.Q * w.dim * 2
    flops = float(np.mean([(2.0 * w.Q * w.dim * counts[c]).sum() for c in cands_np]))

    stream = torch.cuda.current_stream()
    st = int(stream.cuda_stream)
    h = table.handle

    def rerank(i):
        s = i % n_sets
        rc = lib.espn_rerank(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, w.k,
                             out_ids[s].data_ptr(), out_sc[s].data_ptr(), ws.data_ptr(), ws_bytes, st)
        if rc != 0:
            raise RuntimeError("espn_rerank failed: " + espn.last_error())

    def score_then_topk(i, ev0, ev1):
        s = i % n_sets
        ev0.record(stream)
        rc = lib.espn_score(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, ws.data_ptr(), st)
        ev1.record(stream)
        rc |= lib.espn_topk(ws.data_ptr(), cands[s].data_ptr(), w.B, w.K, w.k,
                            out_ids[s].data_ptr(), out_sc[s].data_ptr(), st)
        if rc != 0:
            raise RuntimeError("espn_score/espn_topk failed: " + espn.last_error())

    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)            # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region: exactly `steps` passes of the whole path
    for i in range(warmup):
        rerank(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        rerank(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    espn.espn_table_check(table)
    ms_per_step = wall * 1e3 / steps
    docs_per_s = w.B * w.K * steps / wall

    # ---- the dominant (MaxSim) kernel on its own: `steps` launches back to back between one pair of
    # HIP events on the launch stream -> average duration of a launch (dispatch gap included)
    def score_only(i):
        s = i % n_sets
        rc = lib.espn_score(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, ws.data_ptr(), st)
        if rc != 0:
            raise RuntimeError("espn_score failed: " + espn.last_error())

    for i in range(min(warmup, 3)):
        score_only(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(steps):
        score_only(i)
    e1.record(stream)
    torch.cuda.synchronize()
    kern_avg_ms = e0.elapsed_time(e1) / steps

    # ---- the whole path again with an event pair around every MaxSim launch (each pair adds a few
    # microseconds of its own; reported as a cross-check, not used for the roofline)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for i in range(steps):
        score_then_topk(i, *ev[i])
    torch.cuda.synchronize()
    pair_ms = sorted(a.elapsed_time(b) for a, b in ev)
    achieved = launch_bytes / (kern_avg_ms * 1e-3) / 1e9
    log("wall %.4f ms/step; MaxSim kernel avg %.4f ms back-to-back (event pair per launch: median %.4f); "
        "%.1f GB/s algorithmic" % (ms_per_step, kern_avg_ms, pair_ms[len(pair_ms) // 2], achieved))

    result = {
        "metric": "candidate docs MaxSim-scored/sec",
        "value": docs_per_s,
        "unit": "docs/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": w.name, "n_docs": w.n_docs, "dim": w.dim, "rows": int(emb.shape[0]),
            "table_gb": emb.numel() * 2 / 1e9, "tokens_per_doc": "%s[%d,%d]" % (w.count_law, w.count_lo, w.count_hi),
            "batch_queries": w.B, "query_tokens": w.Q, "candidates_per_query": w.K, "top_k": w.k,
            "candidate_law": w.cand_law, "rotating_sets": n_sets, "accumulate": "f32", "seed": seed,
        },
        "wall_algorithmic_gbs": launch_bytes * steps / wall / 1e9,
        "wall_frac_of_hbm_peak": launch_bytes * steps / wall / 1e9 / HBM_PEAK_GBS,
        "roofline": {
            "bound": "hbm", "kernel": "maxsim_mfma_kernel<%d>" % w.dim,
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
            "algorithmic_bytes_per_launch": launch_bytes, "kernel_ms_avg": kern_avg_ms,
            "kernel_ms_event_pair_median": pair_ms[len(pair_ms) // 2], "mfma_tflops": flops / (kern_avg_ms * 1e-3) / 1e12,
        },
    }

    # ---- the CPU oracle on a bounded sample of the same workload (reported baseline + parity check)
    if not args.no_cpu_baseline:
        import oracle
        from tests.parity import assert_scores_close, assert_topk_matches
        # sample: whole batches 0..nb-1 (c1, c2) or the first nq queries of batch 0 (c3, c4), sized for
        # roughly 10-30 core-seconds of oracle work
        nb = {"c1": min(16, n_sets), "c2": min(8, n_sets)}.get(args.workload, 1)
        nq = w.B if args.workload in ("c1", "c2") else min(128, w.B)
        if args.cpu_sample_queries is not None:
            nb, nq = 1, min(args.cpu_sample_queries, w.B)
        threads = oracle.max_threads()
        cpu_s, worst, pairs = 0.0, 0.0, 0
        for s in range(nb):
            sub, loc_off, loc_cand, ids = synth.subtable(emb, off, cands_np[s][:nq])
            q_np = qs[s][:nq].cpu().numpy()
            t1 = time.perf_counter()
            o_ids, o_top, o_all = oracle.rerank(sub, loc_off, q_np, loc_cand, w.k)
            cpu_s += time.perf_counter() - t1
            # parity of the timed configuration on the same sample
            rerank(s)
            torch.cuda.synchronize()
            g_all = scores_view[:nq].cpu().numpy()
            g_ids, g_top = out_ids[s][:nq].cpu().numpy(), out_sc[s][:nq].cpu().numpy()
            worst = max(worst, assert_scores_close(g_all, o_all, w.Q))
            for b in range(nq):
                assert_topk_matches(g_ids[b], g_top[b], o_all[b], cands_np[s][b], w.k, w.Q)
            pairs += nq * w.K
        result["cpu_baseline"] = {
            "value": pairs / cpu_s, "unit": "docs/s", "cores": threads, "kind": "oracle",
            "sample": "first %d queries of each of the first %d batches (%d pairs), fp64, %.1f s wall" % (
                nq, nb, pairs, cpu_s),
        }
        result["parity"] = {"sample_pairs": pairs, "worst_rel_err": worst, "status": "ok"}
        log("oracle: %.0f docs/s on %d threads; parity ok on %d pairs (worst rel err %.2e)" % (
            pairs / cpu_s, threads, pairs, worst))

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
