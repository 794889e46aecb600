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
PCIE_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction, raw
DEFAULT_STEPS = {"c1": 200, "c2": 400, "c3": 100, "c4": 12, "c5": 12, "c2p64": 400, "c3p64": 100,
                 "c2e4m3": 400, "c3e4m3": 100, "c5e4m3": 12}
DEFAULT_SETS = {"c1": 16, "c2": 32, "c3": 8, "c4": 2, "c5": 3, "c2p64": 16, "c3p64": 4, "c2e4m3": 32, "c3e4m3": 8,
                "c5e4m3": 3}

# HBM bytes per score-kernel launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (profiles/*.md give the commands and the copy-kernel calibration); None until measured.
MEASURED_TRAFFIC_BYTES = {
    # (FETCH_SIZE KiB x 2.0 calibration + WRITE_SIZE KiB x 1.0) x 1024, MaxSim kernel, per launch
    "c2": (88960.87 * 2.0 + 252.42) * 1024,          # profiles/maxsim_d32_c2_pmc.md
    "c3": (2262175.08 * 2.0 + 1173.36) * 1024,       # profiles/maxsim_d128_c3_pmc.md
    "c3e4m3": (1161113.45 * 2.0 + 1056.75) * 1024,   # profiles/maxsim_d128_c3e4m3_pmc.md
    "c4": (17564508.73 * 2.0 + 19738.29) * 1024,     # profiles/maxsim_d128_c4_pmc.md
}


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


def run_host_resident(args, w, seed, steps, warmup, n_sets):
    """Table in pinned host memory; batch n+1 is prefetched over PCIe on a side stream into one HBM
    staging slot while batch n is scored from the other."""
    import numpy as np
    import torch
    from paper_2312_05417_amd import binding as espn, synth

    dev = torch.device("cuda:0")
    lib = espn.lib()
    if args.host_docs is not None:
        w = synth.scaled(w, n_docs=args.host_docs)
    t_setup = time.time()
    e4m3 = w.codec == "e4m3"
    row_bytes = w.dim * (1 if e4m3 else 2)
    doc_scale = None
    # the full table is 156 GB (78 GB compressed); if the machine refuses to pin that much, shrink the document
    # count by 20 % until it fits (the PCIe rate does not depend on it once the table is far larger than any cache)
    while True:
        counts = synth.token_counts(w, seed)
        off = synth.offsets_from_counts(counts)
        rows = int(off[-1])
        try:
            emb = torch.empty((rows, w.dim), dtype=torch.uint8 if e4m3 else torch.float16, pin_memory=True)
            break
        except RuntimeError as exc:
            log("cannot pin %.1f GB for %d docs (%s); shrinking by 20 %%" % (rows * row_bytes / 1e9, w.n_docs,
                                                                   str(exc).splitlines()[0]))
            if w.n_docs < 200_000:
                raise
            w = synth.scaled(w, n_docs=int(w.n_docs * 0.8))
    log("%s: pinned %.1f GB of host memory for %d docs (%.1f s)" % (w.name, rows * row_bytes / 1e9, w.n_docs,
                                                                     time.time() - t_setup))
    if e4m3:
        # drawn and compressed in HBM (binary16 table + codes: 1.5 x 158 GB fit the 288 GB), codes copied to the host
        full, _ = synth.table(w, seed, device=dev)
        codes, doc_scale = synth.compress_e4m3(full, off)
        del full
        emb.copy_(codes)
        del codes
        torch.cuda.empty_cache()
    else:
        synth.table(w, seed, device=dev, out=emb)      # drawn on the GPU chunk by chunk, copied to the host
    torch.cuda.synchronize()
    log("table filled (%.1f s)" % (time.time() - t_setup))
    table = espn.espn_table_load_e4m3(emb, doc_scale, off) if e4m3 else espn.espn_table_load(emb, off)

    cands_np = [synth.candidates(w, seed, s) for s in range(n_sets)]
    cands = [torch.from_numpy(c).to(dev) for c in cands_np]
    qs = [synth.queries(w, seed, s, device=dev) for s in range(n_sets)]
    uniq = [np.unique(c) for c in cands_np]
    uniq_rows = [int(counts[u].sum()) for u in uniq]
    cap_rows = int(max(uniq_rows) * 1.05) + 1024
    cap_docs = int(max(u.size for u in uniq) * 1.05) + 1024
    n_slots = args.slots
    espn.espn_staging_create_ring(table, n_slots, cap_rows, cap_docs)
    out_ids = [torch.empty((w.B, w.k), dtype=torch.int64, device=dev) for _ in range(n_sets)]
    out_sc = [torch.empty((w.B, w.k), dtype=torch.float32, device=dev) for _ in range(n_sets)]
    ws_bytes = espn.espn_workspace_bytes(w.B, w.K)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    log("inputs ready: %d sets; distinct docs per batch %.1f %%, %.2f GB per batch, %d slots x %.2f GB (%.1f s)" % (
        n_sets, 100.0 * np.mean([u.size for u in uniq]) / (w.B * w.K), np.mean(uniq_rows) * row_bytes / 1e9,
        n_slots, cap_rows * row_bytes / 1e9, time.time() - t_setup))

    # reference: a plain pinned-host -> device copy of 1 GiB
    ref_src = emb[: (1 << 30) // row_bytes]
    ref_dst = torch.empty_like(ref_src, device=dev)
    ref_dst.copy_(ref_src, non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        ref_dst.copy_(ref_src, non_blocking=True)
    torch.cuda.synchronize()
    memcpy_gbs = 3 * ref_src.numel() * ref_src.element_size() / (time.perf_counter() - t0) / 1e9
    del ref_dst

    main_s, side_s = torch.cuda.current_stream(), torch.cuda.Stream()
    st_main, st_side, h = int(main_s.cuda_stream), int(side_s.cuda_stream), table.handle

    packed = args.engine == "packed"
    cands_host = [torch.from_numpy(c) for c in cands_np] if packed else None

    def prefetch(n):
        s = n % n_sets
        if packed:       # the host finds the distinct documents and packs them; blocks while it does
            rc = lib.espn_prefetch_packed(h, cands_host[s].data_ptr(), w.B, w.K, n % n_slots, st_side)
        else:
            rc = lib.espn_prefetch(h, cands[s].data_ptr(), w.B, w.K, n % n_slots, st_side)
        if rc != 0:
            raise RuntimeError("prefetch failed: " + espn.last_error())

    def rerank(n):
        s = n % n_sets
        rc = lib.espn_rerank_staged(h, n % n_slots, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, w.k,
                                    out_ids[s].data_ptr(), out_sc[s].data_ptr(), ws.data_ptr(), ws_bytes, st_main)
        if rc != 0:
            raise RuntimeError("espn_rerank_staged failed: " + espn.last_error())

    def pipeline(first, count):
        # batch n is scored while batch n+1 is fetched; batch `first` must already be on its way
        for n in range(first, first + count):
            if packed:                  # the blocking call second, so that the scoring is already enqueued
                rerank(n)
                prefetch(n + 1)
            else:
                prefetch(n + 1)
                rerank(n)

    # Batch numbers keep running through every leg below: batch n uses candidate set n % n_sets and slot
    # n % n_slots, and with more sets than slots no slot ever holds the set that is being fetched.  The
    # ring is warm (every slot filled once) before anything is timed.
    warmup = max(warmup, n_slots)
    prefetch(0)
    pipeline(0, warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipeline(warmup, steps)                 # one prefetch and one staged re-rank per step
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    espn.espn_table_check(table)
    ms_per_step = wall * 1e3 / steps
    nxt = warmup + steps + 1                # batches 0 .. warmup + steps have been prefetched

    # transfer alone and scoring alone, each timed with HIP events on its own stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(side_s)
    for n in range(nxt, nxt + steps):
        prefetch(n)
    e1.record(side_s)
    torch.cuda.synchronize()
    xfer_ms = e0.elapsed_time(e1) / steps
    nxt += steps
    # bytes that crossed PCIe, from the library's own counters: `steps` more prefetches, reading the
    # counters after each (documents another slot already holds do not cross again)
    crossed = []
    for n in range(nxt, nxt + steps):
        prefetch(n)
        crossed.append(espn.espn_staging_counters(table, n % n_slots, side_s)["pcie_bytes"])
    pcie_bytes = float(np.mean(crossed))
    distinct_bytes = float(np.mean([uniq_rows[n % n_sets] for n in range(nxt, nxt + steps)])) * row_bytes
    nxt += steps
    last = nxt - 1                          # the batch its slot still holds
    torch.cuda.synchronize()
    e0.record(main_s)
    for _ in range(steps):
        rerank(last)
    e1.record(main_s)
    torch.cuda.synchronize()
    score_ms = e0.elapsed_time(e1) / steps
    achieved = pcie_bytes / (xfer_ms * 1e-3) / 1e9
    log("wall %.2f ms/batch; prefetch alone %.2f ms (%.2f GB over PCIe of %.2f GB distinct: %.1f GB/s; plain 1 GiB "
        "memcpy %.1f GB/s); scoring alone %.2f ms" % (ms_per_step, xfer_ms, pcie_bytes / 1e9, distinct_bytes / 1e9,
                                                      achieved, memcpy_gbs, score_ms))

    logical = float(np.mean([(row_bytes * counts[c]).sum() for c in cands_np]))
    result = {
        "metric": "candidate docs MaxSim-scored/sec", "value": w.B * w.K * steps / wall, "unit": "docs/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {
            "workload": w.name, "n_docs": w.n_docs, "dim": w.dim, "rows": rows, "table_gb": rows * row_bytes / 1e9,
            "codec": w.codec, "residency": "pinned host memory", "batch_queries": w.B, "query_tokens": w.Q,
            "candidates_per_query": w.K, "top_k": w.k, "candidate_law": "zipf(%.1f)" % w.zipf_alpha,
            "rotating_sets": n_sets, "staging_slots": n_slots,
            "prefetch_engine": "host packs into pinned buffers, plain copies" if packed else "gather kernel reading pinned host memory",
            "distinct_docs_per_batch": float(np.mean([u.size for u in uniq])),
            "accumulate": "f32", "seed": seed,
        },
        "roofline": {
            "bound": "pcie", "kernel": "hipMemcpyAsync of packed buffers" if packed else "staging_gather_kernel", "achieved": achieved, "peak": PCIE_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / PCIE_PEAK_GBS, "traffic": None,
            "algorithmic_bytes_per_launch": pcie_bytes, "kernel_ms_avg": xfer_ms,
            "plain_memcpy_h2d_gbs": memcpy_gbs,
        },
        "overlap": {"batch_ms": ms_per_step, "transfer_ms": xfer_ms, "score_ms": score_ms,
                    "batch_over_transfer": ms_per_step / xfer_ms,
                    "logical_gb_per_batch": logical / 1e9, "distinct_gb_per_batch": distinct_bytes / 1e9,
                    "pcie_gb_per_batch": pcie_bytes / 1e9},
    }
    if args.sweep_batch:
        # Eq. 4 with PCIe in the place of the SSD: the largest batch whose fetch fits a time budget.
        # The prediction uses the measured PCIe rate and the mean bytes of a query's K documents (no
        # sharing between queries, as in the paper); the measurement is the prefetch of the first b
        # queries of batch 0, which benefits from documents shared between queries.
        budget_s = args.budget_ms * 1e-3
        per_query = float(np.mean([(row_bytes * counts[c]).sum() for c in cands_np])) / w.B
        predicted = lib.espn_batch_threshold(achieved * 1e9, budget_s, per_query)
        sweep = {}
        b = 16
        while b <= w.B:
            part = cands[0][:b].contiguous()
            prev = cands[1][:b].contiguous()
            t_ms, moved = [], []
            for rep in range(3):
                # slot 1 holds the first b queries of another batch, as it would in the running pipeline
                rc = lib.espn_prefetch(h, prev.data_ptr(), b, w.K, 1, st_side)
                e0.record(side_s)
                rc = rc or lib.espn_prefetch(h, part.data_ptr(), b, w.K, 0, st_side)
                e1.record(side_s)
                torch.cuda.synchronize()
                if rc != 0:
                    raise RuntimeError("espn_prefetch failed: " + espn.last_error())
                t_ms.append(e0.elapsed_time(e1))
                moved.append(espn.espn_staging_counters(table, 0, side_s)["pcie_bytes"])
            sweep[b] = {"transfer_ms": min(t_ms), "pcie_mb": float(np.mean(moved)) / 1e6,
                        "logical_mb": per_query * b / 1e6}
            b *= 2
        fits = [bb for bb, v in sweep.items() if v["transfer_ms"] <= args.budget_ms]
        over = [bb for bb, v in sweep.items() if v["transfer_ms"] > args.budget_ms]
        measured = None
        if fits and over:                  # linear interpolation between the two batch sizes around the budget
            lo, hi = max(fits), min(over)
            t_lo, t_hi = sweep[lo]["transfer_ms"], sweep[hi]["transfer_ms"]
            measured = lo + (hi - lo) * (args.budget_ms - t_lo) / (t_hi - t_lo)
        result["batch_threshold"] = {"budget_ms": args.budget_ms, "bandwidth_gbs": achieved,
                                     "bytes_per_query_mb": per_query / 1e6, "predicted_eq4": predicted,
                                     "measured": measured, "sweep": sweep}
        log("batch threshold for a %.0f ms budget: Eq. 4 predicts %.1f queries, measured %s" % (
            args.budget_ms, predicted, "%.1f" % measured if measured else "outside the sweep"))
        for bb, v in sweep.items():
            log("  B=%4d: transfer %.2f ms, %.0f MB over PCIe (%.0f MB without sharing)" % (
                bb, v["transfer_ms"], v["pcie_mb"], v["logical_mb"]))

    if not args.no_cpu_baseline:
        import oracle
        from tests.parity import assert_scores_close, assert_topk_matches
        nq = min(args.cpu_sample_queries or 64, w.B)
        sub, loc_off, loc_cand, ids = synth.subtable(emb, off, cands_np[0][:nq])
        q_np = qs[0][:nq].cpu().numpy()
        t1 = time.perf_counter()
        if e4m3:
            o_all = oracle.scores_e4m3(sub, doc_scale[ids], loc_off, q_np, loc_cand)
        else:
            o_all = oracle.scores(sub, loc_off, q_np, loc_cand)
        cpu_s = time.perf_counter() - t1
        prefetch(0)
        rerank(0)
        torch.cuda.synchronize()
        g_all = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K)[:nq].cpu().numpy()
        g_ids, g_top = out_ids[0][:nq].cpu().numpy(), out_sc[0][:nq].cpu().numpy()
        worst = assert_scores_close(g_all, o_all, w.Q)
        for b in range(nq):
            assert_topk_matches(g_ids[b], g_top[b], o_all[b], cands_np[0][b], w.k, w.Q)
        result["cpu_baseline"] = {"value": nq * w.K / cpu_s, "unit": "docs/s", "cores": oracle.max_threads(),
                                  "kind": "oracle",
                                  "sample": "first %d queries of batch 0 (%d pairs), fp64, %.1f s wall" % (
                                      nq, nq * w.K, cpu_s)}
        result["parity"] = {"sample_pairs": nq * w.K, "worst_rel_err": worst, "status": "ok"}
        log("oracle: %.0f docs/s; parity ok on %d pairs" % (nq * w.K / cpu_s, nq * w.K))
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "c2p64", "c3p64", "c2e4m3", "c3e4m3", "c5e4m3"])
    ap.add_argument("--sweep-batch", action="store_true",
                    help="c5 only: also time the prefetch for smaller batches and compare the batch size at which "
                         "it outgrows a time budget with Eq. 4's prediction")
    ap.add_argument("--budget-ms", type=float, default=28.0, help="time budget for --sweep-batch")
    ap.add_argument("--host-docs", type=int, default=None,
                    help="c5 only: number of documents of the host-resident table (default 8.8 M = 156 GB pinned)")
    ap.add_argument("--slots", type=int, default=2,
                    help="c5 only: HBM staging slots (2 = double buffering; more slots also serve as a cache of "
                         "recently fetched documents)")
    ap.add_argument("--fetch", default="auto", choices=["auto", "streaming", "cached"],
                    help="how rows of 128 bytes and more are fetched (espn_table_set_fetch); auto = the library decides")
    ap.add_argument("--engine", default="gather", choices=["gather", "packed"],
                    help="c5 only: which prefetch engine fills the staging slots (espn_prefetch / espn_prefetch_packed)")
    ap.add_argument("--batch", type=int, default=None, help="override the number of queries per batch")
    ap.add_argument("--query-tokens", type=int, default=None,
                    help="override the rows per query (up to 64 run on the matrix cores; more take the plain-ALU "
                         "kernel: a comparison point, not a workload of the paper)")
    ap.add_argument("--top-k", type=int, default=None, help="override the number of ranks returned per query")
    ap.add_argument("--cand-law", default=None, choices=["uniform", "zipf"],
                    help="override the law the candidate lists are drawn from")
    ap.add_argument("--sets", type=int, default=None, help="distinct pre-drawn batches to rotate through")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--two-streams", nargs="?", type=int, const=2, default=0, metavar="N",
                    help="also time the same batches issued in turn on N streams, default 2 (reported beside value)")
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
    if args.batch is not None:
        w = synth.scaled(w, B=args.batch, name="%s-B%d" % (w.name, args.batch))
    if args.top_k is not None:
        w = synth.scaled(w, k=args.top_k, name="%s-k%d" % (w.name, args.top_k))
    if args.cand_law is not None:
        w = synth.scaled(w, cand_law=args.cand_law, name="%s-%s" % (w.name, args.cand_law))
    if args.query_tokens is not None:
        w = synth.scaled(w, Q=args.query_tokens, name="%s-Q%d" % (w.name, args.query_tokens))
    seed = synth.DEFAULT_SEED if args.seed is None else args.seed
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[args.workload]
    # steps of tens of microseconds: a warm-up as long as the timed region (about 15 ms), or the first timed
    # steps still run at the clocks of an idle device (measured on c2: 38.3 us per step after 40 warm-up steps,
    # 37.4 us after 400 or 2000)
    short_steps = args.workload in ("c1", "c2", "c2p64", "c2e4m3")
    if args.warmup is not None:
        warmup = args.warmup
    elif short_steps:
        warmup = steps
    else:       # about 20-30 ms of warm-up for the steps of 0.4-5 ms as well (c3 after 10 steps: 0.70 ms per launch
        warmup = max(4, (steps * 2) // 5)       # in the first timed loop, 0.68 ms in the later ones)
    n_sets = args.sets if args.sets is not None else DEFAULT_SETS[args.workload]
    if w.host_resident:
        if n_sets <= args.slots:
            n_sets = args.slots + 1        # a prefetch takes over what other slots hold: never the same batch again
        run_host_resident(args, w, seed, steps, args.warmup if args.warmup is not None else 1, n_sets)
        return

    t_setup = time.time()
    emb, off = synth.table(w, seed, device=dev)
    counts = np.diff(off)
    elem_bytes, doc_scale = 2, None
    if w.codec == "e4m3":
        codes, doc_scale = synth.compress_e4m3(emb, off)
        del emb
        emb, elem_bytes = codes, 1
        table = espn.espn_table_load_e4m3(emb, doc_scale, off)
    else:
        table = espn.espn_table_load(emb, off)
    espn.espn_table_set_fetch(table, {"auto": espn.ESPN_FETCH_AUTO, "streaming": espn.ESPN_FETCH_STREAMING,
                                      "cached": espn.ESPN_FETCH_CACHED}[args.fetch])
    log("%s: table %d docs, %d rows x %d, %.2f GB in HBM (%.1f s)" % (
        w.name, w.n_docs, emb.shape[0], w.dim, emb.numel() * elem_bytes / 1e9, time.time() - t_setup))
    cands_np = [synth.candidates(w, seed, s) for s in range(n_sets)]
    cands = [torch.from_numpy(c).to(dev) for c in cands_np]
    qs = [synth.queries(w, seed, s, device=dev) for s in range(n_sets)]
    out_ids = [torch.empty((w.B, w.k), dtype=torch.int64, device=dev) for _ in range(n_sets)]
    out_sc = [torch.empty((w.B, w.k), dtype=torch.float32, device=dev) for _ in range(n_sets)]
    R = w.rerank_top if w.rerank_top else w.K          # candidates per query that are actually scored
    ws_bytes = espn.espn_workspace_bytes(w.B, R)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    scores_view = ws[: 4 * w.B * R].view(torch.float32).view(w.B, R)
    log("inputs ready: %d sets of %d x %d candidates, %d scored per query (%.1f s)" % (
        n_sets, w.B, w.K, R, time.time() - t_setup))

    # algorithmic bytes of one score-kernel launch: per scored pair the document's rows, its offset
    # pair, its id and its score; per query its matrix once
    scored_np = [c[:, :R] for c in cands_np]
    per_pair = 28.0 + (4.0 if elem_bytes == 1 else 0.0)             # + the document's scale
    pair_bytes = [float((elem_bytes * w.dim * counts[c]).sum()) + per_pair * c.size for c in scored_np]
    launch_bytes = float(np.mean(pair_bytes)) + w.B * w.Q * w.dim * 2
    flops = float(np.mean([(2.0 * w.Q * w.dim * counts[c]).sum() for c in scored_np]))

    stream = torch.cuda.current_stream()
    st = int(stream.cuda_stream)
    h = table.handle

    def rerank(i, on=None, scratch=None):
        s = i % n_sets
        on = st if on is None else on
        scratch = ws if scratch is None else scratch
        if w.rerank_top:
            rc = lib.espn_rerank_partial(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, R, w.k,
                                         out_ids[s].data_ptr(), out_sc[s].data_ptr(), scratch.data_ptr(), ws_bytes, on)
        else:
            rc = lib.espn_rerank(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, w.k,
                                 out_ids[s].data_ptr(), out_sc[s].data_ptr(), scratch.data_ptr(), ws_bytes, on)
        if rc != 0:
            raise RuntimeError("re-rank failed: " + espn.last_error())

    def score_only(i):
        s = i % n_sets
        if w.rerank_top:      # k = 0: the scoring kernel alone, on the first R candidates of every list
            rc = lib.espn_rerank_partial(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, R, 0,
                                         None, None, ws.data_ptr(), ws_bytes, st)
        else:
            rc = lib.espn_score(h, qs[s].data_ptr(), cands[s].data_ptr(), w.B, w.Q, w.K, ws.data_ptr(), st)
        if rc != 0:
            raise RuntimeError("scoring failed: " + espn.last_error())

    def score_then_topk(i):
        score_only(i)
        if not w.rerank_top:
            s = i % n_sets
            rc = lib.espn_topk(ws.data_ptr(), cands[s].data_ptr(), w.B, w.K, w.k,
                               out_ids[s].data_ptr(), out_sc[s].data_ptr(), st)
            if rc != 0:
                raise RuntimeError("espn_topk failed: " + espn.last_error())

    if args.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)            # reads 2^30 bytes, writes 2^30 bytes
        torch.cuda.synchronize()
        del src, dst

    # ---- timed region: exactly `steps` passes of the whole path
    plan = espn.espn_rerank_plan(table, w.B, w.Q, R, min(w.k, R))
    wake_up = 0
    if args.warmup is not None:
        # an explicit --warmup is run as asked; before it, the same call is repeated for about 30 ms so that the
        # device is at speed whatever W is (reported as wake_up_steps, not part of warmup or steps)
        t_wake = time.perf_counter()
        while time.perf_counter() - t_wake < 0.03 and wake_up < 5000:
            for i in range(8):
                rerank(wake_up + i)
            torch.cuda.synchronize()
            wake_up += 8
    t_warm = time.perf_counter()
    for i in range(warmup):
        rerank(i)
    torch.cuda.synchronize()
    if args.warmup is None:
        # the default warm-up counts assume the workload's own batch size; with a smaller batch they may end
        # before the device is at speed (512 Zipf lists at d=128: 1.32 ms per step in a timed region that follows
        # 5 ms of warm-up, 1.20 ms after 30 ms), so go on to about 30 ms
        spent = time.perf_counter() - t_warm
        if spent < 0.03 and warmup > 0:
            more = min(5000, int((0.03 - spent) / (spent / warmup)) + 1)
            for i in range(warmup, warmup + more):
                rerank(i)
            warmup += more
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for i in range(warmup, warmup + steps):
        rerank(i)
    e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    espn.espn_table_check(table)
    ms_per_step = wall * 1e3 / steps
    path_ms = e0.elapsed_time(e1) / steps
    docs_per_s = w.B * R * steps / wall            # documents actually MaxSim-scored

    # ---- the dominant (MaxSim) kernel: average duration of a launch, dispatch gap included, from one
    # pair of HIP events on the launch stream around `steps` back-to-back launches.  Where one pass is
    # one launch (the scoring kernel ranks as well) that is the timed region itself; where a second
    # launch ranks, the scoring kernel is launched `steps` times on its own.
    for i in range(min(warmup, 3)):
        score_only(i)
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    s0.record(stream)
    for i in range(steps):
        score_only(i)
    s1.record(stream)
    torch.cuda.synchronize()
    score_only_ms = s0.elapsed_time(s1) / steps

    # ---- ... and the path as two launches (scores, then the stand-alone ranking kernel)
    two_launch_ms = None
    if not w.rerank_top:
        for i in range(min(warmup, 3)):
            score_then_topk(i)
        u0, u1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        u0.record(stream)
        for i in range(steps):
            score_then_topk(i)
        u1.record(stream)
        torch.cuda.synchronize()
        two_launch_ms = u0.elapsed_time(u1) / steps
    # ---- the same `steps` batches issued alternately on two streams (each with its own workspace): a
    # server with independent batches in flight hides one batch's launch gaps, look-up latency and
    # ranking behind the other batch's streaming.  Reported beside `value`, never as `value`.
    # Only with --two-streams: overlapped launches would blur the per-kernel averages of a profiler run.
    two_stream_wall = None
    if args.two_streams:
        ns = args.two_streams
        side = [torch.cuda.Stream() for _ in range(ns)]
        side_ws = [ws] + [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(ns - 1)]
        side_st = [int(x.cuda_stream) for x in side]
        for i in range(max(min(warmup, 8), ns)):
            rerank(i, side_st[i % ns], side_ws[i % ns])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            rerank(i, side_st[i % ns], side_ws[i % ns])
        torch.cuda.synchronize()
        two_stream_wall = time.perf_counter() - t0
        espn.espn_table_check(table)

    # ---- a measuring stick: a plain contiguous read (nothing depends on what is read) of as many bytes as one
    # launch of the scoring kernel reads, over successive windows of the table (the last-level cache never holds
    # the window that comes next), `steps` launches back to back, timed like the scoring kernel
    window = min(int(launch_bytes) // 4096 * 4096, emb.numel() * elem_bytes // 4096 * 4096)
    flat = emb.view(torch.uint8).view(-1)
    n_windows = max(1, min(64, flat.numel() // window))
    sink = torch.zeros(1, dtype=torch.int64, device=dev)

    def plain_read(i):
        o = (i % n_windows) * window
        rc = lib.espn_stream_read_probe(flat.data_ptr() + o, window, sink.data_ptr(), st)
        if rc != 0:
            raise RuntimeError("read probe failed: " + espn.last_error())

    for i in range(min(warmup, 8)):
        plain_read(i)
    p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    p0.record(stream)
    for i in range(steps):
        plain_read(i)
    p1.record(stream)
    torch.cuda.synchronize()
    plain_read_gbs = window / (p0.elapsed_time(p1) / steps * 1e-3) / 1e9

    kern_avg_ms = path_ms if plan["launches"] == 1 else score_only_ms
    achieved = launch_bytes / (kern_avg_ms * 1e-3) / 1e9
    log("plain read of %.1f MB windows: %.1f GB/s (%d windows)" % (window / 1e6, plain_read_gbs, n_windows))
    log("wall %.4f ms/step (%d launch(es), %d slice(s) of %d per query); MaxSim kernel avg %.4f ms = %.1f GB/s "
        "algorithmic; scoring without ranking %.4f ms; score + stand-alone ranking %s ms" % (
            ms_per_step, plan["launches"], plan["slices"], plan["slice"], kern_avg_ms, achieved, score_only_ms,
            "n/a" if two_launch_ms is None else "%.4f" % two_launch_ms))
    if two_stream_wall is not None:
        log("on %d streams: %.4f ms/step = %.1f GB/s algorithmic" % (
            args.two_streams, two_stream_wall * 1e3 / steps, launch_bytes * steps / two_stream_wall / 1e9))

    result = {
        "metric": "candidate docs MaxSim-scored/sec",
        "value": docs_per_s,
        "unit": "docs/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "wake_up_steps": wake_up,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": w.name, "n_docs": w.n_docs, "dim": w.dim, "rows": int(emb.shape[0]),
            "table_gb": emb.numel() * elem_bytes / 1e9, "codec": w.codec, "tokens_per_doc": "%s[%d,%d]" % (w.count_law, w.count_lo, w.count_hi),
            "batch_queries": w.B, "query_tokens": w.Q, "candidates_per_query": w.K, "scored_per_query": R,
            "top_k": w.k, "candidate_law": w.cand_law, "rotating_sets": n_sets, "accumulate": "f32", "seed": seed,
            "fetch": args.fetch,
        },
        "queries_per_s": w.B * steps / wall,
        "wall_algorithmic_gbs": launch_bytes * steps / wall / 1e9,
        "wall_frac_of_hbm_peak": launch_bytes * steps / wall / 1e9 / HBM_PEAK_GBS,
        "two_streams": None if two_stream_wall is None else {
            "value": w.B * R * steps / two_stream_wall, "unit": "docs/s", "ms_per_step": two_stream_wall * 1e3 / steps,
            "algorithmic_gbs": launch_bytes * steps / two_stream_wall / 1e9,
            "streams": args.two_streams, "note": "the same batches issued in turn on several streams"},
        "roofline": {
            "bound": "hbm",
            "kernel": ("maxsim_slice_kernel<%d>%s" % (w.dim, " (ranks as well)" if plan["launches"] == 1 else "")
                       if w.dim in (32, 128) and w.Q <= 64 else "maxsim_generic_kernel (plain ALU)"),
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": MEASURED_TRAFFIC_BYTES.get(args.workload),
            "algorithmic_bytes_per_launch": launch_bytes, "kernel_ms_avg": kern_avg_ms,
            "launches_per_step": plan["launches"], "slices_per_query": plan["slices"],
            "whole_path_ms_by_events": path_ms, "scoring_without_ranking_ms": score_only_ms,
            "score_then_standalone_ranking_ms": two_launch_ms,
            "mfma_tflops": flops / (kern_avg_ms * 1e-3) / 1e12,
            "plain_read_same_bytes_gbs": plain_read_gbs, "achieved_over_plain_read": achieved / plain_read_gbs,
        },
    }

    # ---- the CPU oracle on a bounded sample of the same workload (reported baseline + parity check)
    if not args.no_cpu_baseline:
        import oracle
        from tests.parity import assert_scores_close, assert_topk_matches
        # sample: whole batches 0..nb-1 (c1, c2) or the first nq queries of batch 0 (c3, c4), sized for
        # roughly 10-30 core-seconds of oracle work
        nb = {"c1": min(16, n_sets), "c2": min(8, n_sets), "c2p64": min(8, n_sets),
              "c2e4m3": min(4, n_sets)}.get(args.workload, 1)
        nq = w.B if args.workload in ("c1", "c2", "c2p64", "c2e4m3") else min(128 * (w.K // R), w.B)
        if w.codec == "e4m3" and args.workload != "c2e4m3":
            nq = min(32, w.B)
        if args.cpu_sample_queries is not None:
            nb, nq = 1, min(args.cpu_sample_queries, w.B)
        threads = oracle.max_threads()
        cpu_s, worst, pairs = 0.0, 0.0, 0
        for s in range(nb):
            sub, loc_off, loc_cand, ids = synth.subtable(emb, off, scored_np[s][:nq])
            q_np = qs[s][:nq].cpu().numpy()
            t1 = time.perf_counter()
            if w.codec == "e4m3":
                o_all = oracle.scores_e4m3(sub, doc_scale[ids], loc_off, q_np, loc_cand)
                o_ids, o_top = oracle.topk(o_all, loc_cand, w.k)
            else:
                o_ids, o_top, o_all = oracle.rerank(sub, loc_off, q_np, loc_cand, w.k)     # the scored prefix
            cpu_s += time.perf_counter() - t1
            # parity of the timed configuration on the same sample
            rerank(s)
            torch.cuda.synchronize()
            g_all = scores_view[:nq].cpu().numpy()
            g_ids, g_top = out_ids[s][:nq].cpu().numpy(), out_sc[s][:nq].cpu().numpy()
            worst = max(worst, assert_scores_close(g_all, o_all, w.Q))
            for b in range(nq):
                assert_topk_matches(g_ids[b], g_top[b], o_all[b], scored_np[s][b], w.k, w.Q)
            pairs += nq * R
        # the same oracle on ONE thread, on a 16th of the first sample (last: the thread count it sets stays)
        one_thread = None
        if w.codec != "e4m3":
            n1 = max(1, nq // 16)
            sub, loc_off, loc_cand, ids = synth.subtable(emb, off, scored_np[0][:n1])
            t1 = time.perf_counter()
            oracle.rerank(sub, loc_off, qs[0][:n1].cpu().numpy(), loc_cand, w.k, threads=1)
            one_thread = n1 * R / (time.perf_counter() - t1)
        result["cpu_baseline"] = {
            "value": pairs / cpu_s, "unit": "docs/s", "cores": threads, "kind": "oracle",
            "sample": "first %d queries of each of the first %d batches (%d pairs), fp64, %.1f s wall" % (
                nq, nb, pairs, cpu_s),
            "value_one_thread": one_thread,
        }
        result["parity"] = {"sample_pairs": pairs, "worst_rel_err": worst, "status": "ok"}
        log("oracle: %.0f docs/s on %d threads%s; parity ok on %d pairs (worst rel err %.2e)" % (
            pairs / cpu_s, threads, "" if one_thread is None else " (%.0f on one)" % one_thread, pairs, worst))

    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
