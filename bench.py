#!/usr/bin/env python3
"""Benchmark of the re-ranking hot path (candidate gather + MaxSim + ranked top-k) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload all|c1|c2|c3|c4|c5|c5pinned|...]

One step = one pass of the whole path over one batch of synthetic input that is already resident in HBM
(host-resident workloads: one prefetch + one staged re-rank).  Successive steps use different pre-drawn
candidate sets and queries, so that a batch is not simply served from the last-level cache.

The default (`--workload all`) measures every configuration in one process and prints ONE JSON line: the
headline fields are those of c4, the largest configuration a single GPU holds in HBM, and `configs` carries
c3, c2 and the two host-resident runs (c5 at its stated size from ordinary host memory, and the largest
table the machine lets a process pin) with their own ms_per_step, roofline, cpu_baseline and parity.
The timed regions of the HBM-resident configurations run back to back (inputs of all of them are set up
first), each exactly W warm-up and K timed steps; the per-kernel legs and the CPU oracle come afterwards.
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published peak
PCIE_PEAK_GBS = 64.0           # PCIe Gen5 x16, one direction, raw
DEFAULT_STEPS = {"c1": 200, "c2": 400, "c3": 100, "c4": 12, "c5": 12, "c5pinned": 12, "c2p64": 400, "c3p64": 100,
                 "c2e4m3": 400, "c3e4m3": 100, "c5e4m3": 12}
DEFAULT_SETS = {"c1": 16, "c2": 32, "c3": 8, "c4": 2, "c5": 3, "c5pinned": 3, "c2p64": 16, "c3p64": 4, "c2e4m3": 32,
                "c3e4m3": 8, "c5e4m3": 3}
HOST_WORKLOADS = ("c5", "c5pinned", "c5e4m3")
ALL = ("c4", "c3", "c2", "c5", "c5pinned")        # the default run: headline first
SHORT_STEPS = ("c1", "c2", "c2p64", "c2e4m3")     # steps of tens of microseconds


def log(msg):
    print("[bench] " + msg, file=sys.stderr, flush=True)


_ORACLE_THREADS = None


def oracle_threads() -> int:
    """Threads the oracle runs on when it is given all of them: asked once, before any one-thread leg (a thread
    count handed to the oracle stays in force for its later calls)."""
    global _ORACLE_THREADS
    if _ORACLE_THREADS is None:
        import oracle
        _ORACLE_THREADS = oracle.max_threads()
    return _ORACLE_THREADS


# ------------------------------------------------------------------------------------------------------
# Hardware byte counters.  They are collected by separate rocprofv3 --pmc runs (one counter per run) whose
# summaries are tracked under profiles/*_pmc.md; each summary carries one machine-readable line
#     <!-- bench-traffic {json} -->
# naming the workload, the kernel instantiation, the batch shape and the slice plan it was taken at.  A run
# reports `traffic` only if all of that equals what it launches itself; otherwise null.
# ------------------------------------------------------------------------------------------------------
def measured_traffic(signature: dict, per_launch: int):
    """(bytes per launch, where they come from) for a launch of `per_launch` batches, or (None, why not)."""
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_pmc.md"))):
        for m in re.finditer(r"<!-- bench-traffic (\{.*?\}) -->", open(path).read()):
            try:
                rec = json.loads(m.group(1))
            except ValueError:
                continue
            if all(rec.get(key) == val for key, val in signature.items()):
                # the same kernel instantiation on the same workload: traffic is per batch, whatever the number of
                # batches the profiled launches took together
                scale = per_launch / float(rec.get("batches_per_launch", 1))
                traffic = (rec["fetch_size_kib"] * rec["fetch_factor"] + rec["write_size_kib"] * rec["write_factor"]) * 1024 * scale
                return traffic, {"file": os.path.relpath(path, ROOT), "commit": rec.get("commit"),
                                 "profiled_batches_per_launch": rec.get("batches_per_launch", 1),
                                 "fetch_size_kib": rec["fetch_size_kib"], "write_size_kib": rec["write_size_kib"],
                                 "fetch_factor": rec["fetch_factor"], "write_factor": rec["write_factor"]}
    return None, "no counter profile under profiles/ was taken with this kernel on this workload"


class HbmCase:
    """One HBM-resident workload: set-up, the timed region, the per-kernel legs, the CPU oracle."""

    def __init__(self, args, key, seed, steps, warmup, tables):
        import numpy as np
        import torch
        from paper_2312_05417_amd import binding as espn, synth
        self.args, self.key, self.seed, self.steps, self.warmup = args, key, seed, steps, warmup
        self.espn, self.synth, self.torch, self.np = espn, synth, torch, np
        dev = self.dev = torch.device("cuda:0")
        lib = self.lib = espn.lib()
        w = synth.WORKLOADS[key]
        if args.batch is not None:
            w = synth.scaled(w, B=args.batch, name="%s-B%d" % (w.name, args.batch))
        if args.top_k is not None:
            w = synth.scaled(w, k=args.top_k, name="%s-k%d" % (w.name, args.top_k))
        if args.cand_law is not None:
            w = synth.scaled(w, cand_law=args.cand_law, name="%s-%s" % (w.name, args.cand_law))
        if args.query_tokens is not None:
            w = synth.scaled(w, Q=args.query_tokens, name="%s-Q%d" % (w.name, args.query_tokens))
        self.w = w
        n_sets = self.n_sets = args.sets if args.sets is not None else DEFAULT_SETS[key]
        t_setup = time.time()
        # c3 and c4 read the same table: drawn once
        tkey = (w.n_docs, w.dim, w.count_law, w.count_lo, w.count_hi, w.count_mean, w.codec, seed)
        if tkey not in tables:
            emb, off = synth.table(w, seed, device=dev)
            doc_scale = None
            if w.codec == "e4m3":
                codes, doc_scale = synth.compress_e4m3(emb, off)
                del emb
                emb = codes
            tables[tkey] = (emb, off, doc_scale)
        self.emb, self.off, self.doc_scale = emb, off, doc_scale = tables[tkey]
        self.elem_bytes = 1 if w.codec == "e4m3" else 2
        self.counts = np.diff(off)
        self.table = espn.espn_table_load_e4m3(emb, doc_scale, off) if w.codec == "e4m3" else espn.espn_table_load(emb, off)
        espn.espn_table_set_fetch(self.table, {"auto": espn.ESPN_FETCH_AUTO, "streaming": espn.ESPN_FETCH_STREAMING,
                                               "cached": espn.ESPN_FETCH_CACHED}[args.fetch])
        log("%s: table %d docs, %d rows x %d, %.2f GB in HBM (%.1f s)" % (
            w.name, w.n_docs, emb.shape[0], w.dim, emb.numel() * self.elem_bytes / 1e9, time.time() - t_setup))
        self.cands_np = [synth.candidates(w, seed, s) for s in range(n_sets)]
        self.cands = [torch.from_numpy(c).to(dev) for c in self.cands_np]
        self.qs = [synth.queries(w, seed, s, device=dev) for s in range(n_sets)]
        # what the library is told about the lists (once per workload, as a server would at start-up)
        self.overlap = espn.espn_table_sample(self.table, self.cands[0])
        R = self.R = w.rerank_top if w.rerank_top else w.K          # candidates per query that are actually scored
        self.batched = not w.rerank_top                              # partial re-ranking has no queue entry point
        n_out = max(steps, warmup, n_sets)
        self.out_ids = torch.empty((n_out, w.B, w.k), dtype=torch.int64, device=dev)
        self.out_sc = torch.empty((n_out, w.B, w.k), dtype=torch.float32, device=dev)
        self.part = espn.espn_workspace_bytes(w.B, R)
        self.ws_bytes = max(espn.espn_batches_workspace_bytes(self.table, n, w.B, w.Q, R, min(w.k, R)) for n in (1, 3, max(steps, 1), max(warmup, 1)))
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        self.scores_view = self.ws[: 4 * w.B * R].view(torch.float32).view(w.B, R)
        self.stream = torch.cuda.current_stream()
        self.st = int(self.stream.cuda_stream)
        self.h = self.table.handle
        self.plan = espn.espn_rerank_plan(self.table, w.B, w.Q, R, min(w.k, R))
        self.kernels = espn.espn_rerank_plan_kernels(self.table, w.B, w.Q, R, min(w.k, R))
        # overlapping lists in a long launch: sorted by document id first (a launch of its own), then scored
        self.ordered = self.batched and any("order_lists_kernel" in name for name in self.kernels)
        self.one_q = [espn.pointer_list([q], torch.float16, "q") for q in self.qs]
        self.one_cand = [espn.pointer_list([c], torch.int64, "cand") for c in self.cands]
        # how the queue entry point runs the timed region: batches per launch, launches, streams, kernels of a chunk
        self.qplan = (espn.espn_batches_plan(self.table, steps, w.B, w.Q, R, min(w.k, R)) if self.batched else
                      {"fuse": 1, "launches": steps, "streams": 1, "kernels": self.kernels})
        # algorithmic bytes of one score-kernel launch: per scored pair the document's rows, its offset
        # pair, its id and its score; per query its matrix once
        self.scored_np = [c[:, :R] for c in self.cands_np]
        per_pair = 28.0 + (4.0 if self.elem_bytes == 1 else 0.0)             # + the document's scale
        pair_bytes = [float((self.elem_bytes * w.dim * self.counts[c]).sum()) + per_pair * c.size for c in self.scored_np]
        self.launch_bytes = float(np.mean(pair_bytes)) + w.B * w.Q * w.dim * 2
        self.flops = float(np.mean([(2.0 * w.Q * w.dim * self.counts[c]).sum() for c in self.scored_np]))
        # ... and the bytes of the DISTINCT documents of a launch (what memory has to deliver at least once;
        # equal to the above where no two queries list the same document)
        distinct = [np.unique(c) for c in self.scored_np]
        self.distinct_bytes = float(np.mean([float((self.elem_bytes * w.dim * self.counts[u]).sum()) + 16.0 * u.size
                                             for u in distinct])) + (12.0 * w.B * R) + w.B * w.Q * w.dim * 2
        self.distinct_docs = float(np.mean([u.size for u in distinct]))
        log("%s: %d sets of %d x %d candidates, %d scored per query, sampled overlap %.3f (%.1f s)" % (
            w.name, n_sets, w.B, w.K, R, self.overlap, time.time() - t_setup))

    # -- enqueue helpers
    def pointer_lists(self, first, count):
        e, t = self.espn, self.torch
        idx = [(first + i) % self.n_sets for i in range(count)]
        return (e.pointer_list([self.qs[s] for s in idx], t.float16, "q"),
                e.pointer_list([self.cands[s] for s in idx], t.int64, "cand"),
                e.pointer_list([self.out_ids[i] for i in range(count)], t.int64, "out_ids"),
                e.pointer_list([self.out_sc[i] for i in range(count)], t.float32, "out_scores"))

    def rerank_queue(self, lists, count):
        w = self.w
        rc = self.lib.espn_rerank_batches(self.h, count, lists[0], lists[1], w.B, w.Q, w.K, w.k, lists[2], lists[3],
                                          self.ws.data_ptr(), self.ws_bytes, self.st)
        if rc != 0:
            raise RuntimeError("espn_rerank_batches failed: " + self.espn.last_error())

    def rerank(self, i, on=None):
        w, s = self.w, i % self.n_sets
        on = self.st if on is None else on
        o = i % self.out_ids.shape[0]
        if w.rerank_top:
            rc = self.lib.espn_rerank_partial(self.h, self.qs[s].data_ptr(), self.cands[s].data_ptr(), w.B, w.Q, w.K, self.R,
                                              w.k, self.out_ids[o].data_ptr(), self.out_sc[o].data_ptr(), self.ws.data_ptr(),
                                              self.part, on)
        else:
            rc = self.lib.espn_rerank(self.h, self.qs[s].data_ptr(), self.cands[s].data_ptr(), w.B, w.Q, w.K, w.k,
                                      self.out_ids[o].data_ptr(), self.out_sc[o].data_ptr(), self.ws.data_ptr(), self.part, on)
        if rc != 0:
            raise RuntimeError("re-rank failed: " + self.espn.last_error())

    def score_only(self, i):
        w, s = self.w, i % self.n_sets
        if w.rerank_top:      # k = 0: the scoring kernel alone, on the first R candidates of every list
            rc = self.lib.espn_rerank_partial(self.h, self.qs[s].data_ptr(), self.cands[s].data_ptr(), w.B, w.Q, w.K, self.R,
                                              0, None, None, self.ws.data_ptr(), self.part, self.st)
        elif self.ordered:    # lists taken in id order: the ordering launch and the scoring launch, as the timed path runs them
            rc = self.lib.espn_rerank_batches(self.h, 1, self.one_q[s], self.one_cand[s], w.B, w.Q, w.K, 0, None, None,
                                              self.ws.data_ptr(), self.ws_bytes, self.st)
        else:
            rc = self.lib.espn_score(self.h, self.qs[s].data_ptr(), self.cands[s].data_ptr(), w.B, w.Q, w.K,
                                     self.ws.data_ptr(), self.st)
        if rc != 0:
            raise RuntimeError("scoring failed: " + self.espn.last_error())

    # -- the timed region: exactly `warmup` untimed and `steps` timed passes of the whole path
    def timed(self):
        torch, w = self.torch, self.w
        if self.batched:
            # one call per region: the queue of batches goes to the library, which spreads it over its streams
            warm = self.pointer_lists(0, self.warmup) if self.warmup else None
            run = self.pointer_lists(self.warmup, self.steps)
            if warm:
                self.rerank_queue(warm, self.warmup)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            self.rerank_queue(run, self.steps)
            torch.cuda.synchronize()
            self.wall = time.perf_counter() - t0
        else:
            for i in range(self.warmup):
                self.rerank(i)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for i in range(self.warmup, self.warmup + self.steps):
                self.rerank(i)
            torch.cuda.synchronize()
            self.wall = time.perf_counter() - t0
        self.espn.espn_table_check(self.table)
        self.ms_per_step = self.wall * 1e3 / self.steps
        log("%s: %.4f ms/step over %d steps (%s)" % (w.name, self.ms_per_step, self.steps,
                                                      "espn_rerank_batches" if self.batched else "one call per batch"))

    def _events(self, fn, n):
        torch = self.torch
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record(self.stream)
        for i in range(n):
            fn(i)
        b.record(self.stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    # -- per-kernel legs, all on ONE stream with HIP events around `steps` back-to-back launches
    def legs(self):
        torch, w, steps = self.torch, self.w, self.steps
        from paper_2312_05417_amd import benchprobe
        pre = min(max(self.warmup, 1), 3)
        for i in range(pre):
            self.rerank(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        self.path_ms = self._events(self.rerank, steps)            # the whole path, one espn_rerank call per batch
        self.sequential_wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        for i in range(pre):
            self.score_only(i)
        self.score_only_ms = self._events(self.score_only, steps)  # the dominant kernel alone
        self.two_launch_ms = None
        if not w.rerank_top:
            def score_then_topk(i):
                self.score_only(i)
                s = i % self.n_sets
                rc = self.lib.espn_topk(self.ws.data_ptr(), self.cands[s].data_ptr(), w.B, w.K, w.k,
                                        self.out_ids[0].data_ptr(), self.out_sc[0].data_ptr(), self.st)
                if rc != 0:
                    raise RuntimeError("espn_topk failed: " + self.espn.last_error())
            for i in range(pre):
                score_then_topk(i)
            self.two_launch_ms = self._events(score_then_topk, steps)
        # a measuring stick: a plain contiguous read (nothing depends on what is read) of as many bytes as one
        # launch of the dominant scoring kernel reads, over successive windows of the table
        window = min(int(self.qplan["fuse"] * self.launch_bytes) // 4096 * 4096, self.emb.numel() * self.elem_bytes // 4096 * 4096)
        flat = self.emb.view(torch.uint8).view(-1)
        n_windows = max(1, min(64, flat.numel() // window))
        sink = torch.zeros(1, dtype=torch.int64, device=self.dev)

        def plain_read(i):
            benchprobe.stream_read(flat.data_ptr() + (i % n_windows) * window, window, sink.data_ptr(), self.st)

        for i in range(min(max(self.warmup, 1), 8)):
            plain_read(i)
        self.plain_read_gbs = window / (self._events(plain_read, steps) * 1e-3) / 1e9
        if self.args.calibration_copy:      # a copy of known size for the profiler's byte counters: 1 GiB read, 1 GiB written
            src = torch.ones(1 << 28, dtype=torch.float32, device=self.dev)
            dst = torch.empty_like(src)
            torch.cuda.synchronize()
            benchprobe.copy(src.data_ptr(), dst.data_ptr(), 1 << 30, self.st)
            torch.cuda.synchronize()
            del src, dst
        self.single_kern_ms = self.path_ms if self.plan["launches"] == 1 else self.score_only_ms
        # the dominant kernel of the timed region: where the queue entry point scores several batches per launch,
        # that launch alone (no ranking: k = 0), back to back on one stream, as many batches per launch as there
        self.per_launch = per = self.qplan["fuse"]
        self.kern_ms, self.dominant = self.single_kern_ms, (self.kernels[0] if self.kernels else None)
        if per > 1:
            e, t = self.espn, torch
            n_launch = max(4, -(-steps // per))
            lists = []
            for x in range(n_launch):
                idx = [(x * per + i) % self.n_sets for i in range(per)]
                lists.append((e.pointer_list([self.qs[s] for s in idx], t.float16, "q"),
                              e.pointer_list([self.cands[s] for s in idx], t.int64, "cand")))

            def fused_score(x):
                rc = self.lib.espn_rerank_batches(self.h, per, lists[x][0], lists[x][1], w.B, w.Q, w.K, 0, None, None,
                                                  self.ws.data_ptr(), self.ws_bytes, self.st)
                if rc != 0:
                    raise RuntimeError("espn_rerank_batches (scoring only) failed: " + self.espn.last_error())

            for x in range(min(n_launch, 3)):
                fused_score(x)
            self.kern_ms = self._events(fused_score, n_launch)
            self.dominant = self.qplan["kernels"][0]
        log("%s: MaxSim kernel avg %.4f ms for %d batch(es) per launch = %.1f GB/s algorithmic (%s); one batch per launch "
            "%.4f ms; one espn_rerank call per batch %.4f ms; plain read %.1f GB/s" % (
                w.name, self.kern_ms, per, per * self.launch_bytes / (self.kern_ms * 1e-3) / 1e9, self.dominant,
                self.single_kern_ms, self.sequential_wall_ms, self.plain_read_gbs))

    # -- the CPU oracle on a bounded sample of the same workload (reported baseline + parity check)
    def oracle(self, budget_queries=None):
        import oracle
        from tests.parity import assert_scores_close, assert_topk_matches
        torch, w, key, synth = self.torch, self.w, self.key, self.synth
        nb = {"c1": min(16, self.n_sets), "c2": min(8, self.n_sets), "c2p64": min(8, self.n_sets),
              "c2e4m3": min(4, self.n_sets)}.get(key, 1)
        nq = w.B if key in SHORT_STEPS else min(128 * (w.K // self.R), w.B)
        if w.codec == "e4m3" and key != "c2e4m3":
            nq = min(32, w.B)
        if budget_queries is not None:
            nb, nq = 1, min(budget_queries, w.B)
        threads = oracle_threads()
        cpu_s, worst, pairs = 0.0, 0.0, 0
        for s in range(nb):
            sub, loc_off, loc_cand, ids = synth.subtable(self.emb, self.off, self.scored_np[s][:nq])
            q_np = self.qs[s][:nq].cpu().numpy()
            t1 = time.perf_counter()
            if w.codec == "e4m3":
                o_all = oracle.scores_e4m3(sub, self.doc_scale[ids], loc_off, q_np, loc_cand, threads=threads)
                o_ids, o_top = oracle.topk(o_all, loc_cand, w.k)
            else:
                o_ids, o_top, o_all = oracle.rerank(sub, loc_off, q_np, loc_cand, w.k, threads=threads)     # the scored prefix
            cpu_s += time.perf_counter() - t1
            # parity of the timed configuration on the same sample: the queue entry point with three batches
            # in flight (the sampled one first), or the per-batch call where there is no queue
            if self.batched:
                lists = self.pointer_lists(s, 3)
                self.rerank_queue(lists, 3)
            else:
                self.rerank(s)
            torch.cuda.synchronize()
            g_all = self.scores_view[:nq].cpu().numpy()
            o = 0 if self.batched else s % self.out_ids.shape[0]
            g_ids, g_top = self.out_ids[o][:nq].cpu().numpy(), self.out_sc[o][:nq].cpu().numpy()
            worst = max(worst, assert_scores_close(g_all, o_all, w.Q))
            for b in range(nq):
                assert_topk_matches(g_ids[b], g_top[b], o_all[b], self.scored_np[s][b], w.k, w.Q)
            pairs += nq * self.R
        one_thread = None
        if w.codec != "e4m3":       # the same oracle on ONE thread, on a 16th of the first sample
            n1 = max(1, nq // 16)
            sub, loc_off, loc_cand, ids = synth.subtable(self.emb, self.off, self.scored_np[0][:n1])
            t1 = time.perf_counter()
            oracle.rerank(sub, loc_off, self.qs[0][:n1].cpu().numpy(), loc_cand, w.k, threads=1)
            one_thread = n1 * self.R / (time.perf_counter() - t1)
        self.cpu_baseline = {
            "value": pairs / cpu_s, "unit": "docs/s", "cores": threads, "kind": "oracle",
            "sample": "first %d queries of each of the first %d batches (%d pairs), fp64, %.1f s wall" % (nq, nb, pairs, cpu_s),
            "value_one_thread": one_thread,
        }
        self.parity = {"sample_pairs": pairs, "worst_rel_err": worst, "status": "ok",
                       "entry_point": "espn_rerank_batches" if self.batched else "espn_rerank_partial"}
        log("%s: oracle %.0f docs/s on %d threads%s; parity ok on %d pairs (worst rel err %.2e)" % (
            w.name, pairs / cpu_s, threads, "" if one_thread is None else " (%.0f on one)" % one_thread, pairs, worst))

    def result(self):
        w, steps, R, per = self.w, self.steps, self.R, self.per_launch
        launch_bytes, distinct_bytes = per * self.launch_bytes, per * self.distinct_bytes
        achieved = launch_bytes / (self.kern_ms * 1e-3) / 1e9
        overlapping = self.distinct_docs < 0.9 * w.B * R
        signature = {"workload": w.name, "kernel": self.dominant, "n_docs": w.n_docs, "batch_queries": w.B,
                     "scored_per_query": R, "query_tokens": w.Q, "candidate_law": w.cand_law, "seed": self.seed}
        traffic, source = measured_traffic(signature, per)
        single = self.launch_bytes / (self.single_kern_ms * 1e-3) / 1e9
        roofline = {
            "bound": "hbm", "kernel": self.dominant, "batches_per_launch": per,
            "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic, "traffic_source": source,
            "frac_basis": ("logical bytes: every listing of a document counted, repeats are served by the caches"
                           if overlapping else "algorithmic bytes (no two queries of a batch share a document to speak of)"),
            "algorithmic_bytes_per_launch": launch_bytes, "kernel_ms_avg": self.kern_ms,
            "distinct": {"docs_per_batch": self.distinct_docs, "bytes_per_launch": distinct_bytes,
                         "achieved": distinct_bytes / (self.kern_ms * 1e-3) / 1e9,
                         "frac": distinct_bytes / (self.kern_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         "note": "bytes of the distinct documents of each batch: what HBM has to deliver at least once"},
            "queue": self.qplan,
            "ordering_launch_included": self.ordered,
            "one_batch_per_launch": {"kernels": self.kernels, "kernel_ms_avg": self.single_kern_ms, "achieved": single,
                                     "frac": single / HBM_PEAK_GBS, "slices_per_query": self.plan["slices"],
                                     "launches_per_batch": self.plan["launches"],
                                     "whole_path_ms_by_events": self.path_ms,
                                     "scoring_without_ranking_ms": self.score_only_ms,
                                     "score_then_standalone_ranking_ms": self.two_launch_ms},
            "mfma_tflops": per * self.flops / (self.kern_ms * 1e-3) / 1e12,
            "plain_read_gbs": self.plain_read_gbs,
        }
        res = {
            "metric": "candidate docs MaxSim-scored/sec",
            "value": w.B * R * steps / self.wall,            # documents actually MaxSim-scored
            "unit": "docs/s", "n_gpus": 1, "steps": steps, "warmup": self.warmup, "ms_per_step": self.ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
            "config": {
                "workload": w.name, "n_docs": w.n_docs, "dim": w.dim, "rows": int(self.emb.shape[0]),
                "table_gb": self.emb.numel() * self.elem_bytes / 1e9, "codec": w.codec,
                "tokens_per_doc": "%s[%d,%d]" % (w.count_law, w.count_lo, w.count_hi),
                "batch_queries": w.B, "query_tokens": w.Q, "candidates_per_query": w.K, "scored_per_query": R,
                "top_k": w.k, "candidate_law": w.cand_law, "rotating_sets": self.n_sets, "accumulate": "f32",
                "seed": self.seed, "fetch": self.args.fetch, "sampled_overlap": self.overlap,
                "entry_point": ("espn_rerank_batches: the %d timed batches in one call (%d scoring launch(es) of up to %d "
                                "batches on %d stream(s))" % (steps, self.qplan["launches"], per, self.qplan["streams"]))
                if self.batched else "espn_rerank_partial, one call per batch on one stream",
            },
            "queries_per_s": w.B * steps / self.wall,
            "wall_algorithmic_gbs": self.launch_bytes * steps / self.wall / 1e9,
            "wall_frac_of_hbm_peak": self.launch_bytes * steps / self.wall / 1e9 / HBM_PEAK_GBS,
            "one_call_per_batch": {"ms_per_step": self.sequential_wall_ms, "value": w.B * R / (self.sequential_wall_ms * 1e-3),
                                   "wall_frac_of_hbm_peak": self.launch_bytes / (self.sequential_wall_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                                   "note": "espn_rerank (espn_rerank_partial) called once per batch on one stream"},
            "roofline": roofline,
        }
        if hasattr(self, "cpu_baseline"):
            res["cpu_baseline"], res["parity"] = self.cpu_baseline, self.parity
        return res

    def free(self):
        self.table.free()


def host_memory_available():
    """MemAvailable of /proc/meminfo in bytes, or None."""
    try:
        for line in open("/proc/meminfo"):
            if line.startswith("MemAvailable:"):
                return int(line.split()[1]) * 1024
    except OSError:
        pass
    return None


def advise_huge_pages(t):
    """Ask for transparent huge pages under a large host tensor before it is first touched (the packing engine
    reads documents from all over a 156 GB table: fewer TLB misses).  Best effort."""
    import ctypes
    try:
        libc = ctypes.CDLL(None, use_errno=True)
        page = 2 << 20
        start = (t.data_ptr() + page - 1) // page * page
        length = (t.data_ptr() + t.numel() * t.element_size() - start) // page * page
        if length > 0:
            rc = libc.madvise(ctypes.c_void_p(start), ctypes.c_size_t(length), 14)      # MADV_HUGEPAGE
            log("madvise(MADV_HUGEPAGE) on %.1f GB: %s" % (length / 1e9, "ok" if rc == 0 else "errno %d" % ctypes.get_errno()))
    except Exception as exc:        # noqa: BLE001
        log("madvise not available: %r" % (exc,))


def release_pinned_cache(torch):
    """Pinned host blocks that torch has freed stay pinned in its allocator's cache; this machine pins 64 GiB per
    process at most, so they are handed back before a table is pinned."""
    import gc
    gc.collect()
    empty = getattr(torch._C, "_host_emptyCache", None)
    if empty is not None:
        empty()


def run_host_resident(args, key, seed, steps, warmup):
    """Table in host memory; batch n+1 is prefetched over PCIe on a side stream into one HBM staging slot while
    batch n is scored from the other.  c5 / c5e4m3: the stated table size in ORDINARY host memory, packed by the
    host into the library's pinned buffers and sent with plain copies (espn_prefetch_packed) - unless the
    machine pins the whole table, in which case the gather kernel reads it directly.  c5pinned: the largest
    table the machine pins, read by the gather kernel (espn_prefetch)."""
    import numpy as np
    import torch
    from paper_2312_05417_amd import binding as espn, synth

    dev = torch.device("cuda:0")
    lib = espn.lib()
    w = synth.WORKLOADS["c5" if key == "c5pinned" else key]
    asked_docs = w.n_docs
    if args.host_docs is not None:
        w = synth.scaled(w, n_docs=args.host_docs)
    if args.batch is not None:
        w = synth.scaled(w, B=args.batch)
    n_slots = args.slots
    n_sets = max(args.sets if args.sets is not None else DEFAULT_SETS[key], n_slots + 1)
    t_setup = time.time()
    e4m3 = w.codec == "e4m3"
    row_bytes = w.dim * (1 if e4m3 else 2)
    doc_scale = None
    engine = args.engine
    pinned = True
    dtype = torch.uint8 if e4m3 else torch.float16
    release_pinned_cache(torch)
    while True:
        counts = synth.token_counts(w, seed)
        off = synth.offsets_from_counts(counts)
        rows = int(off[-1])
        try:
            emb = torch.empty((rows, w.dim), dtype=dtype, pin_memory=True)
            break
        except RuntimeError as exc:
            log("cannot pin %.1f GB for %d docs (%s)" % (rows * row_bytes / 1e9, w.n_docs, str(exc).splitlines()[0]))
            if key != "c5pinned":
                # the stated size, then, in ordinary host memory: only the host can read it, so the host packs
                free = host_memory_available()
                if free is not None and rows * row_bytes + (48 << 30) > free:
                    log("only %.0f GB of host memory are free: shrinking the table by 20 %%" % (free / 1e9))
                    w = synth.scaled(w, n_docs=int(w.n_docs * 0.8))
                    continue
                emb = torch.empty((rows, w.dim), dtype=dtype)
                advise_huge_pages(emb)
                pinned, engine = False, "packed"
                break
            if w.n_docs < 200_000:
                raise
            w = synth.scaled(w, n_docs=int(w.n_docs * 0.8))        # the largest table that pins, in steps of 20 %
    if engine == "auto":
        engine = "gather"
    log("%s: %.1f GB of %s host memory for %d docs (%.1f s)" % (
        w.name, rows * row_bytes / 1e9, "pinned" if pinned else "ordinary", w.n_docs, time.time() - t_setup))
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
    table = (espn.espn_table_load_e4m3(emb, doc_scale, off, pageable=not pinned) if e4m3
             else espn.espn_table_load(emb, off, pageable=not pinned))

    cands_np = [synth.candidates(w, seed, s) for s in range(n_sets)]
    cands = [torch.from_numpy(c).to(dev) for c in cands_np]
    qs = [synth.queries(w, seed, s, device=dev) for s in range(n_sets)]
    uniq = [np.unique(c) for c in cands_np]
    uniq_rows = [int(counts[u].sum()) for u in uniq]
    cap_rows = int(max(uniq_rows) * 1.05) + 1024
    cap_docs = int(max(u.size for u in uniq) * 1.05) + 1024
    espn.espn_staging_create_ring(table, n_slots, cap_rows, cap_docs)
    out_ids = [torch.empty((w.B, w.k), dtype=torch.int64, device=dev) for _ in range(n_sets)]
    out_sc = [torch.empty((w.B, w.k), dtype=torch.float32, device=dev) for _ in range(n_sets)]
    ws_bytes = espn.espn_workspace_bytes(w.B, w.K)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    log("inputs ready: %d sets; distinct docs per batch %.1f %%, %.2f GB per batch, %d slots x %.2f GB (%.1f s)" % (
        n_sets, 100.0 * np.mean([u.size for u in uniq]) / (w.B * w.K), np.mean(uniq_rows) * row_bytes / 1e9,
        n_slots, cap_rows * row_bytes / 1e9, time.time() - t_setup))

    # reference: a plain pinned-host -> device copy of 1 GiB
    ref_rows = (1 << 30) // row_bytes
    ref_src = emb[:ref_rows] if pinned else torch.empty((ref_rows, w.dim), dtype=dtype, pin_memory=True)
    ref_dst = torch.empty_like(ref_src, device=dev)
    ref_dst.copy_(ref_src, non_blocking=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        ref_dst.copy_(ref_src, non_blocking=True)
    torch.cuda.synchronize()
    memcpy_gbs = 3 * ref_src.numel() * ref_src.element_size() / (time.perf_counter() - t0) / 1e9
    del ref_dst, ref_src

    main_s, side_s = torch.cuda.current_stream(), torch.cuda.Stream()
    st_main, st_side, h = int(main_s.cuda_stream), int(side_s.cuda_stream), table.handle
    packed = engine == "packed"
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
    # ring is filled once (every slot, untimed) before the warm-up steps, so that no timed step meets an empty slot.
    prefetch(0)
    pipeline(0, n_slots + warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pipeline(n_slots + warmup, steps)       # one prefetch and one staged re-rank per step
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    espn.espn_table_check(table)
    ms_per_step = wall * 1e3 / steps
    nxt = n_slots + warmup + steps + 1      # batches 0 .. n_slots + warmup + steps have been prefetched

    # transfer alone and scoring alone, each timed on its own stream
    legs = max(3, min(steps, 12))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for n in range(nxt, nxt + legs):
        prefetch(n)
    torch.cuda.synchronize()
    xfer_ms = (time.perf_counter() - t0) * 1e3 / legs
    nxt += legs
    # bytes that crossed PCIe, from the library's own counters: more prefetches, reading the counters after
    # each (documents another slot already holds do not cross again)
    crossed = []
    for n in range(nxt, nxt + legs):
        prefetch(n)
        crossed.append(espn.espn_staging_counters(table, n % n_slots, side_s)["pcie_bytes"])
    pcie_bytes = float(np.mean(crossed))
    distinct_bytes = float(np.mean([uniq_rows[n % n_sets] for n in range(nxt, nxt + legs)])) * row_bytes
    nxt += legs
    last = nxt - 1                          # the batch its slot still holds
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(main_s)
    for _ in range(legs):
        rerank(last)
    e1.record(main_s)
    torch.cuda.synchronize()
    score_ms = e0.elapsed_time(e1) / legs
    achieved = pcie_bytes / (xfer_ms * 1e-3) / 1e9
    log("%s: wall %.2f ms/batch; prefetch alone %.2f ms (%.2f GB over PCIe of %.2f GB distinct: %.1f GB/s; plain 1 GiB "
        "memcpy %.1f GB/s); scoring alone %.2f ms" % (w.name, ms_per_step, xfer_ms, pcie_bytes / 1e9, distinct_bytes / 1e9,
                                                      achieved, memcpy_gbs, score_ms))

    logical = float(np.mean([(row_bytes * counts[c]).sum() for c in cands_np]))
    result = {
        "metric": "candidate docs MaxSim-scored/sec", "value": w.B * w.K * steps / wall, "unit": "docs/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
        "config": {
            "workload": w.name + ("-pinned" if key == "c5pinned" else ""), "n_docs": w.n_docs, "n_docs_asked": asked_docs,
            "dim": w.dim, "rows": rows, "table_gb": rows * row_bytes / 1e9,
            "codec": w.codec, "residency": "pinned host memory" if pinned else "ordinary (pageable) host memory",
            "batch_queries": w.B, "query_tokens": w.Q,
            "candidates_per_query": w.K, "top_k": w.k, "candidate_law": "zipf(%.1f)" % w.zipf_alpha,
            "rotating_sets": n_sets, "staging_slots": n_slots, "ring_fill_steps_before_warmup": n_slots,
            "prefetch_engine": ("espn_prefetch_packed: the host packs distinct documents into pinned buffers, plain copies"
                                if packed else "espn_prefetch: gather kernel reading pinned host memory"),
            "distinct_docs_per_batch": float(np.mean([u.size for u in uniq])),
            "accumulate": "f32", "seed": seed,
        },
        "roofline": {
            "bound": "pcie", "kernel": "hipMemcpyAsync of packed buffers" if packed else "espn::staging_gather_kernel",
            "achieved": achieved, "peak": PCIE_PEAK_GBS,
            "unit": "GB/s", "frac": achieved / PCIE_PEAK_GBS, "traffic": None,
            "traffic_source": "bytes that crossed PCIe are counted by the library (rows reserved minus rows taken from "
                              "other slots, times the row bytes), not by a hardware counter",
            "algorithmic_bytes_per_launch": pcie_bytes, "kernel_ms_avg": xfer_ms,
            "plain_memcpy_h2d_gbs": memcpy_gbs,
        },
        "overlap": {"batch_ms": ms_per_step, "transfer_ms": xfer_ms, "score_ms": score_ms,
                    "batch_over_transfer": ms_per_step / xfer_ms,
                    "logical_gb_per_batch": logical / 1e9, "distinct_gb_per_batch": distinct_bytes / 1e9,
                    "pcie_gb_per_batch": pcie_bytes / 1e9},
    }
    if args.sweep_batch and not packed:
        # Eq. 4 with PCIe in the place of the SSD: the largest batch whose fetch fits a time budget.
        # The prediction uses the measured PCIe rate and the mean bytes of a query's K documents (no
        # sharing between queries, as in the paper); the measurement is the prefetch of the first b
        # queries of batch 0, which benefits from documents shared between queries.
        budget_s = args.budget_ms * 1e-3
        per_query = logical / w.B
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
            o_all = oracle.scores_e4m3(sub, doc_scale[ids], loc_off, q_np, loc_cand, threads=oracle_threads())
        else:
            o_all = oracle.scores(sub, loc_off, q_np, loc_cand, threads=oracle_threads())
        cpu_s = time.perf_counter() - t1
        m = (nxt // n_sets + 1) * n_sets        # a batch number that uses candidate set 0
        prefetch(m)
        rerank(m)
        torch.cuda.synchronize()
        g_all = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K)[:nq].cpu().numpy()
        g_ids, g_top = out_ids[0][:nq].cpu().numpy(), out_sc[0][:nq].cpu().numpy()
        worst = assert_scores_close(g_all, o_all, w.Q)
        for b in range(nq):
            assert_topk_matches(g_ids[b], g_top[b], o_all[b], cands_np[0][b], w.k, w.Q)
        result["cpu_baseline"] = {"value": nq * w.K / cpu_s, "unit": "docs/s", "cores": oracle_threads(),
                                  "kind": "oracle",
                                  "sample": "first %d queries of batch 0 (%d pairs), fp64, %.1f s wall" % (
                                      nq, nq * w.K, cpu_s)}
        result["parity"] = {"sample_pairs": nq * w.K, "worst_rel_err": worst, "status": "ok"}
        log("%s: oracle %.0f docs/s; parity ok on %d pairs" % (w.name, nq * w.K / cpu_s, nq * w.K))
    espn.espn_table_check(table)
    table.free()
    del emb, table
    release_pinned_cache(torch)
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="all",
                    choices=["all", "c1", "c2", "c3", "c4", "c5", "c5pinned", "c2p64", "c3p64", "c2e4m3", "c3e4m3", "c5e4m3"],
                    help="all (default): c4 as the headline with c3, c2, c5 and c5pinned beside it in `configs`")
    ap.add_argument("--sweep-batch", action="store_true",
                    help="c5pinned only: also time the prefetch for smaller batches and compare the batch size at which "
                         "it outgrows a time budget with Eq. 4's prediction")
    ap.add_argument("--budget-ms", type=float, default=28.0, help="time budget for --sweep-batch")
    ap.add_argument("--host-docs", type=int, default=None,
                    help="host-resident workloads: number of documents of the table (default 8.8 M = 156 GB)")
    ap.add_argument("--slots", type=int, default=2,
                    help="host-resident workloads: HBM staging slots (2 = double buffering; more slots also serve as a "
                         "cache of recently fetched documents)")
    ap.add_argument("--fetch", default="auto", choices=["auto", "streaming", "cached"],
                    help="how rows are fetched (espn_table_set_fetch); auto = the library decides from espn_table_sample")
    ap.add_argument("--engine", default="auto", choices=["auto", "gather", "packed"],
                    help="host-resident workloads: which prefetch engine fills the staging slots (espn_prefetch / "
                         "espn_prefetch_packed); auto = gather where the table is pinned, packed where it is not")
    ap.add_argument("--batch", type=int, default=None, help="override the number of queries per batch")
    ap.add_argument("--query-tokens", type=int, default=None,
                    help="override the rows per query (up to 64 run on the matrix cores; more take the plain-ALU "
                         "kernel: a comparison point, not a workload of the paper)")
    ap.add_argument("--top-k", type=int, default=None, help="override the number of ranks returned per query")
    ap.add_argument("--cand-law", default=None, choices=["uniform", "zipf"],
                    help="override the law the candidate lists are drawn from")
    ap.add_argument("--sets", type=int, default=None, help="distinct pre-drawn batches to rotate through")
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--wake-up-ms", type=float, default=None,
                    help="run the first workload's path untimed for this long before its warm-up steps (default: 30 ms "
                         "when neither --warmup nor --steps is given, so that the device is at speed; 0 when either is "
                         "given: then exactly W warm-up steps precede the K timed ones)")
    ap.add_argument("--kernels-only", action="store_true",
                    help="skip the timed region of the queue entry point (its overlapped launches blur a profiler's "
                         "per-kernel averages): only the one-stream legs run; `value` is then the one-call-per-batch rate")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-queries", type=int, default=None)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB read + 1 GiB write copy kernel (a known-size "
                         "reference for hardware byte counters when profiling)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the path has no cross-GPU step); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if int(os.environ.get("WORLD_SIZE", "1")) > 1:
        print("bench.py: launched with WORLD_SIZE > 1; only one rank on one GPU is supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2312_05417_amd import binding as espn, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(torch.device("cuda:0"))
    espn.lib()                              # fails loudly if the HIP library is not built
    seed = synth.DEFAULT_SEED if args.seed is None else args.seed
    keys = list(ALL) if args.workload == "all" else [args.workload]

    def steps_of(key):
        return args.steps if args.steps is not None else DEFAULT_STEPS[key]

    def warmup_of(key):
        if args.warmup is not None:
            return args.warmup
        steps = steps_of(key)       # short steps: as many as are timed; long ones: two fifths of them
        return steps if key in SHORT_STEPS else max(4, (steps * 2) // 5)

    wake_ms = args.wake_up_ms
    if wake_ms is None:
        wake_ms = 30.0 if (args.warmup is None and args.steps is None) else 0.0

    # ---- HBM-resident workloads: set all of them up, then their timed regions back to back
    tables, cases, results = {}, [], {}

    def guarded(key, fn):
        """Runs fn(); a failure of a configuration beside the headline is reported in its place, not raised."""
        try:
            return fn()
        except Exception as exc:        # noqa: BLE001
            if key == keys[0]:
                raise
            log("%s failed: %r" % (key, exc))
            results[key] = {"config": {"workload": key}, "error": repr(exc)}
            return None

    for key in keys:
        if key not in HOST_WORKLOADS:
            c = guarded(key, lambda: HbmCase(args, key, seed, steps_of(key), warmup_of(key), tables))
            if c is not None:
                cases.append(c)
    woken = 0
    if cases and wake_ms > 0:
        c = cases[0]
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < wake_ms * 1e-3 and woken < 20000:
            for i in range(4):
                c.rerank(woken + i)
            torch.cuda.synchronize()
            woken += 4

    def timed_part(c):
        if args.kernels_only:
            c.legs()
            c.batched = False
            c.wall, c.ms_per_step = c.sequential_wall_ms * 1e-3 * c.steps, c.sequential_wall_ms
        else:
            c.timed()
        return True

    def rest(c):
        if not args.kernels_only:
            c.legs()
        if not args.no_cpu_baseline:
            c.oracle(args.cpu_sample_queries)
        results[c.key] = c.result()
        results[c.key]["wake_up_steps"] = woken if c is cases[0] else 0
        if args.kernels_only:
            results[c.key]["config"]["entry_point"] = "espn_rerank, one call per batch on one stream (--kernels-only)"
        return True

    cases = [c for c in cases if guarded(c.key, lambda: timed_part(c))]
    for c in cases:
        guarded(c.key, lambda: rest(c))
        c.free()
    del cases
    tables.clear()
    torch.cuda.empty_cache()

    # ---- host-resident workloads, one after the other (each holds up to 156 GB of host memory).  A failure in one
    # of the configurations beside the headline is reported in its place and does not cost the line.
    for key in keys:
        if key in HOST_WORKLOADS:
            try:
                results[key] = run_host_resident(args, key, seed, steps_of(key), args.warmup if args.warmup is not None else 1)
            except Exception as exc:        # noqa: BLE001
                if key == keys[0]:
                    raise
                log("%s failed: %r" % (key, exc))
                results[key] = {"config": {"workload": key}, "error": repr(exc)}
            torch.cuda.empty_cache()

    head = results[keys[0]]
    if len(keys) > 1:
        head["configs"] = [results[key] for key in keys[1:]]
    print(json.dumps(head), flush=True)


if __name__ == "__main__":
    main()
