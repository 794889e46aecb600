"""The workloads at their full sizes, in the launch configuration bench.py times (same entry point,
same batch shapes): sampled queries against the oracle, plus properties that hold for every output."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_05417_amd import binding as espn
from paper_2312_05417_amd import synth
from tests.parity import assert_scores_close, assert_topk_matches

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def check_everything_cheap(scores, ids, top, cand, w):
    """Properties that need no oracle: bounds for unit vectors, sorted output, ids from the list,
    the first rank is the maximum, returned scores are the scores of the returned ids."""
    assert np.isfinite(scores).all()
    assert np.abs(scores).max() <= w.Q * (1 + 4e-3)             # Cauchy-Schwarz, rows are unit up to fp16 rounding
    assert np.all(np.diff(top, axis=1) <= 0)
    assert np.array_equal(top[:, 0], scores.max(axis=1))
    order = np.argsort(cand, axis=1)
    pos = np.take_along_axis(order, np.stack([np.searchsorted(cand[b][order[b]], ids[b]) for b in range(w.B)]), 1)
    assert np.array_equal(np.take_along_axis(cand, pos, 1), ids)
    assert np.array_equal(np.take_along_axis(scores, pos, 1), top)
    kth = top[:, -1:]
    assert np.all((scores > kth).sum(axis=1) <= w.k - 1)


def spread_sample(B, n):
    """n query indices spread over the batch, always with the first and last eight (the ends of the grid, and
    every residue modulo 8: workgroups are renumbered per XCD by that residue)."""
    ends = np.concatenate([np.arange(min(8, B)), np.arange(max(0, B - 8), B)])
    return np.unique(np.concatenate([ends, np.linspace(0, B - 1, n).astype(int)]))


@pytest.mark.parametrize("key,sample", [("c2", 64), ("c3", 96), ("c4", 128)])
def test_full_size_hbm_workloads(key, sample):
    """Through espn_rerank_batches, the call bench.py times: three batches in flight on the library's streams
    (the first is checked against the oracle, the other two are the same batch again and must give the same
    bits), and through espn_rerank, which must agree bit for bit."""
    w = synth.WORKLOADS[key]
    say("%s full size: N=%d d=%d B=%d K=%d" % (w.name, w.n_docs, w.dim, w.B, w.K))
    emb, off = synth.table(w, device=DEV)
    table = espn.espn_table_load(emb, off)
    cand = synth.candidates(w)
    cand_d = torch.from_numpy(cand).to(DEV)
    q = synth.queries(w, device=DEV)
    # as bench.py does once per workload: the library is shown a batch's lists (c4's overlap, so its batches are
    # scored in id order, popular documents through the caches; the others' do not)
    espn.espn_table_sample(table, cand_d)
    kernels = espn.espn_rerank_plan_kernels(table, w.B, w.Q, w.K, w.k)
    assert any("order_lists_kernel" in name for name in kernels) == (key == "c4"), kernels
    part = espn.espn_workspace_bytes(w.B, w.K)
    ws = torch.empty(espn.espn_batches_workspace_bytes(table, 3, w.B, w.Q, w.K, w.k), dtype=torch.uint8, device=DEV)
    many_ids, many_top = espn.espn_rerank_batches(table, [q] * 3, [cand_d] * 3, w.k, workspace=ws)
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    first = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K)       # a queue of three leaves batch 0's scores here
    scores = first.cpu().numpy()
    for l in (1, 2):
        assert torch.equal(many_ids[l], many_ids[0]) and torch.equal(many_top[l].view(torch.int32), many_top[0].view(torch.int32))
    one_ids, one_top = espn.espn_rerank(table, q, cand_d, w.k, workspace=ws[:part])
    assert torch.equal(one_ids, many_ids[0]) and torch.equal(one_top.view(torch.int32), many_top[0].view(torch.int32))
    assert torch.equal(first.view(torch.int32), torch.from_numpy(scores).to(DEV).view(torch.int32))
    ids, top = many_ids[0].cpu().numpy(), many_top[0].cpu().numpy()
    check_everything_cheap(scores, ids, top, cand, w)
    # oracle on a sample of queries spread over the batch (its ends, every residue modulo 8, and in between)
    pick = spread_sample(w.B, sample)
    assert pick.size >= min(sample, w.B) and set(pick % 8) == set(range(8))
    sub, loc_off, loc_cand, _ = synth.subtable(emb, off, cand[pick])
    o_ids, o_top, o_all = oracle.rerank(sub, loc_off, q[torch.from_numpy(pick).to(DEV)].cpu().numpy(), loc_cand, w.k)
    worst = assert_scores_close(scores[pick], o_all, w.Q)
    for j, b in enumerate(pick):
        assert_topk_matches(ids[b], top[b], o_all[j], cand[b], w.k, w.Q)
    say("%d sampled pairs match, worst relative error %.2e" % (pick.size * w.K, worst))
    table.free()


def test_host_resident_workload_at_full_batch_shape():
    # the c5 batch shape (1024 x 1000, Zipf) on a table scaled to what a test may pin (3.5 GB)
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=200_000)
    say("%s: N=%d (scaled) B=%d K=%d" % (w.name, w.n_docs, w.B, w.K))
    off = synth.offsets_from_counts(synth.token_counts(w))
    emb = torch.empty((int(off[-1]), w.dim), dtype=torch.float16, pin_memory=True)
    synth.table(w, device=DEV, out=emb)
    torch.cuda.synchronize()
    table = espn.espn_table_load(emb, off)
    cands = [synth.candidates(w, batch=n) for n in range(3)]
    cands_d = [torch.from_numpy(c).to(DEV) for c in cands]
    qs = [synth.queries(w, batch=n, device=DEV) for n in range(3)]
    rows = max(int((off[u + 1] - off[u]).sum()) for u in (np.unique(c) for c in cands))
    espn.espn_staging_create(table, rows + 16, w.n_docs)
    side = torch.cuda.Stream()
    outs = []
    espn.espn_prefetch(table, cands_d[0], 0, side)
    for n in range(3):
        if n < 2:
            espn.espn_prefetch(table, cands_d[n + 1], (n + 1) % 2, side)
        outs.append(espn.espn_rerank_staged(table, n % 2, qs[n], cands_d[n], w.k))
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    for n in range(3):
        ids, top, ws = outs[n]
        scores = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K).cpu().numpy()
        ids, top = ids.cpu().numpy(), top.cpu().numpy()
        check_everything_cheap(scores, ids, top, cands[n], w)
        pick = spread_sample(w.B, 8)                 # 16 to 24 queries per batch
        sub, loc_off, loc_cand, _ = synth.subtable(emb, off, cands[n][pick])
        o_ids, o_top, o_all = oracle.rerank(sub, loc_off, qs[n][torch.from_numpy(pick).to(DEV)].cpu().numpy(),
                                            loc_cand, w.k)
        assert_scores_close(scores[pick], o_all, w.Q)
        for j, b in enumerate(pick):
            assert_topk_matches(ids[b], top[b], o_all[j], cands[n][b], w.k, w.Q)
    c = espn.espn_staging_counters(table, 0)
    u = np.unique(cands[2])
    assert c["distinct_docs"] == u.size and c["rows"] == int((off[u + 1] - off[u]).sum())
    table.free()
