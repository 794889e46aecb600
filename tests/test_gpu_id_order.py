"""Batches whose lists overlap, after espn_table_sample has seen such lists: long launches take every list in the
order of its document ids (an ordering launch, then the scoring launch slice by slice) and fetch the popular
documents through the caches, the others past them.  None of it may change a score or a rank: checked against
the fp64 oracle and, bit for bit, against the same calls before the sample."""
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


def bits(t):
    return t.cpu().numpy().view(np.int32)


def ordered(table, w, B=None):
    return any("order_lists_kernel" in name for name in espn.espn_rerank_plan_kernels(table, B or w.B, w.Q, w.K, w.k))


@pytest.mark.parametrize("key,changes", [
    ("c3", dict(n_docs=6_000, B=320, K=600)),                 # 256-byte rows, 10 slices of 60: 3200 workgroups
    ("c3", dict(n_docs=6_000, B=323, K=600)),                 # a query count that is no multiple of eight
    ("c3", dict(n_docs=6_000, B=320, K=600, dim=64)),         # 128-byte rows
    ("c3", dict(n_docs=4_000, B=264, K=520, dim=256)),        # 512-byte rows
    ("c3", dict(n_docs=6_000, B=280, K=600, Q=48)),           # 48 query rows
    ("c3", dict(n_docs=9_000, B=64, K=4096, k=100)),          # the longest lists that are ordered; ranked by a sort
])
def test_lists_in_id_order_match_the_oracle_and_the_plain_order(key, changes):
    w = synth.scaled(synth.WORKLOADS[key], cand_law="zipf", **changes)
    say("id order %s d=%d B=%d K=%d k=%d" % (w.name, w.dim, w.B, w.K, w.k))
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    q, cand = synth.queries(w), synth.candidates(w)
    q_d, cand_d = q.to(DEV), torch.from_numpy(cand).to(DEV)
    assert not ordered(table, w)                              # nothing sampled yet
    plain_ids, plain_top = espn.espn_rerank(table, q_d, cand_d, w.k)
    plain_all = espn.espn_score(table, q_d, cand_d)
    torch.cuda.synchronize()
    assert espn.espn_table_sample(table, cand_d) > 0.05
    assert ordered(table, w)
    plan = espn.espn_rerank_plan(table, w.B, w.Q, w.K, w.k)
    assert plan["launches"] == 3 and plan["slices"] > 1
    ids, top = espn.espn_rerank(table, q_d, cand_d, w.k)
    # the same through the queue entry point (one batch per launch), scores left in the workspace
    ws = torch.empty(espn.espn_batches_workspace_bytes(table, 2, w.B, w.Q, w.K, w.k), dtype=torch.uint8, device=DEV)
    q_ids, q_top = espn.espn_rerank_batches(table, [q_d, q_d], [cand_d, cand_d], w.k, workspace=ws)
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    all_scores = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K)
    assert np.array_equal(bits(all_scores), bits(plain_all))
    assert torch.equal(ids, plain_ids) and np.array_equal(bits(top), bits(plain_top))
    for n in range(2):
        assert torch.equal(q_ids[n], ids) and np.array_equal(bits(q_top[n]), bits(top))
    o_all = oracle.scores(emb.numpy(), off, q.numpy(), cand)
    assert_scores_close(all_scores.cpu().numpy(), o_all, w.Q)
    for b in range(0, w.B, max(1, w.B // 40)):
        assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cand[b], w.k, w.Q)
    # the entry point without a workspace for the ordered lists scores them as they come: the same results
    n_ids = torch.empty_like(ids)
    n_top = torch.empty_like(top)
    espn.espn_rerank_noalloc(table, q_d, cand_d, w.k, n_ids, n_top)
    torch.cuda.synchronize()
    assert torch.equal(n_ids, ids) and np.array_equal(bits(n_top), bits(top))
    # a sample of lists that do not overlap switches it off again
    uniform = synth.candidates(synth.scaled(w, cand_law="uniform", n_docs=w.n_docs, K=min(w.K, 64)))
    assert espn.espn_table_sample(table, torch.from_numpy(np.ascontiguousarray(uniform[:2])).to(DEV)) < 0.05
    assert not ordered(table, w)
    table.free()


def test_a_fused_launch_of_small_batches_in_id_order():
    """Small batches that the queue entry point scores several per launch: the launch is long, so their lists are
    ordered as well (one ordering launch for all of them)."""
    w = synth.scaled(synth.WORKLOADS["c3"], cand_law="zipf", n_docs=6_000, B=48, K=600)
    n_batches = 19
    say("id order, fused: %s B=%d K=%d x %d" % (w.name, w.B, w.K, n_batches))
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    qs = [synth.queries(w, batch=n) for n in range(n_batches)]
    cands = [synth.candidates(w, batch=n) for n in range(n_batches)]
    qs_d = [q.to(DEV) for q in qs]
    cands_d = [torch.from_numpy(c).to(DEV) for c in cands]
    plain_ids, plain_top = espn.espn_rerank_batches(table, qs_d, cands_d, w.k)
    torch.cuda.synchronize()
    assert espn.espn_table_sample(table, cands_d[0]) > 0.05
    plan = espn.espn_batches_plan(table, n_batches, w.B, w.Q, w.K, w.k)
    assert plan["fuse"] == 10 and plan["launches"] == 2 and "espn::order_lists_kernel<1024, 256>" in plan["kernels"], plan
    assert not ordered(table, w)                              # one batch alone is a short launch
    ids, top = espn.espn_rerank_batches(table, qs_d, cands_d, w.k)
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    for n in range(n_batches):
        assert torch.equal(ids[n], plain_ids[n]) and np.array_equal(bits(top[n]), bits(plain_top[n])), n
    for n in (0, 9, 10, 18):
        o_all = oracle.scores(emb.numpy(), off, qs[n].numpy(), cands[n])
        for b in range(w.B):
            assert_topk_matches(ids[n][b].cpu().numpy(), top[n][b].cpu().numpy(), o_all[b], cands[n][b], w.k, w.Q)
    table.free()


def test_the_ordered_path_in_a_captured_graph():
    """The ordering launch is an ordinary kernel on the caller's stream: a captured call replays with new lists in
    the same buffers, with eager calls and synchronisations in between."""
    w = synth.scaled(synth.WORKLOADS["c3"], cand_law="zipf", n_docs=6_000, B=320, K=600)
    say("id order under graph capture")
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    sets = [(synth.queries(w, batch=r).to(DEV), torch.from_numpy(synth.candidates(w, batch=r)).to(DEV)) for r in range(2)]
    assert espn.espn_table_sample(table, sets[0][1]) > 0.05 and ordered(table, w)
    eager = [tuple(t.clone() for t in espn.espn_rerank(table, q, c, w.k)) for q, c in sets]
    torch.cuda.synchronize()
    q_buf, c_buf = sets[0][0].clone(), sets[0][1].clone()
    ids_buf = torch.empty((w.B, w.k), dtype=torch.int64, device=DEV)
    sc_buf = torch.empty((w.B, w.k), dtype=torch.float32, device=DEV)
    ws = torch.empty(espn.espn_workspace_bytes(w.B, w.K), dtype=torch.uint8, device=DEV)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        espn.espn_rerank(table, q_buf, c_buf, w.k, ids_buf, sc_buf, workspace=ws)
    for rep in range(4):
        which = rep % 2
        q_buf.copy_(sets[which][0])
        c_buf.copy_(sets[which][1])
        ids_buf.fill_(-3)
        ws.fill_(0xff)                                         # nothing may depend on what the workspace held
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(ids_buf, eager[which][0]) and np.array_equal(bits(sc_buf), bits(eager[which][1])), rep
        again = espn.espn_rerank(table, *sets[1 - which], w.k)      # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(again[0], eager[1 - which][0])
    espn.espn_table_check(table)
    del graph
    table.free()


def test_id_order_with_empty_documents_bad_ids_and_repeats():
    """An id outside the table is ordered as -1 whatever its value (so it can alias nothing), scores -inf and raises
    the flag; an empty document scores -inf; an id listed twice by a query is scored twice."""
    say("id order: empty documents, ids out of range, repeated ids")
    rng = np.random.default_rng(11)
    n_docs, B, K, k = 3_000, 288, 520, 520
    counts = rng.integers(0, 60, size=n_docs)
    counts[::5] = 0
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    emb = rng.normal(size=(int(off[-1]), 128)).astype(np.float16)
    table = espn.espn_table_load(torch.from_numpy(emb).to(DEV), off)
    q = rng.normal(size=(B, 32, 128)).astype(np.float16)
    # lists that share a popular head
    head = rng.permutation(n_docs)[:400]
    cand = np.stack([np.concatenate([rng.permutation(head)[:300], rng.permutation(n_docs)[:220]]) for _ in range(B)])
    cand = np.ascontiguousarray(cand.astype(np.int64))
    cand[3, 7] = cand[3, 400]                                  # listed twice (lists may repeat ids anyway)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    assert espn.espn_table_sample(table, cand_d) > 0.05
    assert any("order_lists_kernel" in name for name in espn.espn_rerank_plan_kernels(table, B, 32, K, k))
    ws = torch.empty(espn.espn_workspace_bytes(B, K), dtype=torch.uint8, device=DEV)
    ids, top = espn.espn_rerank(table, q_d, cand_d, k, workspace=ws)
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    got = ws[: 4 * B * K].view(torch.float32).view(B, K).cpu().numpy()
    o_all = oracle.scores(emb, off, q, cand)
    assert_scores_close(got, o_all, 32)
    assert np.array_equal(np.isneginf(got), counts[cand] == 0)
    assert got[3, 7] == got[3, 400]
    for b in range(0, B, 9):
        assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cand[b], k, 32)
    # ids out of range, among them values whose low bits would collide with positions if they were kept
    bad = cand.copy()
    bad[0, 0] = -1
    bad[5, 17] = n_docs
    bad[6, 3] = (1 << 62) + 12345
    bad[7, 249] = -(1 << 50)
    ids, top = espn.espn_rerank(table, q_d, torch.from_numpy(bad).to(DEV), k, workspace=ws)
    torch.cuda.synchronize()
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_check(table)
    assert ei.value.status == espn.ESPN_ERR_ID_RANGE
    got = ws[: 4 * B * K].view(torch.float32).view(B, K).cpu().numpy()
    expect = o_all.copy()
    for b, j in ((0, 0), (5, 17), (6, 3), (7, 249)):
        expect[b, j] = -np.inf
    assert_scores_close(got, expect, 32)
    for b, j in ((0, 0), (5, 17), (6, 3), (7, 249)):
        assert int(bad[b, j]) in ids[b].cpu().numpy().tolist()      # reported under the id the caller gave
    table.free()


def test_compressed_rows_in_id_order():
    w = synth.scaled(synth.WORKLOADS["c3e4m3"], cand_law="zipf", n_docs=6_000, B=320, K=600)
    say("id order %s (E4M3)" % w.name)
    emb, off = synth.table(w)
    codes, scale = synth.compress_e4m3(emb.to(DEV), off)
    table = espn.espn_table_load_e4m3(codes, scale, off)
    q, cand = synth.queries(w), synth.candidates(w)
    q_d, cand_d = q.to(DEV), torch.from_numpy(cand).to(DEV)
    plain_ids, plain_top = espn.espn_rerank(table, q_d, cand_d, w.k)
    torch.cuda.synchronize()
    assert espn.espn_table_sample(table, cand_d) > 0.05
    assert ordered(table, w)
    ids, top = espn.espn_rerank(table, q_d, cand_d, w.k)
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    assert torch.equal(ids, plain_ids) and np.array_equal(bits(top), bits(plain_top))
    table.free()


def test_what_is_not_ordered():
    """Short launches, lists beyond the sort's 4096 entries, lists the scoring launch ranks itself and tables that
    were never sampled run as before; partial re-ranking and a score prior never order."""
    say("id order: plans")
    w = synth.scaled(synth.WORKLOADS["c3"], cand_law="zipf", n_docs=9_000, B=320, K=600)
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    cand = synth.candidates(w)
    cand_d = torch.from_numpy(cand).to(DEV)
    names = lambda B, K, k=10: espn.espn_rerank_plan_kernels(table, B, 32, K, k)
    assert not any("order" in n for n in names(320, 600))
    assert espn.espn_table_sample(table, cand_d) > 0.05
    assert names(320, 600) == ["espn::maxsim_slice_kernel<128, 4, 4, 2, false, 2, false>", "espn::order_lists_kernel<1024, 256>",
                               "espn::topk_wave_kernel<16>"]
    assert names(256, 250)[1] == "espn::order_lists_kernel<256, 64>"
    assert names(320, 1000)[1] == "espn::order_lists_kernel<1024, 256>"
    assert names(128, 2000)[1] == "espn::order_lists_kernel<2048, 512>"
    assert names(128, 4096)[1] == "espn::order_lists_kernel<4096, 512>"
    assert not any("order" in n for n in names(128, 4097))
    assert not any("order" in n for n in names(320, 200))         # 640 workgroups: resident all at once
    assert not any("order" in n for n in names(64, 200))          # 256 workgroups: one round
    assert not any("order" in n for n in names(2048, 60))         # ranked by the scoring launch
    espn.espn_table_set_fetch(table, espn.ESPN_FETCH_STREAMING)   # streamed past the caches: nothing to gain
    assert not any("order" in n for n in names(320, 600))
    espn.espn_table_set_fetch(table, espn.ESPN_FETCH_AUTO)
    # partial re-ranking and a prior: results as before the sample
    q = synth.queries(w)
    q_d = q.to(DEV)
    prior = torch.from_numpy(np.random.default_rng(2).normal(size=cand.shape).astype(np.float32)).to(DEV)
    fresh = espn.espn_table_load(emb.to(DEV), off)
    for fn in (lambda t: espn.espn_rerank_partial(t, q_d, cand_d, 520, 50),
               lambda t: espn.espn_rerank_prior(t, q_d, cand_d, prior, 0.3, 20)):
        a, b = fn(table), fn(fresh)
        torch.cuda.synchronize()
        assert torch.equal(a[0], b[0]) and np.array_equal(bits(a[1]), bits(b[1]))
    espn.espn_table_check(table)
    table.free()
    fresh.free()
    # 64-byte rows: measured to gain nothing from it
    w32 = synth.scaled(synth.WORKLOADS["c2"], cand_law="zipf", n_docs=30_000, B=256, K=1000)
    emb, off = synth.table(w32)
    narrow = espn.espn_table_load(emb.to(DEV), off)
    assert espn.espn_table_sample(narrow, torch.from_numpy(synth.candidates(w32)).to(DEV)) > 0.05
    assert espn.espn_rerank_plan(narrow, 256, 32, 1000, 10) == {"slices": 8, "slice": 125, "launches": 2}
    narrow.free()
