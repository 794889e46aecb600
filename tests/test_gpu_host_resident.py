"""Host-resident table: prefetch into HBM staging slots + staged re-rank, against the fp64 oracle."""
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


def host_table(w, seed=synth.DEFAULT_SEED):
    off = synth.offsets_from_counts(synth.token_counts(w, seed))
    pinned = torch.empty((int(off[-1]), w.dim), dtype=torch.float16, pin_memory=True)
    synth.table(w, seed, device="cpu", out=pinned)
    return pinned, off


def scores_of(ws, B, K):
    return ws[: 4 * B * K].view(torch.float32).view(B, K).cpu().numpy()


@pytest.mark.parametrize("key,changes", [
    ("c5", dict(n_docs=20_000, B=16, K=300)),                  # d=128, Zipf: heavy repeats across queries
    ("c2", dict(n_docs=5_000, B=8, K=200, cand_law="zipf")),   # d=32
    ("c1", dict(dim=64, n_docs=2_000, B=4, K=50)),             # generic kernel
])
def test_double_buffered_batches_match_the_oracle(key, changes):
    w = synth.scaled(synth.WORKLOADS[key], **changes)
    say("host-resident %s d=%d N=%d B=%d K=%d" % (w.name, w.dim, w.n_docs, w.B, w.K))
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    assert table.info()["residency"] == espn.ESPN_RESIDENT_HOST_PINNED
    espn.espn_staging_create(table, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    n_batches = 5
    cands = [synth.candidates(w, batch=n) for n in range(n_batches)]
    cands_d = [torch.from_numpy(c).to(DEV) for c in cands]
    qs = [synth.queries(w, batch=n) for n in range(n_batches)]
    qs_d = [x.to(DEV) for x in qs]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    outs = []
    espn.espn_prefetch(table, cands_d[0], 0, side)
    for n in range(n_batches):
        if n + 1 < n_batches:
            espn.espn_prefetch(table, cands_d[n + 1], (n + 1) % 2, side)
        outs.append(espn.espn_rerank_staged(table, n % 2, qs_d[n], cands_d[n], w.k, stream=main))
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    e = emb.numpy()
    for n in range(n_batches):
        ids, top, ws = outs[n]
        o_ids, o_top, o_all = oracle.rerank(e, off, qs[n].numpy(), cands[n], w.k)
        assert_scores_close(scores_of(ws, w.B, w.K), o_all, w.Q, "batch %d" % n)
        for b in range(w.B):
            assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cands[n][b], w.k, w.Q)
    # what the last prefetches moved: exactly the distinct documents of their batches, each once, and
    # over PCIe only those that the batch before (which sat in the other slot) had not brought in already
    for n in (n_batches - 2, n_batches - 1):
        c = espn.espn_staging_counters(table, n % 2)
        uniq = np.unique(cands[n])
        rows = int((off[uniq + 1] - off[uniq]).sum())
        fresh = np.setdiff1d(uniq, cands[n - 1])
        fresh_rows = int((off[fresh + 1] - off[fresh]).sum())
        assert c["distinct_docs"] == uniq.size and c["rows"] == rows
        assert c["pcie_bytes"] == fresh_rows * w.dim * 2
        assert c["distinct_docs"] < cands[n].size          # the candidate law repeats documents
        if w.cand_law == "zipf":
            assert fresh_rows < rows                        # ... also from batch to batch
    table.free()


def test_documents_are_handed_from_slot_to_slot():
    """A chain of batches in which every document of batch n+1 is also in batch n: after the first
    prefetch nothing crosses PCIe any more, and the scores stay those of the table."""
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=6_000, B=6, K=150)
    say("slot-to-slot hand-over %s" % w.name)
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    espn.espn_staging_create(table, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    base = synth.candidates(w, batch=0)
    rng = np.random.default_rng(2)
    chain = [base]
    for n in range(1, 4):                     # each batch re-draws its lists from the previous batch's documents
        pool = np.unique(chain[-1])
        chain.append(np.stack([rng.permutation(pool)[:w.K] for _ in range(w.B)]).astype(np.int64))
    q = synth.queries(w)
    q_d = q.to(DEV)
    e = emb.numpy()
    for n, cand in enumerate(chain):
        cand_d = torch.from_numpy(cand).to(DEV)
        espn.espn_prefetch(table, cand_d, n % 2)
        ids, top, ws = espn.espn_rerank_staged(table, n % 2, q_d, cand_d, w.k)
        c = espn.espn_staging_counters(table, n % 2)
        uniq = np.unique(cand)
        rows = int((off[uniq + 1] - off[uniq]).sum())
        assert c["distinct_docs"] == uniq.size and c["rows"] == rows
        assert c["pcie_bytes"] == (rows * w.dim * 2 if n == 0 else 0), (n, c)
        o_all = oracle.scores(e, off, q.numpy(), cand)
        assert_scores_close(scores_of(ws, w.B, w.K), o_all, w.Q, "batch %d" % n)
    # slots too small for the batch: whatever fitted the other slot may be taken from it, whatever did
    # not is read from the host again; every document the second slot holds must score right either way
    cand = chain[0]
    cand_d = torch.from_numpy(cand).to(DEV)
    uniq = np.unique(cand)
    rows = int((off[uniq + 1] - off[uniq]).sum())
    espn.espn_staging_create(table, capacity_rows=rows // 2, capacity_docs=w.n_docs)
    espn.espn_prefetch(table, cand_d, 0)
    espn.espn_prefetch(table, cand_d, 1)
    ids, top, ws = espn.espn_rerank_staged(table, 1, q_d, cand_d, w.k)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_check(table)
    assert ei.value.status in (espn.ESPN_ERR_NOMEM, espn.ESPN_ERR_SHAPE)
    g = scores_of(ws, w.B, w.K)
    o_all = oracle.scores(e, off, q.numpy(), cand)
    held = ~np.isneginf(g)
    assert held.any() and (~held).any()
    assert_scores_close(g[held], o_all[held], w.Q)
    table.free()


def test_a_ring_of_slots_serves_as_a_cache_of_recent_documents():
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=30_000, B=12, K=250)
    n_slots, n_batches = 4, 9
    say("ring of %d slots, %s" % (n_slots, w.name))
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    espn.espn_staging_create_ring(table, n_slots, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    with pytest.raises(espn.EspnError):
        espn.espn_prefetch(table, torch.zeros((1, 1), dtype=torch.int64, device=DEV), n_slots)
    cands = [synth.candidates(w, batch=n) for n in range(n_batches)]
    cands_d = [torch.from_numpy(c).to(DEV) for c in cands]
    qs = [synth.queries(w, batch=n) for n in range(n_batches)]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    outs, moved = [], []
    espn.espn_prefetch(table, cands_d[0], 0, side)
    for n in range(n_batches):
        if n + 1 < n_batches:
            espn.espn_prefetch(table, cands_d[n + 1], (n + 1) % n_slots, side)
        outs.append(espn.espn_rerank_staged(table, n % n_slots, qs[n].to(DEV), cands_d[n], w.k, stream=main))
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    e = emb.numpy()
    for n in range(n_batches):
        ids, top, ws = outs[n]
        o_ids, o_top, o_all = oracle.rerank(e, off, qs[n].numpy(), cands[n], w.k)
        assert_scores_close(scores_of(ws, w.B, w.K), o_all, w.Q, "batch %d" % n)
        for b in range(w.B):
            assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cands[n][b], w.k, w.Q)
    # the last prefetches: over PCIe came only what none of the three batches before had brought in
    for n in range(n_batches - n_slots + 1, n_batches):
        c = espn.espn_staging_counters(table, n % n_slots)
        uniq = np.unique(cands[n])
        held = np.unique(np.concatenate([cands[m].ravel() for m in range(n - n_slots + 1, n)]))
        fresh = np.setdiff1d(uniq, held)
        assert c["distinct_docs"] == uniq.size
        assert c["pcie_bytes"] == int((off[fresh + 1] - off[fresh]).sum()) * w.dim * 2
        one_back = np.setdiff1d(uniq, cands[n - 1])
        assert fresh.size < one_back.size          # more slots, more hits
    table.free()


def test_hbm_entry_points_refuse_a_host_table():
    w = synth.scaled(synth.WORKLOADS["c1"], n_docs=500, B=2, K=20)
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    q, cand = synth.queries(w).to(DEV), torch.from_numpy(synth.candidates(w)).to(DEV)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_rerank(table, q, cand, 5)
    assert ei.value.status == espn.ESPN_ERR_UNSUPPORTED
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch(table, cand, 0)                  # no staging yet
    assert ei.value.status == espn.ESPN_ERR_ARG
    espn.espn_staging_create(table, 100, 10)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch(table, cand, 2)
    assert ei.value.status == espn.ESPN_ERR_ARG
    for bad in (1, 9):
        with pytest.raises(espn.EspnError) as ei:
            espn.espn_staging_create_ring(table, bad, 100, 10)
        assert ei.value.status == espn.ESPN_ERR_ARG


def test_an_hbm_table_can_be_staged_too_as_a_standalone_gather():
    w = synth.scaled(synth.WORKLOADS["c4"], n_docs=3_000, B=8, K=100)
    say("stand-alone gather HBM -> HBM")
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    cand = synth.candidates(w)
    cand_d, q = torch.from_numpy(cand).to(DEV), synth.queries(w)
    espn.espn_staging_create(table, int(off[-1]), w.n_docs)
    espn.espn_prefetch(table, cand_d, 0)
    ids, top, ws = espn.espn_rerank_staged(table, 0, q.to(DEV), cand_d, w.k)
    ids2, top2 = espn.espn_rerank(table, q.to(DEV), cand_d, w.k)
    espn.espn_table_check(table)
    assert torch.equal(ids, ids2) and torch.equal(top, top2)          # same rows, same kernel: bit-identical
    o = oracle.scores(emb.numpy(), off, q.numpy(), cand)
    assert_scores_close(scores_of(ws, w.B, w.K), o, w.Q)
    u = np.unique(cand)
    assert espn.espn_staging_counters(table, 0)["distinct_docs"] == u.size


def test_slot_overflow_and_foreign_candidates_are_flagged_not_read():
    w = synth.scaled(synth.WORKLOADS["c1"], n_docs=500, B=4, K=40)
    say("staging overflow / not staged")
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    cand = synth.candidates(w)
    cand_d = torch.from_numpy(cand).to(DEV)
    q = synth.queries(w)
    q_d = q.to(DEV)
    # slot too small for the batch: flagged, the documents that did not fit score -inf, the rest are right
    espn.espn_staging_create(table, capacity_rows=600, capacity_docs=500)
    espn.espn_prefetch(table, cand_d, 0)
    ids, top, ws = espn.espn_rerank_staged(table, 0, q_d, cand_d, w.k)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_check(table)
    assert ei.value.status in (espn.ESPN_ERR_NOMEM, espn.ESPN_ERR_SHAPE)
    g = scores_of(ws, w.B, w.K)
    o = oracle.scores(emb.numpy(), off, q.numpy(), cand)
    held = ~np.isneginf(g)
    assert held.any() and (~held).any()
    assert_scores_close(g[held], o[held], w.Q)
    # big enough slot, but the re-rank names documents that were not prefetched
    espn.espn_staging_create(table, capacity_rows=int(off[-1]), capacity_docs=500)
    part = cand_d[:, :20].contiguous()
    espn.espn_prefetch(table, part, 1)
    ids, top, ws = espn.espn_rerank_staged(table, 1, q_d, cand_d, w.k)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_check(table)
    assert ei.value.status == espn.ESPN_ERR_SHAPE
    g = scores_of(ws, w.B, w.K)
    staged = np.isin(cand, cand[:, :20])
    assert np.all(np.isneginf(g[~staged]))
    assert_scores_close(g[staged], o[staged], w.Q)
    table.free()


@pytest.mark.parametrize("key,changes", [
    ("c5", dict(n_docs=20_000, B=16, K=300)),                  # d=128, Zipf: heavy repeats across queries
    ("c2", dict(n_docs=5_000, B=8, K=200, cand_law="zipf")),   # d=32
    ("c1", dict(dim=40, n_docs=2_000, B=4, K=50)),             # generic kernel
])
def test_the_packing_engine_fills_a_slot_like_the_gather_engine(key, changes):
    """espn_prefetch_packed (host finds the distinct documents, packs rows into pinned buffers, plain
    copies) against the oracle, and bit for bit against a slot filled by espn_prefetch; the two
    engines alternate in one pipeline on two streams."""
    w = synth.scaled(synth.WORKLOADS[key], **changes)
    say("packing engine %s d=%d N=%d B=%d K=%d" % (w.name, w.dim, w.n_docs, w.B, w.K))
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    espn.espn_staging_create(table, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    n_batches = 6
    cands = [synth.candidates(w, batch=n) for n in range(n_batches)]
    cands_h = [torch.from_numpy(c) for c in cands]
    cands_d = [c.to(DEV) for c in cands_h]
    qs = [synth.queries(w, batch=n) for n in range(n_batches)]
    qs_d = [x.to(DEV) for x in qs]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()

    def prefetch(n):
        if n % 3 == 2:                                       # every third batch through the GPU engine
            espn.espn_prefetch(table, cands_d[n], n % 2, side)
        else:
            espn.espn_prefetch_packed(table, cands_h[n], n % 2, side)

    outs = []
    prefetch(0)
    for n in range(n_batches):
        if n + 1 < n_batches:
            prefetch(n + 1)
        outs.append(espn.espn_rerank_staged(table, n % 2, qs_d[n], cands_d[n], w.k, stream=main))
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    e = emb.numpy()
    for n in range(n_batches):
        ids, top, ws = outs[n]
        o_ids, o_top, o_all = oracle.rerank(e, off, qs[n].numpy(), cands[n], w.k)
        assert_scores_close(scores_of(ws, w.B, w.K), o_all, w.Q, "batch %d" % n)
        for b in range(w.B):
            assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cands[n][b], w.k, w.Q)
    # the same batch through both engines: identical scores and ranks; the packing engine moves every
    # distinct document over PCIe (it takes nothing from the other slot)
    n = n_batches - 1
    espn.espn_prefetch(table, cands_d[n], 0)
    a_ids, a_top, a_ws = espn.espn_rerank_staged(table, 0, qs_d[n], cands_d[n], w.k)
    a_scores = scores_of(a_ws, w.B, w.K)
    espn.espn_prefetch_packed(table, cands_h[n], 1)
    b_ids, b_top, b_ws = espn.espn_rerank_staged(table, 1, qs_d[n], cands_d[n], w.k)
    assert np.array_equal(a_scores.view(np.int32), scores_of(b_ws, w.B, w.K).view(np.int32))
    assert torch.equal(a_ids, b_ids) and torch.equal(a_top.view(torch.int32), b_top.view(torch.int32))
    c = espn.espn_staging_counters(table, 1)
    uniq = np.unique(cands[n])
    rows = int((off[uniq + 1] - off[uniq]).sum())
    assert c["distinct_docs"] == uniq.size and c["rows"] == rows and c["pcie_bytes"] == rows * w.dim * 2
    espn.espn_table_check(table)
    table.free()


@pytest.mark.parametrize("n_slots,codec", [(2, "f16"), (3, "f16"), (4, "e4m3")])
def test_the_packing_engine_takes_from_other_slots_what_they_hold(n_slots, codec):
    """The host remembers where its packed prefetches put every document: what another slot of the ring still holds
    is copied from there, only the rest is packed and sent.  Double-buffered on two streams, every batch against the
    oracle and bit for bit against a slot that the gather engine filled."""
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=20_000, B=16, K=300)
    say("packing engine, hand-over in a ring of %d (%s)" % (n_slots, codec))
    emb, off = host_table(w)
    if codec == "e4m3":
        codes, scale = synth.compress_e4m3(emb, off)
        pinned = torch.empty(codes.shape, dtype=torch.uint8, pin_memory=True)
        pinned.copy_(codes)
        table = espn.espn_table_load_e4m3(pinned, scale, off)
        reference = lambda q, cand: oracle.scores_e4m3(codes.numpy(), scale, off, q, cand)
    else:
        table = espn.espn_table_load(emb, off)
        reference = lambda q, cand: oracle.scores(emb.numpy(), off, q, cand)
    espn.espn_staging_create_ring(table, n_slots, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    n_batches = 7
    cands = [synth.candidates(w, batch=n) for n in range(n_batches)]
    cands_h = [torch.from_numpy(c) for c in cands]
    cands_d = [c.to(DEV) for c in cands_h]
    qs = [synth.queries(w, batch=n) for n in range(n_batches)]
    main, side = torch.cuda.current_stream(), torch.cuda.Stream()
    outs = []
    espn.espn_prefetch_packed(table, cands_h[0], 0, side)
    for n in range(n_batches):
        if n + 1 < n_batches:
            espn.espn_prefetch_packed(table, cands_h[n + 1], (n + 1) % n_slots, side)
        outs.append(espn.espn_rerank_staged(table, n % n_slots, qs[n].to(DEV), cands_d[n], w.k, stream=main))
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    for n in range(n_batches):
        ids, top, ws = outs[n]
        o_all = reference(qs[n].numpy(), cands[n])
        assert_scores_close(scores_of(ws, w.B, w.K), o_all, w.Q, "batch %d" % n)
        for b in range(w.B):
            assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cands[n][b], w.k, w.Q)
    # most of the last batch was taken from the other slots
    n = n_batches - 1
    c = espn.espn_staging_counters(table, n % n_slots)
    uniq = np.unique(cands[n])
    assert c["distinct_docs"] == uniq.size
    assert 0 < c["pcie_bytes"] < int((off[uniq + 1] - off[uniq]).sum()) * w.dim * (1 if codec == "e4m3" else 2)
    # the same batches from a slot filled by the gather engine: the same bits
    for n in (n_batches - 1, n_batches - 2):
        spare = (n_batches + 1) % n_slots
        espn.espn_prefetch(table, cands_d[n], spare)
        g_ids, g_top, g_ws = espn.espn_rerank_staged(table, spare, qs[n].to(DEV), cands_d[n], w.k)
        assert torch.equal(g_ids, outs[n][0]) and torch.equal(g_top.view(torch.int32), outs[n][1].view(torch.int32))
        assert np.array_equal(scores_of(g_ws, w.B, w.K).view(np.int32), scores_of(outs[n][2], w.B, w.K).view(np.int32))
    espn.espn_table_check(table)
    table.free()


def test_the_packing_engine_counts_what_it_sends():
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=20_000, B=16, K=300)
    say("packing engine: bytes sent with and without hand-over")
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    n_slots = 3
    espn.espn_staging_create_ring(table, n_slots, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    cands = [synth.candidates(w, batch=n) for n in range(6)]
    rows_of = lambda ids: int((off[ids + 1] - off[ids]).sum())
    for n in range(5):
        espn.espn_prefetch_packed(table, torch.from_numpy(cands[n]), n % n_slots)
        c = espn.espn_staging_counters(table, n % n_slots)
        uniq = np.unique(cands[n])
        held = np.unique(np.concatenate([cands[m].ravel() for m in range(max(0, n - n_slots + 1), n)])) if n else np.empty(0, np.int64)
        fresh = np.setdiff1d(uniq, held)
        assert c["distinct_docs"] == uniq.size and c["rows"] == rows_of(uniq), n
        assert c["pcie_bytes"] == rows_of(fresh) * w.dim * 2, n
        if n >= 1:
            assert fresh.size < uniq.size
    # the gather engine refills slot 1 (batches 1 and 4 went there): the host's notes about it no longer hold
    espn.espn_prefetch(table, torch.from_numpy(cands[5]).to(DEV), 1)
    espn.espn_prefetch_packed(table, torch.from_numpy(cands[5]), 2)
    c = espn.espn_staging_counters(table, 2)
    uniq = np.unique(cands[5])
    # slot 0 still holds batch 3; slot 1 is not trusted, and the host notes only the newest holder of a document
    fresh = np.setdiff1d(uniq, np.setdiff1d(np.unique(cands[3]), np.unique(cands[4])))
    assert c["pcie_bytes"] == rows_of(fresh) * w.dim * 2
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    table.free()


def test_the_packing_engine_reports_its_errors_before_enqueuing_anything():
    w = synth.scaled(synth.WORKLOADS["c1"], n_docs=500, B=4, K=40)
    say("packing engine: errors")
    emb, off = host_table(w)
    table = espn.espn_table_load(emb, off)
    cand = synth.candidates(w)
    cand_h = torch.from_numpy(cand)
    q_d = synth.queries(w).to(DEV)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch_packed(table, cand_h, 0)          # no staging yet
    assert ei.value.status == espn.ESPN_ERR_ARG
    espn.espn_staging_create(table, capacity_rows=int(off[-1]), capacity_docs=500)
    bad = cand_h.clone()
    bad[2, 7] = 500                                          # one past the last document
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch_packed(table, bad, 0)
    assert ei.value.status == espn.ESPN_ERR_ID_RANGE
    bad[2, 7] = -1
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch_packed(table, bad, 0)
    assert ei.value.status == espn.ESPN_ERR_ID_RANGE
    with pytest.raises(ValueError):
        espn.espn_prefetch_packed(table, cand_h.to(DEV), 0)  # a device tensor is not what it takes
    # a refused call leaves the engine usable: the next one works and scores right
    espn.espn_prefetch_packed(table, cand_h, 0)
    ids, top, ws = espn.espn_rerank_staged(table, 0, q_d, cand_h.to(DEV), w.k)
    o = oracle.scores(emb.numpy(), off, synth.queries(w).numpy(), cand)
    assert_scores_close(scores_of(ws, w.B, w.K), o, w.Q)
    espn.espn_table_check(table)
    # a slot too small for the batch is refused on the host
    espn.espn_staging_create(table, capacity_rows=600, capacity_docs=500)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch_packed(table, cand_h, 0)
    assert ei.value.status == espn.ESPN_ERR_NOMEM
    espn.espn_staging_create(table, capacity_rows=int(off[-1]), capacity_docs=3)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch_packed(table, cand_h, 0)
    assert ei.value.status == espn.ESPN_ERR_NOMEM
    table.free()
    # an HBM-resident table has no host copy to pack from
    emb_d, off2 = synth.table(w)
    hbm = espn.espn_table_load(emb_d.to(DEV), off2)
    espn.espn_staging_create(hbm, int(off2[-1]), w.n_docs)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch_packed(hbm, cand_h, 0)
    assert ei.value.status == espn.ESPN_ERR_UNSUPPORTED
    hbm.free()


def test_a_table_in_ordinary_host_memory_is_served_by_the_packing_engine():
    """ESPN_RESIDENT_HOST: the table is not pinned, so only the host reads it (espn_prefetch_packed packs its
    documents into the library's own pinned buffers); double-buffered batches against the oracle, bit for bit
    against the same table pinned, and the gather engine (which would need the device to read the table) refused."""
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=30_000, B=24, K=400)
    say("pageable host table d=%d N=%d B=%d K=%d" % (w.dim, w.n_docs, w.B, w.K))
    emb, off = synth.table(w)                                  # ordinary host memory
    assert not emb.is_pinned()
    with pytest.raises(TypeError):
        espn.espn_table_load(emb, off)                         # the binding wants to be told
    table = espn.espn_table_load(emb, off, pageable=True)
    assert table.info()["residency"] == espn.ESPN_RESIDENT_HOST
    pinned_emb, _ = host_table(w)
    pinned = espn.espn_table_load(pinned_emb, off)
    for t in (table, pinned):
        espn.espn_staging_create(t, capacity_rows=int(off[-1]), capacity_docs=w.n_docs)
    n_batches = 4
    cands = [synth.candidates(w, batch=n) for n in range(n_batches)]
    cands_h = [torch.from_numpy(c) for c in cands]
    cands_d = [c.to(DEV) for c in cands_h]
    qs = [synth.queries(w, batch=n) for n in range(n_batches)]
    qs_d = [x.to(DEV) for x in qs]
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_prefetch(table, cands_d[0], 0)
    assert ei.value.status == espn.ESPN_ERR_UNSUPPORTED
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_rerank(table, qs_d[0], cands_d[0], w.k)
    assert ei.value.status == espn.ESPN_ERR_UNSUPPORTED
    side = torch.cuda.Stream()
    outs = []
    espn.espn_prefetch_packed(table, cands_h[0], 0, side)
    for n in range(n_batches):
        outs.append(espn.espn_rerank_staged(table, n % 2, qs_d[n], cands_d[n], w.k))
        if n + 1 < n_batches:
            espn.espn_prefetch_packed(table, cands_h[n + 1], (n + 1) % 2, side)
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    e = emb.numpy()
    for n in range(n_batches):
        ids, top, ws = outs[n]
        o_ids, o_top, o_all = oracle.rerank(e, off, qs[n].numpy(), cands[n], w.k)
        assert_scores_close(scores_of(ws, w.B, w.K), o_all, w.Q, "batch %d" % n)
        for b in range(w.B):
            assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cands[n][b], w.k, w.Q)
        espn.espn_prefetch(pinned, cands_d[n], 0)
        p_ids, p_top, p_ws = espn.espn_rerank_staged(pinned, 0, qs_d[n], cands_d[n], w.k)
        assert torch.equal(p_ids, ids) and torch.equal(p_top.view(torch.int32), top.view(torch.int32))
        assert np.array_equal(scores_of(p_ws, w.B, w.K).view(np.int32), scores_of(ws, w.B, w.K).view(np.int32))
    # what the batch before left in the other slot is copied from there, the rest crosses PCIe
    c = espn.espn_staging_counters(table, (n_batches - 1) % 2)
    uniq = np.unique(cands[-1])
    rows = int((off[uniq + 1] - off[uniq]).sum())
    fresh = np.setdiff1d(uniq, np.unique(cands[-2]))
    assert 0 < fresh.size < uniq.size
    sent = int((off[fresh + 1] - off[fresh]).sum())
    assert c["distinct_docs"] == uniq.size and c["rows"] == rows and c["pcie_bytes"] == sent * w.dim * 2
    espn.espn_table_check(pinned)
    pinned.free()
    table.free()
