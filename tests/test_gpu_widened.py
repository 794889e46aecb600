"""The steps around the core path: partial re-ranking (Sec. 4.4), score aggregation with a prior
(Sec. 3.1), merge of scored lists (Sec. 4.3) - HIP path vs the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_05417_amd import binding as espn
from paper_2312_05417_amd import synth
from tests.parity import assert_scores_close, assert_topk_matches, tol_of

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def setup(key, **changes):
    w = synth.scaled(synth.WORKLOADS[key], **changes)
    emb, off = synth.table(w)
    q, cand = synth.queries(w), synth.candidates(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    return w, emb.numpy(), off, q.numpy(), cand, table, q.to(DEV), torch.from_numpy(cand).to(DEV)


@pytest.mark.parametrize("key,changes", [("c1", {}), ("c3", dict(n_docs=4000, B=5, K=300)),
                                         ("c1", dict(dim=64, n_docs=1000, B=3, K=90))])
@pytest.mark.parametrize("R,k", [(64, 10), (16, 40), (0, 7), (1, 1), (33, 33)])
def test_partial_reranking(key, changes, R, k):
    w, emb, off, q, cand, table, q_d, cand_d = setup(key, **changes)
    R, k = min(R, w.K), min(k, w.K)
    say("partial %s d=%d K=%d R=%d k=%d" % (w.name, w.dim, w.K, R, k))
    o_ids, o_sc = oracle.rerank_partial(emb, off, q, cand, R, k)
    g_ids, g_sc = espn.espn_rerank_partial(table, q_d, cand_d, R, k)
    espn.espn_table_check(table)
    g_ids, g_sc = g_ids.cpu().numpy(), g_sc.cpu().numpy()
    head = min(R, k)
    # the tail is integer work: bit-exact; its scores are NaN on both sides
    assert np.array_equal(g_ids[:, head:], o_ids[:, head:]) and np.array_equal(g_ids[:, head:], cand[:, head:k])
    assert np.isnan(g_sc[:, head:]).all() and np.isnan(o_sc[:, head:]).all()
    if head:
        o_all = oracle.scores(emb, off, q, np.ascontiguousarray(cand[:, :R]))
        for b in range(w.B):
            assert_topk_matches(g_ids[b, :head], g_sc[b, :head], o_all[b], cand[b, :R], head, w.Q)
    # R = K is the full path
    if R == 64:
        f_ids, f_sc = espn.espn_rerank_partial(table, q_d, cand_d, w.K, k)
        r_ids, r_sc = espn.espn_rerank(table, q_d, cand_d, k)
        assert torch.equal(f_ids, r_ids) and torch.equal(f_sc, r_sc)
    table.free()


@pytest.mark.parametrize("key,changes", [("c1", {}), ("c3", dict(n_docs=4000, B=5, K=300)),
                                         ("c1", dict(dim=64, n_docs=1000, B=3, K=90))])
@pytest.mark.parametrize("alpha", [0.0, 0.25, -1.5])
def test_score_aggregation_with_a_prior(key, changes, alpha):
    w, emb, off, q, cand, table, q_d, cand_d = setup(key, **changes)
    say("prior %s d=%d alpha=%g" % (w.name, w.dim, alpha))
    prior = (np.random.default_rng(5).normal(size=cand.shape) * 4).astype(np.float32)
    o_all = oracle.scores_prior(emb, off, q, cand, prior, alpha)
    g_ids, g_top, ws = espn.espn_rerank_prior(table, q_d, cand_d, torch.from_numpy(prior).to(DEV), alpha, w.k)
    espn.espn_table_check(table)
    g_all = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K).cpu().numpy()
    # tolerance relative to the magnitudes that were added (the total itself may cancel to near zero)
    scale = np.abs(oracle.scores(emb, off, q, cand)) + abs(alpha) * np.abs(prior)
    assert np.all(np.abs(g_all - o_all) <= 1e-3 * np.maximum(scale, 1e-6 * w.Q))
    if alpha == 0.0:
        assert torch.equal(g_ids, espn.espn_rerank(table, q_d, cand_d, w.k)[0])
    for b in range(w.B):
        order = sorted(range(w.K), key=lambda j: (-o_all[b, j], int(cand[b, j])))
        gaps_ok = all(abs(o_all[b, order[r]] - o_all[b, order[r + 1]]) > 4e-3 * max(1.0, scale[b].max())
                      for r in range(w.k))
        if gaps_ok:
            assert g_ids[b].cpu().numpy().tolist() == [int(cand[b, j]) for j in order[:w.k]]
    table.free()


@pytest.mark.parametrize("ka,kb,k", [(10, 10, 10), (64, 1000, 10), (0, 5, 5), (7, 0, 3), (200, 300, 500), (3, 3, 0),
                                      (100, 156, 256), (1000, 1000, 1000), (1000, 1000, 2000), (2000, 2096, 100),
                                      (3000, 1097, 64), (1, 0, 1)])
def test_merge_of_scored_lists(ka, kb, k):
    say("merge ka=%d kb=%d k=%d" % (ka, kb, k))
    rng = np.random.default_rng(ka * 1000 + kb)
    B = 4
    n = ka + kb
    ids = np.stack([rng.permutation(10 * n + 10)[:n] for _ in range(B)]).astype(np.int64) + (1 << 34)
    sc = np.round(rng.normal(size=(B, n)), 1).astype(np.float32)          # many exact ties
    if n:
        sc[0, : min(3, n)] = -np.inf
    a_i, b_i = np.ascontiguousarray(ids[:, :ka]), np.ascontiguousarray(ids[:, ka:])
    a_s, b_s = np.ascontiguousarray(sc[:, :ka]), np.ascontiguousarray(sc[:, ka:])
    o_ids, o_sc = oracle.merge(a_i, a_s, b_i, b_s, k)
    g_ids, g_sc = espn.espn_merge_topk(torch.from_numpy(a_i).to(DEV), torch.from_numpy(a_s).to(DEV),
                                       torch.from_numpy(b_i).to(DEV), torch.from_numpy(b_s).to(DEV), k)
    assert np.array_equal(g_ids.cpu().numpy(), o_ids)                     # fp32 scores are exact: everything pinned
    assert np.array_equal(g_sc.cpu().numpy().astype(np.float64), o_sc)


def test_early_and_late_reranking_merge_to_the_full_ranking():
    # Sec. 4.3 end to end: candidates split into "prefetched" and "missed" documents, each part
    # re-ranked on its own, the two ranked lists merged: same top-k as re-ranking everything at once
    w, emb, off, q, cand, table, q_d, cand_d = setup("c3", n_docs=4000, B=6, K=200)
    say("early + late re-ranking merged")
    hit, miss = cand_d[:, :150].contiguous(), cand_d[:, 150:].contiguous()
    h_ids, h_sc = espn.espn_rerank(table, q_d, hit, w.k)
    m_ids, m_sc = espn.espn_rerank(table, q_d, miss, w.k)
    ids, sc = espn.espn_merge_topk(h_ids, h_sc, m_ids, m_sc, w.k)
    full_ids, full_sc = espn.espn_rerank(table, q_d, cand_d, w.k)
    espn.espn_table_check(table)
    assert torch.equal(ids, full_ids) and torch.equal(sc, full_sc)
    o_ids, o_top, o_all = oracle.rerank(emb, off, q, cand, w.k)
    for b in range(w.B):
        assert_topk_matches(ids[b].cpu().numpy(), sc[b].cpu().numpy(), o_all[b], cand[b], w.k, w.Q)
    table.free()


def test_batch_threshold_matches_eq4():
    for bw, budget, per_query in ((55.9e9, 0.028, 17.8e6), (3.0e9, 0.05, 2.6e6), (1.0, 1.0, 4.0)):
        assert espn.espn_batch_threshold(bw, budget, per_query) == oracle.batch_threshold(bw, budget, per_query)
    assert espn.espn_batch_threshold(1e9, 0.01, 0.0) == 0.0
