"""Batches whose candidate lists are short and whose queries are many are scored AND ranked by one
launch of the scoring kernel (espn_rerank_plan says which).  That path is checked here against the
fp64 oracle and, bit for bit, against the two-launch path (espn_score + espn_topk)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_05417_amd import binding as espn
from tests.parity import assert_scores_close, assert_topk_matches
from tests.test_gpu_parity import random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
B_MANY = 1100          # more queries than workgroups the device holds at once: one slice per query


def say(msg):
    print("[case] " + msg, flush=True)


def both_paths(emb, off, q, cand, k, expect_launches):
    emb_d = torch.from_numpy(np.ascontiguousarray(emb)).to(DEV)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    table = espn.espn_table_load(emb_d, off)
    plan = espn.espn_rerank_plan(table, q.shape[0], q.shape[1], cand.shape[1], k)
    assert plan["launches"] == expect_launches, plan
    ids1, sc1 = espn.espn_rerank(table, q_d, cand_d, k)
    all2 = espn.espn_score(table, q_d, cand_d)
    ids2, sc2 = espn.espn_topk(all2, cand_d, k)
    espn.espn_table_check(table)
    assert torch.equal(ids1, ids2), "ids differ between the one-launch and the two-launch path"
    assert torch.equal(sc1.view(torch.int32), sc2.view(torch.int32)), "scores differ bitwise"
    table.free()
    return ids1.cpu().numpy(), sc1.cpu().numpy(), all2.cpu().numpy()


@pytest.mark.parametrize("d", [32, 128])
@pytest.mark.parametrize("K,k", [(1, 1), (40, 10), (64, 64), (65, 7), (200, 10), (256, 256)])
def test_one_launch_path_matches_oracle_and_two_launch_path(d, K, k):
    say("one launch: d=%d B=%d K=%d k=%d" % (d, B_MANY, K, k))
    emb, off, q, cand = random_problem(31 * K + d, max(K, 300), d, B_MANY, 32, K, 1, 40)
    g_ids, g_sc, g_all = both_paths(emb, off, q, cand, k, expect_launches=1)
    # the oracle on a sample of the queries (first, last, and some in between)
    sample = sorted(set([0, 1, 2, B_MANY // 2, B_MANY - 2, B_MANY - 1] + list(range(7, B_MANY, 97))))
    o_all = oracle.scores(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample]))
    assert_scores_close(g_all[sample], o_all, 32)
    for n, b in enumerate(sample):
        assert_topk_matches(g_ids[b], g_sc[b], o_all[n], cand[b], k, 32)


@pytest.mark.parametrize("K,k", [(3, 2), (64, 10), (130, 130), (256, 7)])
def test_one_launch_path_below_four_workgroups_per_compute_unit(K, k):
    """600 single-slice queries: fewer than four workgroups per compute unit, so 64-byte rows run in
    workgroups of 16 waves (the batches of B_MANY queries above run in workgroups of 8)."""
    B = 600
    say("one launch, wide workgroups: d=32 B=%d K=%d k=%d" % (B, K, k))
    emb, off, q, cand = random_problem(17 * K + 1, max(K, 300), 32, B, 32, K, 1, 40)
    cand[:, K // 2] = cand[:, 0]               # a duplicate candidate in every list: an exact tie
    g_ids, g_sc, g_all = both_paths(emb, off, q, cand, k, expect_launches=1)
    sample = sorted(set([0, 1, B // 2, B - 1] + list(range(5, B, 61))))
    o_all = oracle.scores(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample]))
    assert_scores_close(g_all[sample], o_all, 32)
    for n, b in enumerate(sample):
        assert_topk_matches(g_ids[b], g_sc[b], o_all[n], cand[b], k, 32)


@pytest.mark.parametrize("K,k", [(40, 10), (200, 200)])
def test_one_launch_path_at_eight_workgroups_per_compute_unit(K, k):
    """2100 single-slice queries of 256-byte binary16 rows: from eight workgroups per compute unit on,
    these rows run in workgroups of 4 waves (of 8 below), here with the ranking in the same launch."""
    B = 2100
    say("one launch, 4-wave workgroups: d=128 B=%d K=%d k=%d" % (B, K, k))
    emb, off, q, cand = random_problem(7 * K + 3, max(K, 300), 128, B, 32, K, 1, 40)
    g_ids, g_sc, g_all = both_paths(emb, off, q, cand, k, expect_launches=1)
    sample = sorted(set([0, 1, B // 2, B - 1] + list(range(11, B, 173))))
    o_all = oracle.scores(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample]))
    assert_scores_close(g_all[sample], o_all, 32)
    for n, b in enumerate(sample):
        assert_topk_matches(g_ids[b], g_sc[b], o_all[n], cand[b], k, 32)


@pytest.mark.parametrize("d,B,K,k", [(32, 1, 64, 10), (32, 5, 49, 49), (32, 37, 64, 1), (32, 200, 33, 7), (32, 3, 80, 10),
                                     (32, 180, 112, 5), (32, 400, 100, 100), (128, 1, 16, 10), (128, 190, 64, 10), (128, 9, 16, 16), (128, 130, 9, 3), (64, 6, 16, 5),
                                     (192, 3, 8, 8)])
def test_short_lists_of_small_batches_are_not_cut(d, B, K, k):
    """A list that the waves of one workgroup finish in a few documents each stays one slice however few the
    queries, so that the same launch ranks it (64-byte rows: up to 64 candidates; longer rows: 16, or 8 where
    a workgroup has 4 waves; more from half a workgroup per compute unit on)."""
    say("one launch, few queries: d=%d B=%d K=%d k=%d" % (d, B, K, k))
    emb, off, q, cand = random_problem(13 * K + d + B, 300, d, B, 32, K, 1, 40)
    if K > 2:
        cand[:, K - 1] = cand[:, 1]            # an exact tie in every list
    g_ids, g_sc, g_all = both_paths(emb, off, q, cand, k, expect_launches=1)
    o_all = oracle.scores(emb, off, q, cand)
    assert_scores_close(g_all, o_all, 32)
    for b in range(B):
        assert_topk_matches(g_ids[b], g_sc[b], o_all[b], cand[b], k, 32)


def test_lists_one_candidate_longer_are_cut_when_the_queries_are_few():
    say("d=32 K=81 and d=128 K=17 with 8 queries: two launches")
    emb, off, q, cand = random_problem(6, 300, 32, 8, 32, 81, 1, 20)
    both_paths(emb, off, q, cand, 10, expect_launches=2)
    emb, off, q, cand = random_problem(7, 300, 128, 8, 32, 17, 1, 20)
    both_paths(emb, off, q, cand, 10, expect_launches=2)


def test_longer_lists_take_two_launches():
    say("K = 257: two launches")
    emb, off, q, cand = random_problem(5, 400, 32, B_MANY, 32, 257, 1, 20)
    both_paths(emb, off, q, cand, 10, expect_launches=2)


@pytest.mark.parametrize("d", [32, 128])
def test_one_launch_path_with_empty_documents_exact_ties_and_duplicates(d):
    say("one launch: empty documents, identical documents, duplicate candidates, d=%d" % d)
    rng = np.random.default_rng(11)
    counts = np.array([0, 5, 0, 9, 20, 0, 33, 1, 0, 16] * 8)
    emb, off, q, _ = random_problem(12, counts.size, d, B_MANY, 32, 10, 0, 0, counts=counts)
    # documents 1 and 11, 3 and 13, ... hold the same rows (the count pattern repeats every 10 ids):
    # copy the rows so that they tie exactly
    for i in range(10, counts.size):
        emb[off[i]:off[i + 1]] = emb[off[i - 10]:off[i - 10] + counts[i]]
    K = 70
    cand = np.stack([rng.permutation(counts.size)[:K] for _ in range(B_MANY)]).astype(np.int64)
    cand[:, 5] = cand[:, 4]                    # a duplicate candidate in every list
    g_ids, g_sc, g_all = both_paths(emb, off, q, cand, K, expect_launches=1)
    sample = [0, 3, B_MANY - 1]
    o_all = oracle.scores(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample]))
    assert_scores_close(g_all[sample], o_all, 32)
    for n, b in enumerate(sample):
        assert_topk_matches(g_ids[b], g_sc[b], o_all[n], cand[b], K, 32)
        # exact ties: lower id first; empty documents (-inf) last, by id
        for r in range(1, K):
            if g_sc[b, r] == g_sc[b, r - 1]:
                assert g_ids[b, r - 1] <= g_ids[b, r]
        n_empty = int((counts[cand[b]] == 0).sum())
        assert np.all(np.isneginf(g_sc[b, K - n_empty:])) and not np.isneginf(g_sc[b, K - n_empty - 1])


def test_partial_reranking_and_prior_through_the_one_launch_path():
    say("one launch: partial re-ranking (R = 64 of 300) and a prior")
    emb, off, q, cand = random_problem(77, 900, 32, B_MANY, 32, 300, 2, 30)
    emb_d = torch.from_numpy(emb).to(DEV)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    table = espn.espn_table_load(emb_d, off)
    R, k = 64, 80
    assert espn.espn_rerank_plan(table, B_MANY, 32, R, min(k, R))["launches"] == 1
    g_ids, g_sc = espn.espn_rerank_partial(table, q_d, cand_d, R, k)
    sample = [0, 500, B_MANY - 1]
    o_ids, o_sc = oracle.rerank_partial(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample]),
                                        R, k)
    g_ids, g_sc = g_ids.cpu().numpy(), g_sc.cpu().numpy()
    assert np.array_equal(g_ids[:, R:], cand[:, R:k]) and np.isnan(g_sc[:, R:]).all()
    o_all = oracle.scores(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample][:, :R]))
    for n, b in enumerate(sample):
        assert_topk_matches(g_ids[b, :R], g_sc[b, :R], o_all[n], cand[b, :R], R, 32)
        assert np.array_equal(g_ids[b, R:], o_ids[n, R:])

    # a prior on a short list: totals = MaxSim + alpha * prior, ranked by the same launch
    short = np.ascontiguousarray(cand[:, :100])
    prior = (np.random.default_rng(3).normal(size=short.shape) * 4).astype(np.float32)
    assert espn.espn_rerank_plan(table, B_MANY, 32, 100, 10)["launches"] == 1
    p_ids, p_sc, ws = espn.espn_rerank_prior(table, q_d, torch.from_numpy(short).to(DEV),
                                             torch.from_numpy(prior).to(DEV), 0.5, 10)
    totals = ws[: 4 * B_MANY * 100].view(torch.float32).view(B_MANY, 100)
    t_ids, t_sc = espn.espn_topk(totals.contiguous(), torch.from_numpy(short).to(DEV), 10)
    assert torch.equal(p_ids, t_ids) and torch.equal(p_sc.view(torch.int32), t_sc.view(torch.int32))
    o_tot = oracle.scores_prior(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(short[sample]),
                                np.ascontiguousarray(prior[sample]), 0.5)
    got = totals[sample].cpu().numpy()
    assert np.all(np.abs(got - o_tot) <= 1e-3 * np.maximum(np.abs(o_tot) + 2.0 * np.abs(prior[sample]), 1e-3))
    espn.espn_table_check(table)
    table.free()
