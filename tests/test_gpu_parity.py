"""HIP path vs fp64 oracle, element by element, through the C-ABI.  Needs a MI355X."""
import math
import os

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


def to_dev(emb, off, q, cand):
    return (torch.from_numpy(np.ascontiguousarray(emb)).to(DEV), torch.from_numpy(q).to(DEV),
            torch.from_numpy(cand).to(DEV))


def run_both(emb, off, q, cand, k, check_ids_in_range=True):
    """emb [T,d] f16 numpy, off int64 numpy, q [B,Q,d] f16 numpy, cand [B,K] int64 numpy."""
    B, Q, d = q.shape
    K = cand.shape[1]
    o_ids, o_top, o_all = oracle.rerank(emb, off, q, cand, k)
    emb_d, q_d, cand_d = to_dev(emb, off, q, cand)
    if emb_d.numel() == 0:
        emb_d = torch.zeros((0, d), dtype=torch.float16, device=DEV)
    table = espn.espn_table_load(emb_d, off)
    g_all = espn.espn_score(table, q_d, cand_d)
    g_ids, g_top = espn.espn_rerank(table, q_d, cand_d, k)
    espn.espn_table_check(table)
    g_all, g_ids, g_top = g_all.cpu().numpy(), g_ids.cpu().numpy(), g_top.cpu().numpy()
    worst = assert_scores_close(g_all, o_all, Q)
    for b in range(B):
        assert_topk_matches(g_ids[b], g_top[b], o_all[b], cand[b], k, Q)
    table.free()
    return worst, (g_all, g_ids, g_top), (o_all, o_ids, o_top)


def random_problem(seed, N, d, B, Q, K, lo, hi, unit=True, counts=None):
    rng = np.random.default_rng(seed)
    if counts is None:
        counts = rng.integers(lo, hi + 1, size=N)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    x = rng.normal(size=(int(off[-1]), d)).astype(np.float32)
    qq = rng.normal(size=(B, Q, d)).astype(np.float32)
    if unit:
        x /= np.maximum(np.linalg.norm(x, axis=1, keepdims=True), 1e-20)
        qq /= np.linalg.norm(qq, axis=2, keepdims=True)
    else:
        x *= 3
        qq *= 2
    cand = np.stack([rng.permutation(N)[:K] for _ in range(B)]).astype(np.int64)
    return x.astype(np.float16), off, qq.astype(np.float16), cand


# ------------------------------------------------------------------ the small configuration, whole
def test_c1_tiny_every_pair():
    w = synth.WORKLOADS["c1"]
    say("c1 tiny: N=%d d=%d B=%d K=%d" % (w.n_docs, w.dim, w.B, w.K))
    emb, off = synth.table(w)
    q = synth.queries(w).numpy()
    cand = synth.candidates(w)
    worst, _, _ = run_both(emb.numpy(), off, q, cand, w.k)
    say("worst relative error %.2e" % worst)
    assert worst < 1e-4


@pytest.mark.parametrize("d", [32, 128])
@pytest.mark.parametrize("Q", [1, 7, 16, 17, 32, 33, 47, 48, 49, 64])
def test_query_lengths_and_ragged_documents(d, Q):
    # token counts straddle the 16-row tile: 1, 15, 16, 17, 31, 32, 33 ... and up to 180
    counts = np.array([1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 100, 127, 128, 129, 179, 180] * 8)
    say("ragged d=%d Q=%d" % (d, Q))
    emb, off, q, cand = random_problem(100 + Q, counts.size, d, 3, Q, 157, 0, 0, counts=counts)
    run_both(emb, off, q, cand, 10)


@pytest.mark.parametrize("d", [32, 128])
def test_arbitrary_values_not_unit_norm(d):
    say("non-unit values d=%d" % d)
    emb, off, q, cand = random_problem(7, 300, d, 4, 32, 123, 1, 90, unit=False)
    run_both(emb, off, q, cand, 123)      # k = K: the full ranking


@pytest.mark.parametrize("K,k", [(1, 1), (3, 0), (5, 5), (33, 1), (1000, 10), (1025, 7), (4100, 12)])
def test_candidate_count_shapes(K, k):
    say("K=%d k=%d" % (K, k))
    emb, off, q, cand = random_problem(K, max(K, 50), 32, 2, 32, K, 3, 40)
    run_both(emb, off, q, cand, k)


@pytest.mark.parametrize("d,Q", [(8, 4), (40, 32), (72, 5), (32, 65), (128, 100), (160, 33), (264, 16)])
def test_generic_kernel_shapes(d, Q):
    say("generic d=%d Q=%d" % (d, Q))
    emb, off, q, cand = random_problem(d + Q, 200, d, 2, Q, 61, 0, 70)
    run_both(emb, off, q, cand, 9)


@pytest.mark.parametrize("d,Q", [(d, Q) for d in (64, 96, 160, 192, 224, 256) for Q in (5, 32)] +
                         [(64, 33), (64, 64), (96, 50), (96, 64)])
def test_other_row_lengths_on_the_matrix_cores(d, Q):
    # every multiple of 32 up to 256 takes the matrix-core kernel (up to 64 query rows for rows of up to 128
    # components, 32 beyond); lengths straddle the 16-row tile
    counts = np.array([0, 1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 100, 127, 128, 129, 180] * 6)
    say("matrix cores d=%d Q=%d" % (d, Q))
    emb, off, q, cand = random_problem(3 * d + Q, counts.size, d, 3, Q, 117, 0, 0, counts=counts)
    run_both(emb, off, q, cand, 10)


@pytest.mark.parametrize("d,Q", [(32, 32), (32, 64), (64, 5), (64, 32), (64, 64), (96, 32), (96, 50), (128, 1), (128, 17),
                                 (128, 32), (128, 33), (128, 64), (160, 32), (192, 7), (224, 32), (256, 32)])
def test_few_pairs_against_a_large_table_take_the_lane_linear_loads(d, Q):
    """With at most half as many (query, candidate) pairs as the table has documents, rows longer than 64 bytes
    are fetched lane-linearly with non-temporal loads and put in order through LDS; with more pairs every lane
    loads its own part of a row.  Same documents both ways: the scores have to be bit-identical, and right."""
    lengths = np.array([0, 1, 2, 3, 4, 5, 15, 16, 17, 31, 32, 33, 47, 48, 49, 63, 64, 65, 100, 127, 128, 129, 180, 7])
    counts = np.tile(lengths, 40)                              # 960 documents
    say("lane-linear loads d=%d Q=%d" % (d, Q))
    emb, off, q, cand = random_problem(5 * d + Q, counts.size, d, 3, Q, 150, 0, 0, counts=counts)
    assert 2 * cand.size <= counts.size
    worst, (g_few, _, _), _ = run_both(emb, off, q, cand, 10)
    # the same queries in a batch too large for that path (the extra queries are copies)
    reps = 4
    q_many, cand_many = np.tile(q, (reps, 1, 1)), np.tile(cand, (reps, 1))
    assert 2 * cand_many.size > counts.size
    table = espn.espn_table_load(torch.from_numpy(emb).to(DEV), off)
    q_d, cand_d = torch.from_numpy(q_many).to(DEV), torch.from_numpy(cand_many).to(DEV)
    few = np.asarray(g_few, dtype=np.float32).view(np.int32)
    # ... and both batches with the choice made by the caller instead of by the library
    for mode in (espn.ESPN_FETCH_AUTO, espn.ESPN_FETCH_STREAMING, espn.ESPN_FETCH_CACHED):
        espn.espn_table_set_fetch(table, mode)
        g_many = espn.espn_score(table, q_d, cand_d).cpu().numpy()
        g_again = espn.espn_score(table, q_d[:3].contiguous(), cand_d[:3].contiguous()).cpu().numpy()
        espn.espn_table_check(table)
        assert np.array_equal(g_again.view(np.int32), few), mode
        for rep in range(reps):
            assert np.array_equal(g_many[rep * 3:(rep + 1) * 3].view(np.int32), few), (mode, rep)
    with pytest.raises(espn.EspnError):
        espn.espn_table_set_fetch(table, 3)
    table.free()


def test_the_library_is_told_whether_the_lists_of_a_batch_share_documents():
    """espn_table_sample looks at a batch's candidate lists when the caller asks for it (never on its own); the
    estimate (the share of sampled pairs that repeat a document) separates uniformly drawn lists from lists that
    share popular documents, decides how the default fetch mode loads the rows from then on, and the scores are
    the same whichever way that is."""
    say("sharing estimate")
    rng = np.random.default_rng(21)
    N, d, B, K = 30_000, 128, 8, 200            # 1600 uniform pairs over 30 000 documents: about 2.7 % repeat
    counts = rng.integers(1, 30, size=N)
    emb, off, q, _ = random_problem(77, N, d, B, 32, K, 0, 0, counts=counts)
    uniform = np.stack([rng.permutation(N)[:K] for _ in range(B)]).astype(np.int64)
    popular = rng.permutation(N)[:260]
    shared = np.stack([rng.permutation(popular)[:K] for _ in range(B)]).astype(np.int64)   # every list from 260 documents
    table = espn.espn_table_load(torch.from_numpy(emb).to(DEV), off)
    assert espn.espn_table_sharing_estimate(table) == -1.0
    q_d = torch.from_numpy(q).to(DEV)
    # scoring never samples by itself, however often it is called
    for call in range(70):
        espn.espn_score(table, q_d, torch.from_numpy(shared).to(DEV))
    torch.cuda.synchronize()
    assert espn.espn_table_sharing_estimate(table) == -1.0
    results = {}
    for name, cand in (("uniform", uniform), ("shared", shared), ("uniform again", uniform)):
        cand_d = torch.from_numpy(cand).to(DEV)
        before = espn.espn_score(table, q_d, cand_d).cpu().numpy()      # planned with the previous estimate
        est = espn.espn_table_sample(table, cand_d)
        assert est == espn.espn_table_sharing_estimate(table)
        after = espn.espn_score(table, q_d, cand_d).cpu().numpy()       # planned with this one
        assert np.array_equal(before.view(np.int32), after.view(np.int32)), name
        results[name] = (est, after)
    espn.espn_table_check(table)
    assert 0.0 <= results["uniform"][0] < 0.05, results["uniform"][0]
    assert results["shared"][0] > 0.5, results["shared"][0]
    assert results["uniform again"][0] == results["uniform"][0]          # the same lists, the same sample
    assert np.array_equal(results["uniform"][1].view(np.int32), results["uniform again"][1].view(np.int32))
    assert_scores_close(results["shared"][1], oracle.scores(emb, off, q, shared), 32)
    assert_scores_close(results["uniform"][1], oracle.scores(emb, off, q, uniform), 32)
    # an empty batch is a sample of nothing
    assert espn.espn_table_sample(table, torch.zeros((0, 5), dtype=torch.int64, device=DEV)) == 0.0
    table.free()


@pytest.mark.parametrize("d", [32, 128, 64])
def test_empty_documents_score_minus_infinity_and_rank_last(d):
    say("empty docs d=%d" % d)
    counts = np.array([0, 5, 0, 9, 20, 0, 33, 1, 0, 16] * 6)
    emb, off, q, cand = random_problem(5, counts.size, d, 2, 32, 60, 0, 0, counts=counts)
    _, (g_all, g_ids, g_top), _ = run_both(emb, off, q, cand, 60)
    n_empty = int((counts == 0).sum())
    for b in range(2):
        tail_ids = g_ids[b, -n_empty:]
        assert np.all(np.isneginf(g_top[b, -n_empty:]))
        assert np.all(np.diff(tail_ids) > 0)              # ties at -inf: ascending id
        assert np.all(counts[tail_ids] == 0)


def test_all_documents_empty_and_zero_sized_batches():
    say("all-empty table, B=0, K=0")
    off = np.zeros(11, dtype=np.int64)
    emb = np.zeros((0, 32), dtype=np.float16)
    q = np.ones((2, 32, 32), dtype=np.float16)
    cand = np.stack([np.arange(10)[::-1], np.arange(10)]).astype(np.int64)
    _, (g_all, g_ids, g_top), _ = run_both(emb, off, q, cand, 4)
    assert np.all(np.isneginf(g_all)) and g_ids.tolist() == [[0, 1, 2, 3], [0, 1, 2, 3]]
    emb_d = torch.zeros((16, 32), dtype=torch.float16, device=DEV)
    table = espn.espn_table_load(emb_d, np.array([0, 16], dtype=np.int64))
    q0 = torch.zeros((0, 32, 32), dtype=torch.float16, device=DEV)
    c0 = torch.zeros((0, 5), dtype=torch.int64, device=DEV)
    ids, sc = espn.espn_rerank(table, q0, c0, 2)
    assert ids.shape == (0, 2)
    q1 = torch.zeros((3, 32, 32), dtype=torch.float16, device=DEV)
    c1 = torch.zeros((3, 0), dtype=torch.int64, device=DEV)
    ids, sc = espn.espn_rerank(table, q1, c1, 0)
    assert ids.shape == (3, 0)
    espn.espn_table_check(table)


def test_handworked_ranking_through_the_gpu():
    # the hand-worked fixture (d = 2) zero-padded to d = 8, the smallest vector length supported
    from tests.test_oracle_pins import parse_rerank, GOLDEN
    emb2, off, q2, cand, want = parse_rerank(os.path.join(GOLDEN, "handworked_rerank.txt"))
    emb = np.zeros((emb2.shape[0], 8), dtype=np.float16); emb[:, :2] = emb2
    q = np.zeros((1, q2.shape[1], 8), dtype=np.float16); q[:, :, :2] = q2
    say("hand-worked ranking, d padded to 8")
    _, (g_all, g_ids, g_top), _ = run_both(emb, off, q, cand, 5)
    assert g_ids[0].tolist() == want["ids"]
    assert g_top[0].tolist() == want["scores"]
    # and on the matrix-core kernel: pad to d = 32
    emb32 = np.zeros((emb2.shape[0], 32), dtype=np.float16); emb32[:, :2] = emb2
    q32 = np.zeros((1, q2.shape[1], 32), dtype=np.float16); q32[:, :, :2] = q2
    _, (g_all, g_ids, g_top), _ = run_both(emb32, off, q32, cand, 5)
    assert g_ids[0].tolist() == want["ids"] and g_top[0].tolist() == want["scores"]


@pytest.mark.parametrize("d", [32, 128])
def test_identical_documents_tie_exactly_and_lower_id_first(d):
    say("byte-identical docs d=%d" % d)
    rng = np.random.default_rng(3)
    rows = rng.normal(size=(37, d)).astype(np.float16)
    other = rng.normal(size=(20, d)).astype(np.float16)
    emb = np.concatenate([rows, other, rows, rows])
    off = np.array([0, 37, 57, 94, 131], dtype=np.int64)
    q = rng.normal(size=(2, 32, d)).astype(np.float16)
    cand = np.array([[3, 1, 2, 0], [0, 2, 1, 3]], dtype=np.int64)
    _, (g_all, g_ids, g_top), _ = run_both(emb, off, q, cand, 4)
    for b in range(2):
        same = [i for i in g_ids[b].tolist() if i != 1]
        assert same == [0, 2, 3]
        sc = {int(i): float(s) for i, s in zip(g_ids[b], g_top[b])}
        assert sc[0] == sc[2] == sc[3]


def test_duplicate_candidates_are_scored_and_ranked_independently():
    say("duplicate candidate ids")
    emb, off, q, cand = random_problem(9, 50, 32, 2, 32, 40, 1, 30)
    cand[:, 10:20] = cand[:, 0:10]
    run_both(emb, off, q, cand, 40)


@pytest.mark.parametrize("d", [32, 128, 64])
def test_out_of_range_ids_are_flagged_and_read_nothing(d):
    say("out-of-range ids d=%d" % d)
    emb, off, q, cand = random_problem(11, 64, d, 2, 32, 33, 1, 30)
    good_all = oracle.scores(emb, off, q, cand)
    bad = cand.copy()
    bad[0, 5], bad[1, 32], bad[1, 0] = 64, -1, 1 << 40
    emb_d, q_d, cand_d = to_dev(emb, off, q, bad)
    table = espn.espn_table_load(emb_d, off)
    g_all = espn.espn_score(table, q_d, cand_d).cpu().numpy()
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_check(table)
    assert ei.value.status == espn.ESPN_ERR_ID_RANGE
    espn.espn_table_check(table)                       # flag was cleared
    mask = bad != cand
    assert np.all(np.isneginf(g_all[mask]))
    assert_scores_close(g_all[~mask], good_all[~mask], 32)


def test_same_inputs_give_bit_identical_outputs():
    say("determinism")
    w = synth.WORKLOADS["c1"]
    emb, off = synth.table(w)
    q, cand = synth.queries(w).to(DEV), torch.from_numpy(synth.candidates(w)).to(DEV)
    table = espn.espn_table_load(emb.to(DEV), off)
    a = espn.espn_score(table, q, cand).clone()
    ia, sa = espn.espn_rerank(table, q, cand, w.k)
    for _ in range(3):
        b = espn.espn_score(table, q, cand)
        ib, sb = espn.espn_rerank(table, q, cand, w.k)
        assert torch.equal(a, b) and torch.equal(ia, ib) and torch.equal(sa, sb)


def test_binding_rejects_wrong_shapes_before_launching():
    emb = torch.zeros((16, 32), dtype=torch.float16, device=DEV)
    table = espn.espn_table_load(emb, np.array([0, 16], dtype=np.int64))
    q = torch.zeros((2, 32, 32), dtype=torch.float16, device=DEV)
    cand = torch.zeros((2, 4), dtype=torch.int64, device=DEV)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_rerank(table, q, cand, 5)
    assert ei.value.status == espn.ESPN_ERR_SHAPE
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_rerank(table, q, cand, 2, workspace=torch.empty(256, dtype=torch.uint8, device=DEV)[:16])
    assert ei.value.status == espn.ESPN_ERR_SHAPE
    with pytest.raises(ValueError):
        espn.espn_score(table, torch.zeros((2, 32, 64), dtype=torch.float16, device=DEV), cand)
    info = table.info()
    assert info["n_docs"] == 1 and info["total_rows"] == 16 and info["dim"] == 32 and info["residency"] == 0


# ------------------------------------------------------------------ top-k on its own
@pytest.mark.parametrize("K,k", [(1000, 10), (1000, 1000), (64, 64), (5000, 33), (257, 256), (1, 1), (2, 2), (100, 40),
                                 (256, 256), (300, 33), (1000, 32), (1024, 500), (1025, 1025), (2048, 20),
                                 (3000, 100), (4096, 4096), (4097, 50)])
def test_topk_alone_with_many_exact_ties(K, k):
    say("topk alone K=%d k=%d" % (K, k))
    rng = np.random.default_rng(K + k)
    B = 3
    sc = np.round(rng.normal(size=(B, K)), 1).astype(np.float32)
    sc[0, :7] = -np.inf
    cand = np.stack([rng.permutation(10 * K)[:K] for _ in range(B)]).astype(np.int64)
    cand[1, :] += 1 << 33                                # ids beyond 32 bits
    o_ids, o_top = oracle.topk(sc.astype(np.float64), cand, k)
    g_ids, g_top = espn.espn_topk(torch.from_numpy(sc).to(DEV), torch.from_numpy(cand).to(DEV), k)
    assert np.array_equal(g_ids.cpu().numpy(), o_ids)       # scores are exact in fp32: everything is pinned
    assert np.array_equal(g_top.cpu().numpy().astype(np.float64), o_top)


@pytest.mark.parametrize("K,k", [(1000, 1000), (1000, 100), (200, 200), (4000, 64)])
def test_topk_alone_when_all_scores_are_equal(K, k):
    """Every score is the same (all documents empty, or identical): the ranking is by id alone, and
    duplicate ids stay next to each other."""
    say("topk alone, all scores equal, K=%d k=%d" % (K, k))
    rng = np.random.default_rng(K * 7 + k)
    B = 4
    sc = np.empty((B, K), dtype=np.float32)
    sc[0], sc[1], sc[2], sc[3] = -np.inf, 3.25, 0.0, -1.5
    sc[2, ::2] = -0.0                                      # -0 and +0 are the same score
    cand = np.stack([rng.permutation(3 * K)[:K] for _ in range(B)]).astype(np.int64) - K
    cand[3, K // 2:] = cand[3, : K - K // 2]             # every id of the last list twice
    o_ids, o_top = oracle.topk(sc.astype(np.float64), cand, k)
    g_ids, g_top = espn.espn_topk(torch.from_numpy(sc).to(DEV), torch.from_numpy(cand).to(DEV), k)
    assert np.array_equal(g_ids.cpu().numpy(), o_ids)
    assert np.array_equal(g_top.cpu().numpy().astype(np.float64), o_top)
