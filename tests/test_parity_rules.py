"""The comparison rules themselves (CPU): they accept what they should and catch planted mistakes.
Mistakes are planted in copies of the oracle's output, never on the GPU."""
import numpy as np
import pytest

import oracle
from tests.parity import assert_scores_close, assert_topk_matches, cancellation_floor, tol_of


def problem(seed=0, K=60, Q=8, d=16):
    rng = np.random.default_rng(seed)
    counts = rng.integers(1, 9, size=200)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    emb = rng.normal(size=(off[-1], d)).astype(np.float16)
    q = rng.normal(size=(1, Q, d)).astype(np.float16)
    cand = rng.permutation(200)[:K].astype(np.int64)[None]
    ids, top, allsc = oracle.rerank(emb, off, q, cand, 10)
    return ids[0], top[0], allsc[0], cand[0], Q


def test_exact_answer_and_fp32_rounding_are_accepted():
    ids, top, allsc, cand, Q = problem()
    assert_topk_matches(ids, top, allsc, cand, 10, Q)
    assert_topk_matches(ids, top.astype(np.float32), allsc, cand, 10, Q)
    assert_scores_close(allsc.astype(np.float32), allsc, Q)


def test_wrong_id_at_a_separated_rank_is_caught():
    ids, top, allsc, cand, Q = problem()
    bad = ids.copy()
    bad[0], bad[1] = ids[1], ids[0]                      # top two swapped, scores left in place
    with pytest.raises(AssertionError):
        assert_topk_matches(bad, top, allsc, cand, 10, Q)
    bad = ids.copy()
    bad[9] = [c for c in cand if c not in ids][0]        # an id from outside the top 10
    with pytest.raises(AssertionError):
        assert_topk_matches(bad, top, allsc, cand, 10, Q)
    with pytest.raises(AssertionError):
        assert_topk_matches(np.where(ids == ids[3], 10**6, ids), top, allsc, cand, 10, Q)   # not a candidate


def test_wrong_scores_are_caught():
    ids, top, allsc, cand, Q = problem()
    off_by = top.copy()
    off_by[4] *= 1 + 5e-3
    with pytest.raises(AssertionError):
        assert_topk_matches(ids, off_by, allsc, cand, 10, Q)
    g = allsc.copy()
    g[7] += 3 * tol_of(g[7], Q)
    with pytest.raises(AssertionError):
        assert_scores_close(g, allsc, Q)
    g = allsc.copy()
    g[7] = -np.inf
    with pytest.raises(AssertionError):
        assert_scores_close(g, allsc, Q)


def test_near_ties_may_swap_but_exact_ties_must_follow_the_id_rule():
    # two candidates whose oracle scores differ by far less than the tolerance: either order is fine
    allsc = np.array([5.0, 4.0, 4.0 + 1e-9, 1.0])
    cand = np.array([10, 30, 20, 40], dtype=np.int64)
    assert_topk_matches([10, 20, 30], [5.0, 4.0, 4.0], allsc, cand, 3, 32)
    assert_topk_matches([10, 30, 20], [5.0, 4.0 + 1e-7, 4.0], allsc, cand, 3, 32)
    # the GPU reported equal scores but listed the higher id first: its own output is out of order
    with pytest.raises(AssertionError):
        assert_topk_matches([10, 30, 20], [5.0, 4.0, 4.0], allsc, cand, 3, 32)
    # an id returned twice although listed once
    with pytest.raises(AssertionError):
        assert_topk_matches([10, 20, 20], [5.0, 4.0, 4.0], allsc, cand, 3, 32)


def test_cancelling_terms_get_the_floor_binary32_accumulation_can_keep():
    # a two-row query against one-row documents: the two maxima are dot products of either sign
    rng = np.random.default_rng(5)
    d, Q, n = 192, 2, 4000
    emb = (rng.normal(size=(n, d)) * 7).astype(np.float16)
    off = np.arange(n + 1, dtype=np.int64)
    q = (rng.normal(size=(1, Q, d)) * 3).astype(np.float16)
    cand = np.arange(n, dtype=np.int64)[None]
    exact = oracle.scores(emb, off, q, cand)
    magnitude = oracle.scores(np.abs(emb), off, np.abs(q), cand)
    assert np.all(magnitude >= np.abs(exact))
    floor = cancellation_floor(magnitude, d, Q)
    # the same scores accumulated in binary32, row by row
    e32, q32 = emb.astype(np.float32), q[0].astype(np.float32)
    approx = np.array([[np.float32((q32 @ e32[j]).sum(dtype=np.float32)) for j in range(n)]], dtype=np.float64)
    worst = np.abs(approx - exact).max()
    assert worst > 0 and np.all(np.abs(approx - exact) <= floor)          # the bound holds, with room
    assert_scores_close(approx, exact, Q, floor=floor)
    small = np.argmin(np.abs(exact[0]) / magnitude[0])                      # the pair that cancels most
    assert abs(exact[0, small]) < 1e-3 * magnitude[0, small]
    # ordinary pairs are still held to the relative tolerance: the floor is far below it there
    ordinary = np.abs(exact[0]) > 0.1 * magnitude[0]
    assert ordinary.sum() > 100 and np.all(floor[0, ordinary] < 0.2 * 1e-3 * np.abs(exact[0, ordinary]))
    # and a mistake of the size of one dropped component is caught even at the cancelling pair
    g = approx.copy()
    g[0, small] += float(q32[0, 0] * e32[small, 0])
    with pytest.raises(AssertionError):
        assert_scores_close(g, exact, Q, floor=floor)
