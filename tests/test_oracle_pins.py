"""Pins for the CPU oracle: each test fixes the oracle against something other than itself
(hand-worked values, closed forms, invariants of Eq. 1, numpy's own binary16 and matmul)."""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def h(a):
    return np.asarray(a, dtype=np.float16)


def parse_cases(path):
    cases, cur = [], None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tag, *rest = line.split()
        if tag == "case":
            cur = {"name": rest[0], "q": [], "t": []}
        elif tag == "d":
            cur["d"] = int(rest[0])
        elif tag in ("q", "t"):
            cur[tag].append([float(x) for x in rest])
        elif tag == "expect":
            cur["expect"] = float(rest[0])
        elif tag == "end":
            cases.append(cur)
    return cases


# ---------------------------------------------------------------- binary16 widening
def test_half_widening_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_to_double(int(b)) for b in bits])
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


# ---------------------------------------------------------------- P1 hand-worked values
@pytest.mark.parametrize("case", parse_cases(os.path.join(GOLDEN, "handworked_maxsim.txt")),
                         ids=lambda c: c["name"])
def test_handworked_pairs(case):
    q, t = h(case["q"]), h(case["t"])
    assert q.shape[1] == case["d"] and t.shape[1] == case["d"]
    assert oracle.maxsim_pair(q, t) == case["expect"]


def parse_rerank(path):
    d, q, docs, cur = None, [], {}, None
    out = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tag, *rest = line.split()
        if tag == "d":
            d = int(rest[0])
        elif tag == "q":
            q.append([float(x) for x in rest])
        elif tag == "doc":
            cur = int(rest[0])
            docs[cur] = []
        elif tag == "t":
            docs[cur].append([float(x) for x in rest])
        elif tag == "cand":
            out["cand"] = [int(x) for x in rest]
        elif tag == "rank_ids":
            out["ids"] = [int(x) for x in rest]
        elif tag == "rank_scores":
            out["scores"] = [float(x) for x in rest]
    n = max(docs) + 1
    counts = np.array([len(docs[i]) for i in range(n)], dtype=np.int64)
    rows = [r for i in range(n) for r in docs[i]]
    emb = h(rows).reshape(-1, d)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    return emb, off, h(q)[None], np.array([out["cand"]], dtype=np.int64), out


def test_handworked_ranked_list_every_k():
    emb, off, q, cand, want = parse_rerank(os.path.join(GOLDEN, "handworked_rerank.txt"))
    K = cand.shape[1]
    for k in range(0, K + 1):
        ids, top, allsc = oracle.rerank(emb, off, q, cand, k)
        assert ids[0].tolist() == want["ids"][:k]
        assert top[0].tolist() == want["scores"][:k]
    # candidate order must not matter for the ranked list
    perm = np.array([[3, 0, 4, 1, 2]])
    ids, top, _ = oracle.rerank(emb, off, q, np.take_along_axis(cand, perm, 1), K)
    assert ids[0].tolist() == want["ids"] and top[0].tolist() == want["scores"]


# ---------------------------------------------------------------- P2 brute force in another shape
def brute(q, t):
    """Full Q x t matrix by numpy matmul in fp64, row-wise max, then sum."""
    if t.shape[0] == 0:
        return -math.inf
    m = q.astype(np.float64) @ t.astype(np.float64).T
    return float(m.max(axis=1).sum())


@pytest.mark.parametrize("seed", range(6))
def test_matches_matmul_bruteforce_random(seed):
    rng = np.random.default_rng(seed)
    Q, d, t = int(rng.integers(1, 9)), int(rng.integers(1, 20)), int(rng.integers(1, 12))
    q = h(rng.normal(size=(Q, d)) * 3)
    doc = h(rng.normal(size=(t, d)) * 3)
    got, want = oracle.maxsim_pair(q, doc), brute(q, doc)
    assert abs(got - want) <= 1e-12 * max(1.0, abs(want))


@pytest.mark.parametrize("seed", range(4))
def test_matches_matmul_bruteforce_exact_on_integers(seed):
    # small integers: every product and partial sum is exact, so the two must agree bit for bit
    rng = np.random.default_rng(100 + seed)
    Q, d, t = 5, 16, 9
    q = h(rng.integers(-8, 9, size=(Q, d)))
    doc = h(rng.integers(-8, 9, size=(t, d)))
    assert oracle.maxsim_pair(q, doc) == brute(q, doc)


def small_problem(seed, N=40, d=8, B=3, Q=5, K=12, lo=0, hi=7, integer=False):
    rng = np.random.default_rng(seed)
    counts = rng.integers(lo, hi + 1, size=N)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    if integer:
        emb = h(rng.integers(-6, 7, size=(off[-1], d)))
        q = h(rng.integers(-6, 7, size=(B, Q, d)))
    else:
        emb = h(rng.normal(size=(off[-1], d)))
        q = h(rng.normal(size=(B, Q, d)))
    cand = np.stack([rng.permutation(N)[:K] for _ in range(B)]).astype(np.int64)
    return emb, off, q, cand


def test_csr_scores_match_bruteforce_per_pair():
    emb, off, q, cand = small_problem(7, integer=True)
    sc = oracle.scores(emb, off, q, cand)
    for b in range(q.shape[0]):
        for kk in range(cand.shape[1]):
            i = cand[b, kk]
            assert sc[b, kk] == brute(q[b], emb[off[i]:off[i + 1]])


# ---------------------------------------------------------------- P3 / P4 permutations
def test_permuting_document_rows_changes_nothing():
    rng = np.random.default_rng(3)
    q, doc = h(rng.normal(size=(6, 16))), h(rng.normal(size=(11, 16)))
    base = oracle.maxsim_pair(q, doc)
    for _ in range(5):
        assert oracle.maxsim_pair(q, doc[rng.permutation(11)]) == base


def test_permuting_query_rows_changes_only_rounding():
    rng = np.random.default_rng(4)
    q, doc = h(rng.normal(size=(6, 16))), h(rng.normal(size=(11, 16)))
    base = oracle.maxsim_pair(q, doc)
    for _ in range(5):
        assert abs(oracle.maxsim_pair(q[rng.permutation(6)], doc) - base) <= 1e-13 * abs(base)


def test_permuting_vector_components_consistently_changes_only_rounding():
    rng = np.random.default_rng(5)
    q, doc = h(rng.normal(size=(4, 32))), h(rng.normal(size=(9, 32)))
    p = rng.permutation(32)
    a, b = oracle.maxsim_pair(q, doc), oracle.maxsim_pair(q[:, p], doc[:, p])
    assert abs(a - b) <= 1e-13 * abs(a)


# ---------------------------------------------------------------- P5 document identical to the query
def test_document_equal_to_query_scores_sum_of_squared_norms():
    # orthogonal rows: the self match wins by construction, value exact
    q = h(np.diag([1.0, 2.0, 0.5, 4.0]))
    assert oracle.maxsim_pair(q, q) == 1 + 4 + 0.25 + 16
    # random near-unit rows (what the workloads use): self match wins with overwhelming probability
    rng = np.random.default_rng(11)
    x = rng.normal(size=(32, 32))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    q = h(x)
    want = float((q.astype(np.float64) ** 2).sum())
    got = oracle.maxsim_pair(q, q)
    assert abs(got - want) <= 1e-12 * want
    assert abs(got - 32) < 0.05                      # unit norms up to binary16 rounding
    # in general it is a lower bound
    q = h(rng.normal(size=(5, 3)))
    assert oracle.maxsim_pair(q, q) >= float((q.astype(np.float64) ** 2).sum()) - 1e-12


# ---------------------------------------------------------------- P6 single-row document
def test_single_row_document_is_one_dot_product_with_the_summed_query():
    rng = np.random.default_rng(12)
    q = h(rng.integers(-5, 6, size=(7, 8)))
    t0 = h(rng.integers(-5, 6, size=(1, 8)))
    want = float(q.astype(np.float64).sum(axis=0) @ t0[0].astype(np.float64))
    assert oracle.maxsim_pair(q, t0) == want


# ---------------------------------------------------------------- P7 homogeneity (raw dot product)
def test_positive_scaling_scales_the_score_and_negative_scaling_does_not():
    rng = np.random.default_rng(13)
    q, doc = h(rng.normal(size=(4, 8))), h(rng.normal(size=(6, 8)))
    base = oracle.maxsim_pair(q, doc)
    assert oracle.maxsim_pair(h(q * 4), doc) == 4 * base        # powers of two: exact
    assert oracle.maxsim_pair(q, h(doc * 0.5)) == 0.5 * base
    assert oracle.maxsim_pair(h(-q), doc) != -base              # max turns into min
    # no normalisation hidden anywhere: a cosine would ignore the length of a lone document row
    one = doc[:1]
    assert oracle.maxsim_pair(q, h(one * 2)) == 2 * oracle.maxsim_pair(q, one)


# ---------------------------------------------------------------- P8 monotone in the row set
def test_appending_rows_never_lowers_and_duplicates_change_nothing():
    rng = np.random.default_rng(14)
    q = h(rng.normal(size=(5, 8)))
    d1, d2 = h(rng.normal(size=(4, 8))), h(rng.normal(size=(3, 8)))
    s1, s2 = oracle.maxsim_pair(q, d1), oracle.maxsim_pair(q, d2)
    s12 = oracle.maxsim_pair(q, np.concatenate([d1, d2]))
    assert s12 >= max(s1, s2)
    assert oracle.maxsim_pair(q, np.concatenate([d1, d1[2:3], d1[0:1]])) == s1


# ---------------------------------------------------------------- P9 bound, empty document
def test_unit_vectors_bound_and_empty_document():
    rng = np.random.default_rng(15)
    x = rng.normal(size=(40, 16))
    x /= np.linalg.norm(x, axis=1, keepdims=True)
    q, doc = h(x[:32]), h(x[32:])
    s = oracle.maxsim_pair(q, doc)
    assert abs(s) <= 32 * (1 + 2e-3)
    assert oracle.maxsim_pair(q, np.zeros((0, 16), dtype=np.float16)) == -math.inf


# ---------------------------------------------------------------- P10 ranked list vs other definitions
def test_topk_equals_full_sort_and_repeated_extract_max():
    rng = np.random.default_rng(16)
    B, K = 4, 50
    sc = np.round(rng.normal(size=(B, K)), 1)            # coarse: many exact ties
    cand = np.stack([rng.permutation(1000)[:K] for _ in range(B)]).astype(np.int64)
    for k in (0, 1, 7, K):
        ids, top = oracle.topk(sc, cand, k)
        for b in range(B):
            order = sorted(range(K), key=lambda j: (-sc[b, j], cand[b, j]))[:k]   # python's own sort
            assert ids[b].tolist() == [int(cand[b, j]) for j in order]
            assert top[b].tolist() == [sc[b, j] for j in order]
            # k rounds of extract-max with the same tie rule
            left = list(range(K))
            for r in range(k):
                best = left[0]
                for j in left[1:]:
                    if sc[b, j] > sc[b, best] or (sc[b, j] == sc[b, best] and cand[b, j] < cand[b, best]):
                        best = j
                assert ids[b, r] == cand[b, best]
                left.remove(best)
    _, top1 = oracle.topk(sc, cand, 1)
    assert np.array_equal(top1[:, 0], sc.max(axis=1))
    with pytest.raises(ValueError):
        oracle.topk(sc, cand, K + 1)


def test_topk_with_lexsort():
    rng = np.random.default_rng(17)
    sc = np.round(rng.normal(size=(3, 64)), 1)
    cand = np.stack([rng.permutation(500)[:64] for _ in range(3)]).astype(np.int64)
    ids, top = oracle.topk(sc, cand, 64)
    for b in range(3):
        order = np.lexsort((cand[b], -sc[b]))            # numpy: last key is primary
        assert np.array_equal(ids[b], cand[b][order]) and np.array_equal(top[b], sc[b][order])


# ---------------------------------------------------------------- P11 identical bytes tie
def test_identical_documents_tie_and_lower_id_wins():
    rng = np.random.default_rng(18)
    d = 8
    rows = h(rng.normal(size=(5, d)))
    other = h(rng.normal(size=(3, d)))
    emb = np.concatenate([rows, other, rows])            # doc 0 and doc 2 hold the same bytes
    off = np.array([0, 5, 8, 13], dtype=np.int64)
    q = h(rng.normal(size=(1, 4, d)))
    for cand in ([[2, 1, 0]], [[0, 1, 2]], [[1, 2, 0]]):
        ids, top, allsc = oracle.rerank(emb, off, q, np.array(cand, dtype=np.int64), 3)
        pos = {int(i): p for p, i in enumerate(ids[0])}
        assert pos[0] + 1 == pos[2]
        assert top[0, pos[0]] == top[0, pos[2]]


# ---------------------------------------------------------------- P12 CSR boundaries
def test_one_hot_table_detects_reading_a_neighbours_rows():
    # document i holds (i % 3) + 1 copies of (i+1) * e_{i mod d}: score = (i+1) * sum_r max(q[r, i mod d], ...)
    # i.e. exactly (i+1) * column sum of q at column i mod d when that is what the only rows say.
    d, N = 4, 12
    counts = np.array([(i % 3) + 1 for i in range(N)])
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    emb = np.zeros((off[-1], d), dtype=np.float16)
    for i in range(N):
        emb[off[i]:off[i + 1], i % d] = i + 1
    q = h([[[1, -2, 3, 0.5], [2, 1, -1, -4]]])
    cand = np.arange(N, dtype=np.int64)[None]
    sc = oracle.scores(emb, off, q, cand)
    colsum = q[0].astype(np.float64).sum(axis=0)
    for i in range(N):
        assert sc[0, i] == (i + 1) * colsum[i % d]


# ---------------------------------------------------------------- argument checks of the wrapper
def test_invalid_ids_and_offsets_are_rejected():
    emb, off, q, cand = small_problem(1)
    bad = cand.copy()
    bad[0, 0] = 40
    with pytest.raises(ValueError):
        oracle.scores(emb, off, q, bad)
    bad[0, 0] = -1
    with pytest.raises(ValueError):
        oracle.scores(emb, off, q, bad)
    off2 = off.copy()
    off2[3], off2[4] = off2[4] + 1, off2[3]
    with pytest.raises(ValueError):
        oracle.scores(emb, off2, q, cand)


def test_thread_count_does_not_change_results():
    emb, off, q, cand = small_problem(2, B=6)
    a = oracle.rerank(emb, off, q, cand, 5, threads=1)
    b = oracle.rerank(emb, off, q, cand, 5, threads=4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ================================================================ widened path: partial re-ranking,
# score aggregation, merging, batch threshold
def parse_extras(path):
    out = {"partial": []}
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tag, *rest = line.split()
        if tag == "partial":
            i, j = rest.index("ids"), rest.index("scores")
            out["partial"].append((int(rest[0]), [int(x) for x in rest[i + 1:j]], [float(x) for x in rest[j + 1:]]))
        elif tag == "prior_alpha":
            out["alpha"] = float(rest[0])
        elif tag == "prior":
            out["prior"] = [float(x) for x in rest]
        elif tag == "prior_rank_ids":
            out["prior_ids"] = [int(x) for x in rest]
        elif tag == "prior_rank_scores":
            out["prior_scores"] = [float(x) for x in rest]
    return out


def same_with_nan(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return np.array_equal(np.isnan(a), np.isnan(b)) and np.array_equal(a[~np.isnan(a)], b[~np.isnan(b)])


def test_handworked_partial_reranking():
    path = os.path.join(GOLDEN, "handworked_rerank.txt")
    emb, off, q, cand, _ = parse_rerank(path)
    for R, ids_want, sc_want in parse_extras(path)["partial"]:
        for k in range(0, 6):
            ids, sc = oracle.rerank_partial(emb, off, q, cand, R, k)
            assert ids[0].tolist() == ids_want[:k]
            assert same_with_nan(sc[0], sc_want[:k])


def test_partial_reranking_reduces_to_the_full_ranking_and_to_the_prefix_ranking():
    emb, off, q, cand = small_problem(21, N=60, K=30, B=4)
    K = cand.shape[1]
    full_ids, full_top, _ = oracle.rerank(emb, off, q, cand, K)
    ids, sc = oracle.rerank_partial(emb, off, q, cand, K, K)
    assert np.array_equal(ids, full_ids) and np.array_equal(sc, full_top)
    for R in (1, 7, 16):
        head_ids, head_top, _ = oracle.rerank(emb, off, q, np.ascontiguousarray(cand[:, :R]), R)
        ids, sc = oracle.rerank_partial(emb, off, q, cand, R, K)
        assert np.array_equal(ids[:, :R], head_ids) and np.array_equal(sc[:, :R], head_top)
        assert np.array_equal(ids[:, R:], cand[:, R:]) and np.isnan(sc[:, R:]).all()
        assert all(sorted(r.tolist()) == sorted(c.tolist()) for r, c in zip(ids, cand))   # a permutation of the list
    ids, sc = oracle.rerank_partial(emb, off, q, cand, 0, 9)
    assert np.array_equal(ids, cand[:, :9]) and np.isnan(sc).all()
    with pytest.raises(ValueError):
        oracle.rerank_partial(emb, off, q, cand, K + 1, 3)


def test_handworked_score_aggregation_and_its_special_cases():
    path = os.path.join(GOLDEN, "handworked_rerank.txt")
    emb, off, q, cand, _ = parse_rerank(path)
    ex = parse_extras(path)
    tot = oracle.scores_prior(emb, off, q, cand, np.array([ex["prior"]], dtype=np.float32), ex["alpha"])
    ids, top = oracle.topk(tot, cand, 5)
    assert ids[0].tolist() == ex["prior_ids"] and top[0].tolist() == ex["prior_scores"]
    emb, off, q, cand = small_problem(22, integer=True, lo=1)
    base = oracle.scores(emb, off, q, cand)
    prior = np.random.default_rng(0).integers(-9, 10, size=cand.shape).astype(np.float32)
    assert np.array_equal(oracle.scores_prior(emb, off, q, cand, prior, 0.0), base)            # alpha = 0
    assert np.array_equal(oracle.scores_prior(emb, off, q, cand, prior, 0.5), base + 0.5 * prior)   # exact values
    assert np.array_equal(oracle.scores_prior(emb, off, q, cand, np.zeros_like(prior), 3.0), base)
    a = oracle.scores_prior(emb, off, q, cand, prior, 1.0) + oracle.scores_prior(emb, off, q, cand, -prior, 1.0)
    assert np.array_equal(a, 2 * base)


def test_merging_two_parts_of_a_list_gives_the_ranking_of_the_whole():
    rng = np.random.default_rng(23)
    B, K = 3, 40
    sc = np.round(rng.normal(size=(B, K)), 1)
    ids = np.stack([rng.permutation(500)[:K] for _ in range(B)]).astype(np.int64)
    for cut, k in ((0, 5), (13, 10), (39, 40), (40, 7)):
        want_ids, want_sc = oracle.topk(sc, ids, k)
        got_ids, got_sc = oracle.merge(ids[:, :cut], sc[:, :cut], ids[:, cut:], sc[:, cut:], k)
        assert np.array_equal(got_ids, want_ids) and np.array_equal(got_sc, want_sc)
    # merging ranked top lists of the two parts is enough for the top of the whole
    a_ids, a_sc = oracle.topk(sc[:, :20], ids[:, :20], 6)
    b_ids, b_sc = oracle.topk(sc[:, 20:], ids[:, 20:], 6)
    want_ids, want_sc = oracle.topk(sc, ids, 6)
    got_ids, got_sc = oracle.merge(a_ids, a_sc, b_ids, b_sc, 6)
    assert np.array_equal(got_ids, want_ids) and np.array_equal(got_sc, want_sc)
    # hand-made: a = (5: id 7), (1: id 2); b = (5: id 3), (4: id 9) -> 3, 7, 9, 2
    got_ids, got_sc = oracle.merge([[7, 2]], [[5.0, 1.0]], [[3, 9]], [[5.0, 4.0]], 4)
    assert got_ids.tolist() == [[3, 7, 9, 2]] and got_sc.tolist() == [[5.0, 5.0, 4.0, 1.0]]
    with pytest.raises(ValueError):
        oracle.merge([[7, 2]], [[5.0, 1.0]], [[3, 9]], [[5.0, 4.0]], 5)


def test_batch_threshold_follows_eq4_and_the_papers_own_scaling_statements():
    # the value itself
    assert oracle.batch_threshold(3e9, 0.028, 7e6) == 3e9 * 0.028 / 7e6
    # Sec. 5.4: twice the bandwidth doubles the limit (12 -> "around 24")
    base = oracle.batch_threshold(1.0e9, 0.05, 4.0e6)
    assert oracle.batch_threshold(2.0e9, 0.05, 4.0e6) == 2 * base
    # Sec. 5.5: fetching the top 64 instead of 1000 documents per query cuts the data per query by
    # 1000/64 and raises a limit of 12 to about the 192 the paper reports (187.5)
    limit = 12 * oracle.batch_threshold(1.0, 1.0, 64.0) / oracle.batch_threshold(1.0, 1.0, 1000.0)
    assert abs(limit - 192) / 192 < 0.03


# ================================================================ compressed (E4M3) table
def test_e4m3_decoding_matches_the_format_for_every_code():
    import torch
    want = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()   # torch's own decoder
    got = np.array([oracle.e4m3_to_double(c) for c in range(256)])
    nan = np.isnan(want)
    assert nan.sum() == 2 and np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan]) and np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))
    # values the format's definition fixes: 1.0, the largest finite number, the smallest subnormal and normal
    assert oracle.e4m3_to_double(0x38) == 1.0 and oracle.e4m3_to_double(0x7E) == 448.0
    assert oracle.e4m3_to_double(0x01) == 2.0 ** -9 and oracle.e4m3_to_double(0x08) == 2.0 ** -6
    assert oracle.e4m3_to_double(0xB8) == -1.0 and oracle.e4m3_to_double(0x00) == 0.0


def test_compressed_scores_reduce_to_the_plain_path_on_the_decoded_table():
    # every E4M3 value is exactly a binary16 value, so scoring the codes with scale s must equal
    # s times the (pinned) plain scores of the decoded table when s is a power of two
    rng = np.random.default_rng(31)
    counts = rng.integers(0, 6, size=30)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    codes = rng.integers(0, 256, size=(int(off[-1]), 8), dtype=np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x38                                  # no NaN codes
    decoded = np.array([oracle.e4m3_to_double(c) for c in range(256)])[codes].astype(np.float16)
    assert np.array_equal(decoded.astype(np.float64), np.array([oracle.e4m3_to_double(c) for c in range(256)])[codes])
    q = (rng.integers(-8, 9, size=(2, 3, 8)) / 4).astype(np.float16)
    cand = np.stack([rng.permutation(30)[:12] for _ in range(2)]).astype(np.int64)
    scale = (2.0 ** rng.integers(-3, 4, size=30)).astype(np.float32)
    got = oracle.scores_e4m3(codes, scale, off, q, cand)
    plain = oracle.scores(decoded, off, q, cand)
    want = plain * scale[cand]
    assert np.array_equal(np.isneginf(got), np.isneginf(want))
    fin = ~np.isneginf(want)
    assert np.allclose(got[fin], want[fin], rtol=1e-13, atol=0)
    # a general (not power-of-two) scale is still just a factor on the document's score
    scale2 = (scale * 1.3).astype(np.float32)
    got2 = oracle.scores_e4m3(codes, scale2, off, q, cand)
    assert np.allclose(got2[fin], (plain * scale2[cand].astype(np.float64))[fin], rtol=1e-12, atol=0)
    with pytest.raises(ValueError):
        oracle.scores_e4m3(codes, -scale, off, q, cand)


def test_compression_recipe_round_trips_within_the_format_s_precision():
    import torch
    from paper_2312_05417_amd import synth
    w = synth.scaled(synth.WORKLOADS["c1"], n_docs=300)
    emb, off = synth.table(w)
    codes, scale = synth.compress_e4m3(emb, off)
    assert codes.dtype == torch.uint8 and codes.shape == emb.shape and scale.shape == (300,) and np.all(scale > 0)
    lut = np.array([oracle.e4m3_to_double(c) for c in range(256)])
    assert not np.isnan(lut[codes.numpy()]).any()
    back = lut[codes.numpy()] * np.repeat(scale.astype(np.float64), np.diff(off))[:, None]
    err = np.abs(back - emb.double().numpy())
    amax = np.repeat(scale.astype(np.float64) * 448, np.diff(off))[:, None]
    # 3 fraction bits: relative step 2^-3, so rounding error <= 2^-4 of the value (or of the smallest normal / subnormal step)
    assert np.all(err <= np.maximum(np.abs(emb.double().numpy()) * 2.0 ** -4, amax / 448 * 2.0 ** -10) * (1 + 1e-6))
    assert np.abs(lut[codes.numpy()]).max() == 448.0                       # the largest entry of some document maps to the top code
