"""Seeded random launch shapes through the whole path against the fp64 oracle: query length, list
length, batch size, k, document-length law (with empty documents, single rows, tile-straddling
lengths and a few very long documents), for both matrix-core row lengths and both codecs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_05417_amd import binding as espn
from paper_2312_05417_amd import synth
from tests.parity import assert_scores_close, assert_topk_matches, cancellation_floor

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([32, 128, 32, 128, 64, 192]))
    Q = int(rng.choice([1, 2, 5, 15, 16, 17, 31, 32]))
    B = int(rng.choice([1, 2, 3, 7, 33, 130, 600]))
    K = int(rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 127, 200, 256, 257, 511, 1000, 1500, 2049]))
    if B * K > 300_000:
        B = max(1, 300_000 // K)
    k = int(rng.choice([0, 1, 2, 10, 64, 65, K]))
    k = min(k, K)
    N = int(rng.choice([1, 3, 50, 2000]))
    law = int(rng.integers(0, 4))
    if law == 0:
        counts = rng.integers(0, 40, size=N)                       # short, some empty
    elif law == 1:
        counts = rng.choice([0, 1, 15, 16, 17, 31, 32, 33, 48, 64], size=N)   # around the 16-row tile
    elif law == 2:
        counts = np.clip(rng.lognormal(np.log(40) - 0.125, 0.5, size=N).round(), 4, 128).astype(np.int64)
    else:
        counts = rng.integers(1, 12, size=N)
        counts[rng.integers(0, N, size=max(1, N // 50))] = rng.integers(300, 700)   # a few very long ones
    counts = counts.astype(np.int64)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    x = rng.normal(size=(int(off[-1]), d)).astype(np.float32) * rng.choice([0.05, 1.0, 7.0])
    qq = rng.normal(size=(B, Q, d)).astype(np.float32) * rng.choice([0.1, 1.0, 3.0])
    cand = rng.integers(0, N, size=(B, K)).astype(np.int64)        # with repeats
    return d, Q, B, K, k, N, x.astype(np.float16), off, qq.astype(np.float16), cand


@pytest.mark.parametrize("seed", range(40))
def test_random_shape(seed):
    d, Q, B, K, k, N, emb, off, q, cand = draw_case(seed)
    say("seed %d: d=%d Q=%d B=%d K=%d k=%d N=%d rows=%d" % (seed, d, Q, B, K, k, N, emb.shape[0]))
    emb_d = torch.from_numpy(emb).to(DEV) if emb.shape[0] else torch.zeros((0, d), dtype=torch.float16, device=DEV)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    table = espn.espn_table_load(emb_d, off)
    g_all = espn.espn_score(table, q_d, cand_d)
    g_ids, g_top = espn.espn_rerank(table, q_d, cand_d, k)
    espn.espn_table_check(table)
    # the whole path against scoring + the stand-alone ranking kernel: bit for bit, every query
    t_ids, t_top = espn.espn_topk(g_all, cand_d, k)
    assert torch.equal(g_ids, t_ids) and torch.equal(g_top.view(torch.int32), t_top.view(torch.int32))
    # against the oracle: all scores; ranks on a sample of queries
    o_all = oracle.scores(emb, off, q, cand)
    # short queries against short documents: maxima of both signs can cancel (see cancellation_floor)
    floor = cancellation_floor(oracle.scores(np.abs(emb), off, np.abs(q), cand), d, Q)
    assert_scores_close(g_all.cpu().numpy(), o_all, Q, floor=floor)
    ids, top = g_ids.cpu().numpy(), g_top.cpu().numpy()
    for b in sorted(set([0, B // 2, B - 1])):
        assert_topk_matches(ids[b], top[b], o_all[b], cand[b], k, Q, floor=floor[b])
    table.free()


@pytest.mark.parametrize("seed", range(16))
def test_random_shape_with_long_queries(seed):
    """The same shapes with 33 to 64 query rows (rows of up to 128 components keep them on the matrix cores, 192
    sends them to the plain-ALU kernel)."""
    d, _, B, K, k, N, emb, off, _, cand = draw_case(200 + seed)
    rng = np.random.default_rng(5000 + seed)
    Q = int(rng.choice([33, 40, 47, 48, 49, 63, 64]))
    B = min(B, 40)
    cand = np.ascontiguousarray(cand[:B])
    q = (rng.normal(size=(B, Q, d)) * rng.choice([0.1, 1.0, 3.0])).astype(np.float16)
    say("long query, seed %d: d=%d Q=%d B=%d K=%d k=%d N=%d rows=%d" % (seed, d, Q, B, K, k, N, emb.shape[0]))
    emb_d = torch.from_numpy(emb).to(DEV) if emb.shape[0] else torch.zeros((0, d), dtype=torch.float16, device=DEV)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    table = espn.espn_table_load(emb_d, off)
    g_all = espn.espn_score(table, q_d, cand_d)
    g_ids, g_top = espn.espn_rerank(table, q_d, cand_d, k)
    espn.espn_table_check(table)
    t_ids, t_top = espn.espn_topk(g_all, cand_d, k)
    assert torch.equal(g_ids, t_ids) and torch.equal(g_top.view(torch.int32), t_top.view(torch.int32))
    o_all = oracle.scores(emb, off, q, cand)
    floor = cancellation_floor(oracle.scores(np.abs(emb), off, np.abs(q), cand), d, Q)
    assert_scores_close(g_all.cpu().numpy(), o_all, Q, floor=floor)
    ids, top = g_ids.cpu().numpy(), g_top.cpu().numpy()
    for b in sorted(set([0, B // 2, B - 1])):
        assert_topk_matches(ids[b], top[b], o_all[b], cand[b], k, Q, floor=floor[b])
    table.free()


@pytest.mark.parametrize("seed", range(8))
def test_random_shape_compressed(seed):
    # the first draw of this seed's sequence that a compressed table can hold (rows of 32 or 128 components, not empty)
    for attempt in range(200):
        d, Q, B, K, k, N, emb, off, q, cand = draw_case(100 + seed + 1000 * attempt)
        if emb.shape[0] > 0 and d in (32, 128):
            break
    else:
        raise AssertionError("no compressible shape in 200 draws")
    say("e4m3 seed %d: d=%d Q=%d B=%d K=%d k=%d N=%d" % (seed, d, Q, B, K, k, N))
    codes, scale = synth.compress_e4m3(torch.from_numpy(emb), off)
    table = espn.espn_table_load_e4m3(codes.to(DEV), scale, off)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    g_all = espn.espn_score(table, q_d, cand_d)
    g_ids, g_top = espn.espn_rerank(table, q_d, cand_d, k)
    espn.espn_table_check(table)
    t_ids, t_top = espn.espn_topk(g_all, cand_d, k)
    assert torch.equal(g_ids, t_ids) and torch.equal(g_top.view(torch.int32), t_top.view(torch.int32))
    o_all = oracle.scores_e4m3(codes.numpy(), scale, off, q, cand)
    magnitude = oracle.scores_e4m3(codes.numpy() & 0x7F, scale, off, np.abs(q), cand)     # sign bits cleared
    assert_scores_close(g_all.cpu().numpy(), o_all, Q, floor=cancellation_floor(magnitude, d, Q))
    table.free()


@pytest.mark.parametrize("seed", range(24))
def test_random_shape_partial_and_with_a_prior(seed):
    """The same shapes through partial re-ranking (Sec. 4.4; a random prefix length R) and through the
    aggregated score (Sec. 3.1; a random prior and weight)."""
    for attempt in range(200):          # the first draw of this seed's sequence whose table is not empty
        d, Q, B, K, k, N, emb, off, q, cand = draw_case(300 + seed + 1000 * attempt)
        if emb.shape[0] > 0:
            break
    else:
        raise AssertionError("no non-empty table in 200 draws")
    rng = np.random.default_rng(31000 + seed)
    B = min(B, 50)
    cand, q = np.ascontiguousarray(cand[:B]), np.ascontiguousarray(q[:B])
    R = min(K, int(rng.choice([0, 1, 16, 64, 128, 256, 257, K // 2, K])))
    alpha = float(rng.choice([0.0, 0.5, -2.0]))
    say("partial / prior, seed %d: d=%d Q=%d B=%d K=%d k=%d R=%d alpha=%g N=%d" % (seed, d, Q, B, K, k, R, alpha, N))
    table = espn.espn_table_load(torch.from_numpy(emb).to(DEV), off)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)

    o_ids, o_sc = oracle.rerank_partial(emb, off, q, cand, R, k)
    g_ids, g_sc = espn.espn_rerank_partial(table, q_d, cand_d, R, k)
    espn.espn_table_check(table)
    g_ids, g_sc = g_ids.cpu().numpy(), g_sc.cpu().numpy()
    head = min(R, k)
    # the appended tail is integer work: exact, and its scores are NaN on both sides
    assert np.array_equal(g_ids[:, head:], o_ids[:, head:]) and np.array_equal(g_ids[:, head:], cand[:, head:k])
    assert np.isnan(g_sc[:, head:]).all() and np.isnan(o_sc[:, head:]).all()
    if head:
        prefix = np.ascontiguousarray(cand[:, :R])
        o_all = oracle.scores(emb, off, q, prefix)
        floor = cancellation_floor(oracle.scores(np.abs(emb), off, np.abs(q), prefix), d, Q)
        for b in sorted(set([0, B // 2, B - 1])):
            assert_topk_matches(g_ids[b, :head], g_sc[b, :head], o_all[b], prefix[b], head, Q, floor=floor[b])

    prior = (rng.normal(size=cand.shape) * 4).astype(np.float32)
    o_tot = oracle.scores_prior(emb, off, q, cand, prior, alpha)
    p_ids, p_top, ws = espn.espn_rerank_prior(table, q_d, cand_d, torch.from_numpy(prior).to(DEV), alpha, k)
    espn.espn_table_check(table)
    g_tot = ws[: 4 * B * K].view(torch.float32).view(B, K)
    got = g_tot.cpu().numpy().astype(np.float64)
    assert np.array_equal(np.isneginf(got), np.isneginf(o_tot))
    # relative to the magnitudes that were added (the total itself may cancel to nearly nothing)
    added = np.abs(oracle.scores(emb, off, q, cand)) + abs(alpha) * np.abs(prior)
    tol = np.maximum(1e-3 * np.maximum(added, 1e-6 * Q),
                     cancellation_floor(oracle.scores(np.abs(emb), off, np.abs(q), cand), d, Q))
    fin = np.isfinite(o_tot)
    assert np.all(np.abs(got[fin] - o_tot[fin]) <= tol[fin])
    # the ranks of these totals: bit for bit those of the stand-alone ranking kernel on the same numbers
    r_ids, r_top = espn.espn_topk(g_tot.contiguous(), cand_d, k)
    assert torch.equal(p_ids, r_ids) and torch.equal(p_top.view(torch.int32), r_top.view(torch.int32))
    table.free()
