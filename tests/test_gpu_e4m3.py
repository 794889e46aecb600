"""Compressed (E4M3 + per-document scale) tables: HIP path vs the fp64 oracle."""
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


def check(codes, scale, off, q, cand, k, Q, fetch=None):
    """codes uint8 numpy, scale fp32 numpy, off, q fp16 numpy, cand int64 numpy; fetch: a mode for
    espn_table_set_fetch, or None for the library's default."""
    o_all = oracle.scores_e4m3(codes, scale, off, q, cand)
    o_ids, o_top = oracle.topk(o_all, cand, k)
    codes_d = torch.from_numpy(codes).to(DEV) if codes.size else torch.zeros((0, codes.shape[1]), dtype=torch.uint8, device=DEV)
    table = espn.espn_table_load_e4m3(codes_d, scale, off)
    if fetch is not None:
        espn.espn_table_set_fetch(table, fetch)
    q_d, cand_d = torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    g_all = espn.espn_score(table, q_d, cand_d).cpu().numpy()
    g_ids, g_top = espn.espn_rerank(table, q_d, cand_d, k)
    espn.espn_table_check(table)
    worst = assert_scores_close(g_all, o_all, Q)
    for b in range(q.shape[0]):
        assert_topk_matches(g_ids[b].cpu().numpy(), g_top[b].cpu().numpy(), o_all[b], cand[b], k, Q)
    table.free()
    return worst, g_all, o_all


@pytest.mark.parametrize("d", [32, 128])
def test_every_code_in_every_component_position(d):
    # documents of one row; row j carries code (j + c) mod 256 in component c (NaN codes replaced), and
    # the query picks single components, so a wrong byte order or a wrong decode of any code shows
    say("all codes, d=%d" % d)
    n = 256
    codes = ((np.arange(n)[:, None] + np.arange(d)[None, :]) % 256).astype(np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x3C
    off = np.arange(n + 1, dtype=np.int64)
    scale = np.ones(n, dtype=np.float32)
    lut = np.array([oracle.e4m3_to_double(c) for c in range(256)])
    for comps in ([0, 1, 2, 3, 4, 5, 6, 7], list(range(d - 8, d)), [9, 17, 30, 31 if d == 32 else 77]):
        q = np.zeros((1, len(comps), d), dtype=np.float16)
        for i, c in enumerate(comps):
            q[0, i, c] = 1.0
        cand = np.arange(n, dtype=np.int64)[None]
        worst, g_all, o_all = check(codes, scale, off, q, cand, 10, len(comps))
        want = lut[codes[:, comps]].sum(axis=1)                  # one row per document: the max is the row itself
        assert np.array_equal(g_all[0].astype(np.float64), want)           # sums of a few E4M3 values: exact in fp32
    say("ok")


@pytest.mark.parametrize("key,changes", [("c1", {}), ("c3", dict(n_docs=4000, B=5, K=300)),
                                         ("c2", dict(n_docs=20000, B=3, K=1000))])
def test_compressed_workloads_match_the_oracle(key, changes):
    w = synth.scaled(synth.WORKLOADS[key], **changes)
    say("E4M3 %s d=%d N=%d B=%d K=%d" % (w.name, w.dim, w.n_docs, w.B, w.K))
    emb, off = synth.table(w)
    codes, scale = synth.compress_e4m3(emb, off)
    q, cand = synth.queries(w).numpy(), synth.candidates(w)
    worst, g_all, o_all = check(codes.numpy(), scale, off, q, cand, w.k, w.Q)
    say("worst relative error %.2e" % worst)
    assert worst < 1e-4
    # the compressed scores stay close to the uncompressed ones (3 fraction bits per component)
    plain = oracle.scores(emb.numpy(), off, q, cand)
    assert np.abs(o_all - plain).max() < 0.6 and np.corrcoef(o_all.ravel(), plain.ravel())[0, 1] > 0.98


@pytest.mark.parametrize("d,Q", [(32, 1), (32, 17), (128, 7), (128, 32), (32, 33), (32, 64), (128, 48), (128, 64)])
def test_ragged_documents_scales_and_empty_documents(d, Q):
    say("E4M3 ragged d=%d Q=%d" % (d, Q))
    rng = np.random.default_rng(d + Q)
    counts = np.array([0, 1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 64, 65, 100, 128, 129, 179, 180, 0] * 5)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    codes = rng.integers(0, 256, size=(int(off[-1]), d), dtype=np.uint8)
    codes[(codes & 0x7F) == 0x7F] = 0x12
    codes[(codes & 0x78) == 0x78] &= 0xB7                       # keep magnitudes moderate (below 256)
    scale = rng.uniform(1e-3, 3.0, size=counts.size).astype(np.float32)
    q = rng.normal(size=(3, Q, d)).astype(np.float16)
    cand = np.stack([rng.permutation(counts.size)[:77] for _ in range(3)]).astype(np.int64)
    worst, g_all, o_all = check(codes, scale, off, q, cand, 77, Q)
    assert np.isneginf(g_all[counts[cand] == 0]).all()
    # both ways of fetching the rows, forced (the default picks one from the batch's size): the lane-linear
    # streaming loads with their partial last tiles and the ordinary loads give the same bits
    for mode in (espn.ESPN_FETCH_STREAMING, espn.ESPN_FETCH_CACHED):
        _, g_mode, _ = check(codes, scale, off, q, cand, 77, Q, fetch=mode)
        assert np.array_equal(g_mode.view(np.int32), g_all.view(np.int32)), mode


def test_host_resident_compressed_table():
    w = synth.scaled(synth.WORKLOADS["c5"], n_docs=20_000, B=16, K=300)
    say("E4M3 host-resident d=%d" % w.dim)
    emb, off = synth.table(w)
    codes, scale = synth.compress_e4m3(emb, off)
    pinned = torch.empty(codes.shape, dtype=torch.uint8, pin_memory=True)
    pinned.copy_(codes)
    table = espn.espn_table_load_e4m3(pinned, scale, off)
    espn.espn_staging_create(table, int(off[-1]), w.n_docs)
    side = torch.cuda.Stream()
    before = np.zeros(0, dtype=np.int64)      # documents the other slot holds
    for n in range(3):
        cand = synth.candidates(w, batch=n)
        q = synth.queries(w, batch=n)
        cand_d = torch.from_numpy(cand).to(DEV)
        espn.espn_prefetch(table, cand_d, n % 2, side)
        ids, top, ws = espn.espn_rerank_staged(table, n % 2, q.to(DEV), cand_d, w.k)
        torch.cuda.synchronize()
        espn.espn_table_check(table)
        o_all = oracle.scores_e4m3(codes.numpy(), scale, off, q.numpy(), cand)
        g_all = ws[: 4 * w.B * w.K].view(torch.float32).view(w.B, w.K).cpu().numpy()
        assert_scores_close(g_all, o_all, w.Q)
        for b in range(w.B):
            assert_topk_matches(ids[b].cpu().numpy(), top[b].cpu().numpy(), o_all[b], cand[b], w.k, w.Q)
        u = np.unique(cand)
        fresh = np.setdiff1d(u, before)       # one byte per component crosses PCIe, once per document
        c = espn.espn_staging_counters(table, n % 2)
        assert c["distinct_docs"] == u.size and c["pcie_bytes"] == int((off[fresh + 1] - off[fresh]).sum()) * w.dim
        before = u
    table.free()


def test_loading_rejects_bad_scales_and_dims():
    codes = torch.zeros((16, 32), dtype=torch.uint8, device=DEV)
    off = np.array([0, 16], dtype=np.int64)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_load_e4m3(codes, np.array([0.0], dtype=np.float32), off)
    assert ei.value.status == espn.ESPN_ERR_ARG
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_load_e4m3(codes, np.array([np.inf], dtype=np.float32), off)
    assert ei.value.status == espn.ESPN_ERR_ARG
    codes64 = torch.zeros((16, 64), dtype=torch.uint8, device=DEV)
    with pytest.raises(espn.EspnError) as ei:
        espn.espn_table_load_e4m3(codes64, np.array([1.0], dtype=np.float32), off)
    assert ei.value.status == espn.ESPN_ERR_UNSUPPORTED
