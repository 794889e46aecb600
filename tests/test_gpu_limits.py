"""Largest and oddest launch shapes of the scoring path, and what espn_rerank_plan says about them."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_05417_amd import binding as espn
from tests.parity import assert_scores_close, assert_topk_matches
from tests.test_gpu_parity import random_problem

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


@pytest.mark.parametrize("d,B", [(32, 65535), (32, 70003), (128, 66000), (40, 70003)])
def test_very_many_queries_in_one_call(d, B):
    """More queries than a grid dimension other than the first can count (65535): the grids are
    one-dimensional.  d = 40 takes the plain-ALU kernel."""
    K, k = 3, 2
    say("B = %d, K = %d, d = %d" % (B, K, d))
    emb, off, q1, _ = random_problem(9, 500, d, 1, 32, K, 1, 20)
    rng = np.random.default_rng(4)
    cand = rng.integers(0, 500, size=(B, K)).astype(np.int64)
    # a few distinct queries, repeated: the expected scores of every query are then cheap to get
    q_few = random_problem(10, 10, d, 7, 32, 1, 1, 2)[2]
    q = np.ascontiguousarray(q_few[np.arange(B) % 7])
    emb_d, q_d, cand_d = torch.from_numpy(emb).to(DEV), torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    table = espn.espn_table_load(emb_d, off)
    g_all = espn.espn_score(table, q_d, cand_d)
    g_ids, g_sc = espn.espn_rerank(table, q_d, cand_d, k)
    p_ids, p_sc = espn.espn_rerank_partial(table, q_d, cand_d, 2, 3)       # two ranked, the third appended
    espn.espn_table_check(table)
    sample = np.array([0, 1, 6, 7, 32767, 65533, 65534, B - 2, B - 1])
    o_all = oracle.scores(emb, off, np.ascontiguousarray(q[sample]), np.ascontiguousarray(cand[sample]))
    assert_scores_close(g_all[sample].cpu().numpy(), o_all, 32)
    for n, b in enumerate(sample):
        assert_topk_matches(g_ids[b].cpu().numpy(), g_sc[b].cpu().numpy(), o_all[n], cand[b], k, 32)
    # every query against the two-launch path
    t_ids, t_sc = espn.espn_topk(g_all, cand_d, k)
    assert torch.equal(g_ids, t_ids) and torch.equal(g_sc.view(torch.int32), t_sc.view(torch.int32))
    # partial re-ranking: the appended rank is the third candidate of every list, unscored
    assert torch.equal(p_ids[:, 2], cand_d[:, 2]) and bool(torch.isnan(p_sc[:, 2]).all())
    h_ids, h_sc = espn.espn_topk(g_all[:, :2].contiguous(), cand_d[:, :2].contiguous(), 2)
    assert torch.equal(p_ids[:, :2], h_ids) and torch.equal(p_sc[:, :2].view(torch.int32), h_sc.view(torch.int32))
    table.free()


def test_more_pairs_than_a_grid_can_count_are_refused():
    """B * K beyond 2^31 - 1 is refused before anything is launched (the pointers are never read)."""
    emb, off, q1, _ = random_problem(9, 50, 32, 1, 32, 1, 1, 5)
    table = espn.espn_table_load(torch.from_numpy(emb).to(DEV), off)
    B, K = 70000, 40000
    lib = espn.lib()
    dummy = torch.zeros(16, dtype=torch.int64, device=DEV)
    rc = lib.espn_score(table.handle, dummy.data_ptr(), dummy.data_ptr(), B, 32, K, dummy.data_ptr(), None)
    assert rc == espn.ESPN_ERR_UNSUPPORTED, espn.last_error()
    table.free()


@pytest.mark.parametrize("d", [32, 128])
def test_one_query_with_a_very_long_list(d):
    K, k = 70001, 25
    say("B = 1, K = %d, d = %d: hundreds of slices of one query" % (K, d))
    emb, off, q, _ = random_problem(3, 3000, d, 1, 32, 1, 1, 12)
    cand = np.random.default_rng(8).integers(0, 3000, size=(1, K)).astype(np.int64)     # with repeats
    emb_d, q_d, cand_d = torch.from_numpy(emb).to(DEV), torch.from_numpy(q).to(DEV), torch.from_numpy(cand).to(DEV)
    table = espn.espn_table_load(emb_d, off)
    plan = espn.espn_rerank_plan(table, 1, 32, K, k)
    assert plan["slices"] * plan["slice"] >= K > (plan["slices"] - 1) * plan["slice"] and plan["slice"] <= 1024
    assert plan["launches"] == 2
    g_all = espn.espn_score(table, q_d, cand_d).cpu().numpy()
    g_ids, g_sc = espn.espn_rerank(table, q_d, cand_d, k)
    espn.espn_table_check(table)
    o_all = oracle.scores(emb, off, q, cand)
    assert_scores_close(g_all, o_all, 32)
    # 70 001 draws from 3000 documents: every score appears ~23 times, so the head is all exact ties
    ids, sc = g_ids[0].cpu().numpy(), g_sc[0].cpu().numpy()
    order = np.lexsort((cand[0], -g_all[0]))
    assert np.array_equal(ids, cand[0][order[:k]]) and np.array_equal(sc, g_all[0][order[:k]])
    table.free()


def test_plan_of_typical_shapes():
    say("espn_rerank_plan on the benchmark shapes")
    emb = torch.zeros((64, 32), dtype=torch.float16, device=DEV)
    t32 = espn.espn_table_load(emb, np.array([0, 64], dtype=np.int64))
    emb128 = torch.zeros((64, 128), dtype=torch.float16, device=DEV)
    t128 = espn.espn_table_load(emb128, np.array([0, 64], dtype=np.int64))
    emb72 = torch.zeros((64, 72), dtype=torch.float16, device=DEV)
    t72 = espn.espn_table_load(emb72, np.array([0, 64], dtype=np.int64))
    for table, B, K, k in ((t32, 64, 1000, 10), (t32, 8, 100, 10), (t32, 1024, 64, 10), (t128, 256, 1000, 10),
                           (t128, 2048, 1000, 10), (t128, 4096, 64, 10), (t32, 1, 1, 1), (t128, 3, 5000, 0)):
        p = espn.espn_rerank_plan(table, B, 32, K, k)
        assert 1 <= p["slice"] <= 1024 and p["slices"] * p["slice"] >= K > (p["slices"] - 1) * p["slice"], p
        one_launch = p["slices"] == 1 and K <= 256 and k >= 1
        assert p["launches"] == (1 if one_launch or k == 0 else 2), (B, K, k, p)
    # a batch that fits the device at once is cut to fill it once: 64 queries x 8 slices = 512 workgroups
    assert espn.espn_rerank_plan(t32, 64, 32, 1000, 10) == {"slices": 8, "slice": 125, "launches": 2}
    assert espn.espn_rerank_plan(t32, 1024, 32, 64, 10) == {"slices": 1, "slice": 64, "launches": 1}
    # the cut never makes more workgroups than the device holds at once: 192 queries x 2 slices, not x 3
    assert espn.espn_rerank_plan(t32, 200, 32, 256, 10) == {"slices": 2, "slice": 128, "launches": 2}
    assert espn.espn_rerank_plan(t32, 192, 32, 256, 10) == {"slices": 4, "slice": 64, "launches": 2}      # 3 per compute unit
    assert espn.espn_rerank_plan(t32, 192, 32, 1000, 10) == {"slices": 4, "slice": 250, "launches": 2}
    assert espn.espn_rerank_plan(t128, 136, 32, 400, 10) == {"slices": 3, "slice": 134, "launches": 2}
    assert espn.espn_rerank_plan(t128, 300, 32, 400, 10) == {"slices": 2, "slice": 200, "launches": 2}
    # (the limits for rows longer than 64 bytes depend on how the rows are fetched: say which, this table of one
    # document would otherwise count as one whose lists share documents)
    espn.espn_table_set_fetch(t128, espn.ESPN_FETCH_STREAMING)
    # lists that the waves of one workgroup finish in a few documents each are not cut, whatever the batch:
    # the scoring kernel ranks them (64-byte rows: 5 documents per wave of 16, longer rows: 2 per wave of 8)
    assert espn.espn_rerank_plan(t32, 8, 32, 64, 10) == {"slices": 1, "slice": 64, "launches": 1}
    assert espn.espn_rerank_plan(t128, 8, 32, 16, 10) == {"slices": 1, "slice": 16, "launches": 1}
    assert espn.espn_rerank_plan(t128, 8, 32, 17, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t32, 8, 32, 80, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t32, 8, 32, 81, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t32, 8, 32, 64, 0)["slices"] > 1          # scoring alone is still spread out
    # ... and longer lists stay whole from half a workgroup per compute unit on, where the cut has little left to
    # spread the queries to (not where some compute units would get two workgroups and others one)
    assert espn.espn_rerank_plan(t32, 192, 32, 112, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t32, 150, 32, 112, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t32, 300, 32, 112, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t32, 400, 32, 112, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t128, 100, 32, 32, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t128, 192, 32, 64, 10) == {"slices": 1, "slice": 64, "launches": 1}
    assert espn.espn_rerank_plan(t128, 192, 32, 128, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t128, 170, 32, 128, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t128, 300, 32, 64, 10)["launches"] == 2
    # rows longer than 64 bytes are cut for ONE workgroup per compute unit (64-byte rows: two), and may leave
    # half the waves of a workgroup without a document
    assert espn.espn_rerank_plan(t128, 64, 32, 300, 10) == {"slices": 4, "slice": 75, "launches": 2}
    assert espn.espn_rerank_plan(t32, 64, 32, 300, 10) == {"slices": 8, "slice": 38, "launches": 2}
    assert espn.espn_rerank_plan(t128, 20, 32, 128, 10) == {"slices": 12, "slice": 11, "launches": 2}
    assert espn.espn_rerank_plan(t128, 8, 32, 128, 10) == {"slices": 32, "slice": 4, "launches": 2}
    assert espn.espn_rerank_plan(t128, 150, 32, 300, 10) == {"slices": 3, "slice": 100, "launches": 2}
    # 171 to 255 queries: the slice count whose workgroups come closest, from below, to a whole number per compute
    # unit; a full device's worth of queries keeps the fixed slices (the c3 shape)
    assert espn.espn_rerank_plan(t128, 192, 32, 600, 10) == {"slices": 4, "slice": 150, "launches": 2}
    assert espn.espn_rerank_plan(t128, 200, 32, 600, 10) == {"slices": 5, "slice": 120, "launches": 2}
    assert espn.espn_rerank_plan(t128, 210, 32, 600, 10) == {"slices": 6, "slice": 100, "launches": 2}
    assert espn.espn_rerank_plan(t128, 240, 32, 600, 10) == {"slices": 4, "slice": 150, "launches": 2}
    assert espn.espn_rerank_plan(t128, 256, 32, 1000, 10) == {"slices": 16, "slice": 63, "launches": 2}
    # rows fetched with ordinary loads (lists that share documents): a document costs more while the launch is
    # short, so the lists of few queries are cut sooner; from 171 queries on the limits are the same
    espn.espn_table_set_fetch(t128, espn.ESPN_FETCH_CACHED)
    assert espn.espn_rerank_plan(t128, 16, 32, 16, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t128, 16, 32, 8, 5)["launches"] == 1
    assert espn.espn_rerank_plan(t128, 100, 32, 32, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t128, 150, 32, 64, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t128, 192, 32, 128, 10)["launches"] == 1
    espn.espn_table_set_fetch(t128, espn.ESPN_FETCH_AUTO)
    assert espn.espn_rerank_plan(t128, 400, 32, 64, 10)["launches"] == 1
    # rows of 32 E4M3 codes: the cut list is cheaper there, so the limits are lower
    codes = torch.zeros((64, 32), dtype=torch.uint8, device=DEV)
    t32c = espn.espn_table_load_e4m3(codes, np.ones(1, dtype=np.float32), np.array([0, 64], dtype=np.int64))
    assert espn.espn_rerank_plan(t32c, 8, 32, 64, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t32c, 8, 32, 80, 10)["launches"] == 2
    assert espn.espn_rerank_plan(t32c, 192, 32, 80, 10)["launches"] == 1
    assert espn.espn_rerank_plan(t32c, 192, 32, 96, 10)["launches"] == 2
    t32c.free()
    # shapes the matrix-core kernel does not take: one wave per candidate, a second launch ranks
    assert espn.espn_rerank_plan(t72, 5, 32, 40, 3) == {"slices": 40, "slice": 1, "launches": 2}
    assert espn.espn_rerank_plan(t32, 5, 65, 40, 3) == {"slices": 40, "slice": 1, "launches": 2}
    # up to 64 query rows run on the matrix cores
    assert espn.espn_rerank_plan(t32, 5, 64, 40, 3) == espn.espn_rerank_plan(t32, 5, 32, 40, 3)
    assert espn.espn_rerank_plan(t32, 0, 32, 40, 3) == {"slices": 0, "slice": 0, "launches": 0}
    with pytest.raises(espn.EspnError):
        espn.espn_rerank_plan(t32, 4, 32, 10, 11)
    for t in (t32, t128, t72):
        t.free()


def test_plans_and_kernels_of_the_workloads_are_pinned():
    """The slice plan and the kernel instantiations of every benchmark workload, as espn_rerank_plan and
    espn_rerank_plan_kernels report them: later tuning of the planner cannot change them unnoticed.  (The fetch
    mode is set by hand because these one-document tables are too small for the library's own rule.)"""
    say("plans of the workloads")
    S, C = espn.ESPN_FETCH_STREAMING, espn.ESPN_FETCH_CACHED
    t32 = espn.espn_table_load(torch.zeros((64, 32), dtype=torch.float16, device=DEV), np.array([0, 64], dtype=np.int64))
    t128 = espn.espn_table_load(torch.zeros((64, 128), dtype=torch.float16, device=DEV), np.array([0, 64], dtype=np.int64))
    c32 = espn.espn_table_load_e4m3(torch.zeros((64, 32), dtype=torch.uint8, device=DEV), np.ones(1, dtype=np.float32),
                                    np.array([0, 64], dtype=np.int64))
    c128 = espn.espn_table_load_e4m3(torch.zeros((64, 128), dtype=torch.uint8, device=DEV), np.ones(1, dtype=np.float32),
                                     np.array([0, 64], dtype=np.int64))
    want = [
        # workload, table, fetch, B, K scored, k -> slices, slice, launches, kernels
        ("c1", t32, S, 8, 100, 10, 6, 17, 2, ["espn::maxsim_slice_kernel<32, 16, 4, 2, false, 2, true>", "espn::topk_wave_kernel<4>"]),
        ("c2", t32, S, 64, 1000, 10, 8, 125, 2, ["espn::maxsim_slice_kernel<32, 16, 4, 2, false, 2, true>", "espn::topk_wave_kernel<16>"]),
        ("c3", t128, S, 256, 1000, 10, 16, 63, 2, ["espn::maxsim_slice_kernel<128, 4, 4, 2, false, 2, true>", "espn::topk_wave_kernel<16>"]),
        ("c4", t128, C, 2048, 1000, 10, 16, 63, 2, ["espn::maxsim_slice_kernel<128, 4, 4, 2, false, 2, false>", "espn::topk_wave_kernel<16>"]),
        ("c5 (a staged batch is scored like c4 at half the queries)", t128, C, 1024, 1000, 10, 16, 63, 2,
         ["espn::maxsim_slice_kernel<128, 4, 4, 2, false, 2, false>", "espn::topk_wave_kernel<16>"]),
        ("c2p64", t32, S, 1024, 64, 10, 1, 64, 1, ["espn::maxsim_slice_kernel<32, 8, 4, 2, true, 2, true>"]),
        ("c3p64", t128, S, 4096, 64, 10, 1, 64, 1, ["espn::maxsim_slice_kernel<128, 4, 4, 2, true, 2, true>"]),
        ("c2e4m3", c32, S, 64, 1000, 10, 8, 125, 2, ["espn::maxsim_slice_kernel<32, 16, 4, 1, false, 2, true>", "espn::topk_wave_kernel<16>"]),
        ("c3e4m3", c128, S, 256, 1000, 10, 16, 63, 2, ["espn::maxsim_slice_kernel<128, 8, 4, 1, false, 2, true>", "espn::topk_wave_kernel<16>"]),
    ]
    wrong = []
    for name, table, fetch, B, K, k, slices, slice_, launches, kernels in want:
        espn.espn_table_set_fetch(table, fetch)
        got = (espn.espn_rerank_plan(table, B, 32, K, k), espn.espn_rerank_plan_kernels(table, B, 32, K, k))
        if got != ({"slices": slices, "slice": slice_, "launches": launches}, kernels):
            wrong.append((name, got))
    assert not wrong, wrong
    # scoring alone (k = 0) names one kernel, an empty batch none, other shapes the plain kernel or a sort
    assert espn.espn_rerank_plan_kernels(t32, 64, 32, 1000, 0) == ["espn::maxsim_slice_kernel<32, 16, 4, 2, false, 2, true>"]
    assert espn.espn_rerank_plan_kernels(t32, 0, 32, 1000, 10) == []
    assert espn.espn_rerank_plan_kernels(t32, 64, 65, 1000, 100) == ["espn::maxsim_generic_kernel",
                                                                    "espn::topk_sort_kernel<1024, 256, espn::OneList>"]
    assert espn.espn_rerank_plan_kernels(t128, 3, 48, 5000, 10)[1] == "espn::topk_rounds_kernel<16>"
    for t in (t32, t128, c32, c128):
        t.free()
