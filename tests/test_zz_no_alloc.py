"""espn_rerank_noalloc (the entry point that allocates nothing: the scores of a batch go to an array
inside the library's code object) against espn_rerank, through the C ABI.  Same kernels, so the bar is
bit equality; two calls in a row on one device, the second smaller than the first, so that whatever the
first left in the shared array would show."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(lib, espn, table, w, synth, seed, B, K, k, dev, st):
    ws = synth.scaled(w, B=B, K=K, k=k)
    q = synth.queries(ws, seed, 0, device=dev)
    cand = torch.from_numpy(synth.candidates(ws, seed, 0)).to(dev)
    # reference: the existing entry point with a caller-owned workspace
    want_ids = torch.full((B, k), -7, dtype=torch.int64, device=dev)
    want_sc = torch.full((B, k), -7.0, dtype=torch.float32, device=dev)
    nbytes = int(lib.espn_workspace_bytes(B, K))
    wsp = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    rc = lib.espn_rerank(table.handle, q.data_ptr(), cand.data_ptr(), B, ws.Q, K, k, want_ids.data_ptr(),
                         want_sc.data_ptr(), wsp.data_ptr(), nbytes, st)
    assert rc == 0, espn.last_error()
    got_ids = torch.full((B, k), -9, dtype=torch.int64, device=dev)
    got_sc = torch.full((B, k), -9.0, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(dev)
    rc = lib.espn_rerank_noalloc(table.handle, q.data_ptr(), cand.data_ptr(), B, ws.Q, K, k, got_ids.data_ptr(),
                                 got_sc.data_ptr(), st)
    assert rc == 0, espn.last_error()
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(dev) == before
    espn.espn_table_check(table)
    assert torch.equal(got_ids, want_ids)
    assert np.array_equal(got_sc.cpu().numpy().view(np.uint32), want_sc.cpu().numpy().view(np.uint32))
    return got_ids


@pytest.mark.parametrize("key,n_docs,first,second", [
    ("c2", 30000, (24, 1000, 10), (5, 300, 7)),        # 64-byte rows, two launches (scores, then ranking)
    ("c3", 6000, (12, 700, 10), (3, 16, 4)),           # 256-byte rows; the second list is short enough for one launch
])
def test_noalloc_equals_rerank_twice_in_a_row(key, n_docs, first, second):
    from paper_2312_05417_amd import binding as espn, synth
    dev = torch.device("cuda:0")
    lib = espn.lib()
    w = synth.scaled(synth.WORKLOADS[key], n_docs=n_docs)
    seed = 77
    emb, off = synth.table(w, seed, device=dev)
    table = espn.espn_table_load(emb, off)
    st = int(torch.cuda.current_stream().cuda_stream)
    a = _case(lib, espn, table, w, synth, seed, *first, dev, st)
    b = _case(lib, espn, table, w, synth, seed + 1, *second, dev, st)
    assert a.shape[0] == first[0] and b.shape[0] == second[0]
    table.free()


def test_noalloc_refuses_more_pairs_than_the_scratch_holds():
    from paper_2312_05417_amd import binding as espn, synth
    dev = torch.device("cuda:0")
    lib = espn.lib()
    w = synth.scaled(synth.WORKLOADS["c1"], n_docs=500)
    emb, off = synth.table(w, 5, device=dev)
    table = espn.espn_table_load(emb, off)
    B, K = 2049, 2048                                   # 2049 * 2048 > 4 Mi pairs
    assert B * K > espn.ESPN_NOALLOC_MAX_PAIRS
    q = torch.zeros((B, 32, w.dim), dtype=torch.float16, device=dev)
    cand = torch.zeros((B, K), dtype=torch.int64, device=dev)
    out_ids = torch.empty((B, 1), dtype=torch.int64, device=dev)
    out_sc = torch.empty((B, 1), dtype=torch.float32, device=dev)
    rc = lib.espn_rerank_noalloc(table.handle, q.data_ptr(), cand.data_ptr(), B, 32, K, 1, out_ids.data_ptr(),
                                 out_sc.data_ptr(), int(torch.cuda.current_stream().cuda_stream))
    assert rc == espn.ESPN_ERR_SHAPE
    assert "static scratch" in espn.last_error()
    # exactly the limit is accepted
    B = 2048
    rc = lib.espn_rerank_noalloc(table.handle, q.data_ptr(), cand.data_ptr(), B, 32, K, 1, out_ids.data_ptr(),
                                 out_sc.data_ptr(), int(torch.cuda.current_stream().cuda_stream))
    assert rc == 0, espn.last_error()
    torch.cuda.synchronize()
    espn.espn_table_check(table)
    table.free()


def test_noalloc_inside_a_captured_graph():
    """What the entry point is for: a caller under HIP graph capture, where nothing may be allocated.  Replayed
    with other calls on the shared array in between; every replay against the eager result."""
    from paper_2312_05417_amd import binding as espn, synth
    dev = torch.device("cuda:0")
    w = synth.scaled(synth.WORKLOADS["c2"], n_docs=20000, B=8, K=600)
    emb, off = synth.table(w, 11, device=dev)
    table = espn.espn_table_load(emb, off)
    qs = [synth.queries(w, 11, n, device=dev) for n in range(3)]
    cs = [torch.from_numpy(synth.candidates(w, 11, n)).to(dev) for n in range(3)]
    eager = [tuple(t.clone() for t in espn.espn_rerank(table, q, c, w.k)) for q, c in zip(qs, cs)]
    torch.cuda.synchronize()
    q_buf, c_buf = qs[0].clone(), cs[0].clone()
    ids_buf = torch.empty((w.B, w.k), dtype=torch.int64, device=dev)
    sc_buf = torch.empty((w.B, w.k), dtype=torch.float32, device=dev)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        espn.espn_rerank_noalloc(table, q_buf, c_buf, w.k, ids_buf, sc_buf)
    other_ids, other_sc = torch.empty_like(ids_buf), torch.empty_like(sc_buf)
    for rep in range(2):
        for n in range(3):
            q_buf.copy_(qs[n])
            c_buf.copy_(cs[n])
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(ids_buf, eager[n][0]) and torch.equal(sc_buf, eager[n][1]), (rep, n)
            # an eager call on the same array between replays
            espn.espn_rerank_noalloc(table, qs[(n + 1) % 3], cs[(n + 1) % 3], w.k, other_ids, other_sc)
            torch.cuda.synchronize()
            assert torch.equal(other_ids, eager[(n + 1) % 3][0])
    espn.espn_table_check(table)
    del graph
    table.free()
