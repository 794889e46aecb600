"""Calls only enqueue on the caller's stream: they work on side streams and inside a captured HIP graph."""
import numpy as np
import pytest
import torch

from paper_2312_05417_amd import binding as espn
from paper_2312_05417_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print("[case] " + msg, flush=True)


def test_rerank_on_a_side_stream_equals_the_default_stream():
    w = synth.scaled(synth.WORKLOADS["c3"], n_docs=3000, B=6, K=250)
    say("side stream")
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    q, cand = synth.queries(w).to(DEV), torch.from_numpy(synth.candidates(w)).to(DEV)
    ids0, sc0 = espn.espn_rerank(table, q, cand, w.k)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ids1, sc1 = espn.espn_rerank(table, q, cand, w.k)          # binding picks up the current stream
    ids2, sc2 = espn.espn_rerank(table, q, cand, w.k, stream=side)  # or an explicit one
    side.synchronize()
    espn.espn_table_check(table, stream=side)
    assert torch.equal(ids0, ids1) and torch.equal(sc0, sc1) and torch.equal(ids0, ids2) and torch.equal(sc0, sc2)
    table.free()


@pytest.mark.parametrize("key,changes", [("c1", {}), ("c3", dict(n_docs=3000, B=6, K=250))])
def test_captured_graph_replays_match_eager_results(key, changes):
    w = synth.scaled(synth.WORKLOADS[key], **changes)
    say("graph capture %s" % w.name)
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    batches = [(synth.queries(w, batch=n).to(DEV), torch.from_numpy(synth.candidates(w, batch=n)).to(DEV))
               for n in range(4)]
    eager = [espn.espn_rerank(table, q, c, w.k) for q, c in batches]
    eager = [(i.clone(), s.clone()) for i, s in eager]
    torch.cuda.synchronize()
    # static buffers the graph reads and writes
    q_buf, c_buf = batches[0][0].clone(), batches[0][1].clone()
    ids_buf = torch.empty((w.B, w.k), dtype=torch.int64, device=DEV)
    sc_buf = torch.empty((w.B, w.k), dtype=torch.float32, device=DEV)
    ws = torch.empty(espn.espn_workspace_bytes(w.B, w.K), dtype=torch.uint8, device=DEV)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        espn.espn_rerank(table, q_buf, c_buf, w.k, out_ids=ids_buf, out_scores=sc_buf, workspace=ws)
    for rep in range(2):
        for n, (q, c) in enumerate(batches):
            q_buf.copy_(q)
            c_buf.copy_(c)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(ids_buf, eager[n][0]) and torch.equal(sc_buf, eager[n][1]), (rep, n)
            # eager work of the program between replays
            again = espn.espn_rerank(table, q, c, w.k)
            assert torch.equal(again[0], eager[n][0])
    espn.espn_table_check(table)
    del graph
    table.free()


def test_a_queue_of_batches_can_be_captured_too():
    """espn_rerank_batches inside a captured graph: its fork to the library's streams and the join back are event
    records and waits, which a capture turns into graph edges.  Replayed with eager work and synchronisations of
    the program in between, every replay checked against the eager results."""
    w = synth.scaled(synth.WORKLOADS["c3"], n_docs=3000, B=6, K=250)
    say("graph capture of a queue")
    emb, off = synth.table(w)
    table = espn.espn_table_load(emb.to(DEV), off)
    n = 20
    plan = espn.espn_batches_plan(table, n, w.B, w.Q, w.K, w.k)
    assert plan["launches"] == 2 and plan["streams"] == 2              # so that there is a fork and a join to capture
    sets = [[(synth.queries(w, batch=10 * r + i).to(DEV), torch.from_numpy(synth.candidates(w, batch=10 * r + i)).to(DEV))
             for i in range(n)] for r in range(2)]
    eager = [[tuple(t.clone() for t in espn.espn_rerank(table, q, c, w.k)) for q, c in one] for one in sets]
    torch.cuda.synchronize()
    q_buf = [sets[0][i][0].clone() for i in range(n)]
    c_buf = [sets[0][i][1].clone() for i in range(n)]
    ids_buf = [torch.empty((w.B, w.k), dtype=torch.int64, device=DEV) for _ in range(n)]
    sc_buf = [torch.empty((w.B, w.k), dtype=torch.float32, device=DEV) for _ in range(n)]
    ws = torch.empty(espn.espn_batches_workspace_bytes(table, n, w.B, w.Q, w.K, w.k), dtype=torch.uint8, device=DEV)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        espn.espn_rerank_batches(table, q_buf, c_buf, w.k, ids_buf, sc_buf, workspace=ws)
    for rep in range(4):
        which = rep % 2
        for i in range(n):
            q_buf[i].copy_(sets[which][i][0])
            c_buf[i].copy_(sets[which][i][1])
            ids_buf[i].fill_(-3)
        graph.replay()
        torch.cuda.synchronize()
        for i in range(n):
            assert torch.equal(ids_buf[i], eager[which][i][0]) and torch.equal(sc_buf[i], eager[which][i][1]), (rep, i)
        again = espn.espn_rerank_batches(table, [x[0] for x in sets[which]], [x[1] for x in sets[which]], w.k)   # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(again[0][3], eager[which][3][0])
    espn.espn_table_check(table)
    del graph
    table.free()


def test_two_tables_and_two_streams_do_not_disturb_each_other():
    say("two tables, two streams")
    wa = synth.scaled(synth.WORKLOADS["c1"], n_docs=2000)
    wb = synth.scaled(synth.WORKLOADS["c3"], n_docs=1500, B=4, K=120)
    ea, oa = synth.table(wa, seed=1)
    eb, ob = synth.table(wb, seed=2)
    ta, tb = espn.espn_table_load(ea.to(DEV), oa), espn.espn_table_load(eb.to(DEV), ob)
    qa, ca = synth.queries(wa, 1).to(DEV), torch.from_numpy(synth.candidates(wa, 1)).to(DEV)
    qb, cb = synth.queries(wb, 2).to(DEV), torch.from_numpy(synth.candidates(wb, 2)).to(DEV)
    ref_a, ref_b = espn.espn_rerank(ta, qa, ca, 10), espn.espn_rerank(tb, qb, cb, 10)
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(5):
        outs.append((espn.espn_rerank(ta, qa, ca, 10, stream=sa), espn.espn_rerank(tb, qb, cb, 10, stream=sb)))
    torch.cuda.synchronize()
    for (a, b) in outs:
        assert torch.equal(a[0], ref_a[0]) and torch.equal(a[1], ref_a[1])
        assert torch.equal(b[0], ref_b[0]) and torch.equal(b[1], ref_b[1])
    ta.free()
    tb.free()


def test_read_probe_reads_whatever_it_is_given_and_stores_nothing():
    """The measuring stick of the benchmark: any 16-byte-multiple size, sizes smaller than one round of a
    workgroup included; its sink is written only if the xor of everything read is all ones."""
    say("read probe")
    buf = torch.arange(0, 1 << 22, dtype=torch.int32, device=DEV)              # 16 MiB, xor of the words is 0
    sink = torch.full((1,), 7, dtype=torch.int64, device=DEV)
    from paper_2312_05417_amd import benchprobe
    st = int(torch.cuda.current_stream().cuda_stream)

    def read(t):
        benchprobe.stream_read(t.data_ptr(), t.numel() * t.element_size(), sink.data_ptr(), st)

    for n_words in (4, 8, 1 << 10, (1 << 22) - 4, 1 << 22):
        read(buf[:n_words])
    torch.cuda.synchronize()
    assert int(sink.item()) == 7
    ones = torch.full((4,), -1, dtype=torch.int32, device=DEV)                 # one chunk of all ones: stored
    read(ones)
    torch.cuda.synchronize()
    assert int(sink.item()) == -1
    with pytest.raises(ValueError):
        read(buf[:3])                                                          # 12 bytes
    with pytest.raises(ValueError):
        read(buf[1:5])                                                         # not 16-byte aligned
    # the calibration copy copies
    dst = torch.zeros(1 << 20, dtype=torch.int32, device=DEV)
    benchprobe.copy(buf.data_ptr(), dst.data_ptr(), dst.numel() * 4, st)
    torch.cuda.synchronize()
    assert torch.equal(dst, buf[: 1 << 20])
