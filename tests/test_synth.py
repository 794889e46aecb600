"""The seeded input generators: reproducible, shaped as stated, and free of surprises."""
import numpy as np
import torch

from paper_2312_05417_amd import synth


def test_same_seed_same_bytes_and_different_seed_differs():
    w = synth.WORKLOADS["c1"]
    e1, o1 = synth.table(w, seed=5)
    e2, o2 = synth.table(w, seed=5)
    e3, o3 = synth.table(w, seed=6)
    assert torch.equal(e1, e2) and np.array_equal(o1, o2)
    assert not np.array_equal(o1, o3)
    assert torch.equal(synth.queries(w, 5, 3), synth.queries(w, 5, 3))
    assert not torch.equal(synth.queries(w, 5, 3), synth.queries(w, 5, 4))
    assert np.array_equal(synth.candidates(w, 5, 2), synth.candidates(w, 5, 2))
    assert not np.array_equal(synth.candidates(w, 5, 2), synth.candidates(w, 5, 1))


def test_c1_shapes_and_ranges():
    w = synth.WORKLOADS["c1"]
    emb, off = synth.table(w)
    counts = np.diff(off)
    assert off[0] == 0 and off.shape == (w.n_docs + 1,) and emb.shape == (off[-1], 32) and emb.dtype == torch.float16
    assert counts.min() == 8 and counts.max() == 64
    norms = emb.float().norm(dim=1)
    assert float((norms - 1).abs().max()) < 2e-3
    q = synth.queries(w)
    assert q.shape == (8, 32, 32)
    cand = synth.candidates(w)
    assert cand.shape == (8, 100) and cand.min() >= 0 and cand.max() < w.n_docs
    assert all(len(set(r.tolist())) == 100 for r in cand)


def test_lognormal_counts_have_the_stated_mean_and_clip():
    for key, lo, hi, mean in (("c2", 4, 128, 40.0), ("c3", 8, 180, 70.0)):
        w = synth.scaled(synth.WORKLOADS[key], n_docs=200_000)
        c = synth.token_counts(w)
        assert c.min() == lo and c.max() == hi
        assert abs(c.mean() - mean) < 0.02 * mean + 0.7


def test_zipf_candidates_are_distinct_and_repeat_across_queries():
    w = synth.scaled(synth.WORKLOADS["c4"], n_docs=50_000, B=16, K=200)
    cand = synth.candidates(w)
    assert all(len(set(r.tolist())) == w.K for r in cand)
    uniq = np.unique(cand).size
    assert uniq < 0.8 * cand.size                      # heavy head: many repeats across queries
    common = set(cand[0].tolist())
    for r in cand[1:]:
        common &= set(r.tolist())
    assert len(common) >= 3                            # the hottest documents are in every list
    assert np.unique(cand).max() > w.n_docs // 2       # and hot ids are scattered, not the first rows


def test_subtable_keeps_bytes_and_id_order():
    w = synth.scaled(synth.WORKLOADS["c1"], n_docs=500)
    emb, off = synth.table(w)
    cand = synth.candidates(w)[:2]
    sub, loc_off, loc_cand, ids = synth.subtable(emb, off, cand)
    assert np.all(np.diff(ids) > 0)
    assert np.array_equal(ids[loc_cand], cand)
    e = emb.numpy()
    for u in (0, 7, ids.size - 1):
        assert np.array_equal(sub[loc_off[u]:loc_off[u + 1]], e[off[ids[u]]:off[ids[u] + 1]])
