"""Seeded random shapes through the ranking kernels on their own (espn_topk, espn_merge_topk) against
the oracle, exactly: list lengths around every kernel's limits, k from 0 to the whole list, scores
with runs of exact ties, -inf, both zeros, all equal; ids negative, beyond 32 bits, heavily
repeated.  Scores are binary32 on both sides, so ids and scores are pinned bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2312_05417_amd import binding as espn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
LENGTHS = [1, 2, 3, 63, 64, 65, 255, 256, 257, 700, 1000, 1023, 1024, 1025, 2047, 2048, 2049, 3000, 4095, 4096,
           4097, 6000]


def draw(seed):
    rng = np.random.default_rng(77000 + seed)
    B = int(rng.integers(1, 6))
    K = int(rng.choice(LENGTHS))
    k = int(rng.choice([0, 1, 2, 10, 31, 32, 33, 64, 65, 100, K // 2, K - 1, K]))
    k = max(0, min(k, K))
    mode = int(rng.integers(0, 5))
    sc = rng.normal(size=(B, K)).astype(np.float32) * 5
    if mode == 1:
        sc = np.round(sc)                                       # a few dozen distinct values
    elif mode == 2:
        sc = np.where(rng.random((B, K)) < 0.3, -np.inf, np.round(sc * 2) / 2).astype(np.float32)
    elif mode == 3:
        sc[:] = 1.5                                             # the ranking is by id alone
    elif mode == 4:
        sc = np.round(sc, 1)
        sc[rng.random((B, K)) < 0.05] = 0.0
        sc[rng.random((B, K)) < 0.05] = -0.0                    # the same score as +0
    spread = int(rng.choice([5, 50, 10 * K + 10]))
    cand = rng.integers(-spread, spread + 1, size=(B, K)).astype(np.int64)
    if rng.random() < 0.3:
        cand += 1 << 35
    return B, K, k, mode, sc, cand, int(rng.integers(0, K + 1))


@pytest.mark.parametrize("seed", range(80))
def test_random_ranking_and_merge(seed):
    B, K, k, mode, sc, cand, ka = draw(seed)
    print("[case] seed %d: B=%d K=%d k=%d mode=%d split=%d" % (seed, B, K, k, mode, ka), flush=True)
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    o_ids, o_top = oracle.topk(sc.astype(np.float64), cand, k)
    g_ids, g_top = espn.espn_topk(dev(sc), dev(cand), k)
    assert np.array_equal(g_ids.cpu().numpy(), o_ids)
    assert np.array_equal(g_top.cpu().numpy().astype(np.float64), o_top)
    # the list cut in two at a random place and merged again (Sec. 4.3)
    a_i, b_i, a_s, b_s = cand[:, :ka], cand[:, ka:], sc[:, :ka], sc[:, ka:]
    m_ids, m_top = oracle.merge(np.ascontiguousarray(a_i), np.ascontiguousarray(a_s), np.ascontiguousarray(b_i),
                                np.ascontiguousarray(b_s), k)
    assert np.array_equal(m_ids, o_ids)                        # merging the parts = ranking the whole
    gm_ids, gm_top = espn.espn_merge_topk(dev(a_i), dev(a_s), dev(b_i), dev(b_s), k)
    assert np.array_equal(gm_ids.cpu().numpy(), m_ids)
    assert np.array_equal(gm_top.cpu().numpy().astype(np.float64), m_top)
