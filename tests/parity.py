"""Comparison rules between the HIP path and the fp64 oracle (shared by the GPU tests, the smoke
check and nothing else).  Holds no scoring arithmetic: only tolerances and rank bookkeeping."""
import math

import numpy as np

REL_TOL = 1e-3        # fp16 inputs, fp32 accumulation: relative error allowed on a score
UNIT_ROUNDOFF = 2.0 ** -24     # binary32


def cancellation_floor(magnitude, d: int, Q: int):
    """A score is a sum of Q maxima of d-term dot products and these terms may cancel (a query row
    that points away from every row of a short document contributes a negative maximum): then the
    score is small against its terms and no arithmetic can promise an error relative to the score.
    What binary32 accumulation does promise is an error of at most (d + Q) * 2^-24 relative to the
    sum of the terms' magnitudes.  `magnitude` is that sum, or an upper bound of it: the oracle's
    score of the same pair with every component of the query and of the table replaced by its
    absolute value.  For ordinary scores (a tenth of the magnitude or more) REL_TOL is 50 times
    larger than this floor, which therefore only decides where terms cancel."""
    return (d + Q) * UNIT_ROUNDOFF * np.asarray(magnitude, dtype=np.float64)


def tol_of(score: float, Q: int, floor: float = 0.0) -> float:
    """Absolute tolerance on one score: REL_TOL relative, with a floor for scores near zero."""
    return max(REL_TOL * max(abs(score), 1e-6 * Q), floor)


def assert_scores_close(gpu: np.ndarray, ora: np.ndarray, Q: int, what: str = "scores", floor=None):
    """Element by element: -inf must match exactly, finite values within tol_of (floor: an array
    like ora from cancellation_floor, or None)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ora = np.asarray(ora, dtype=np.float64)
    assert gpu.shape == ora.shape, (what, gpu.shape, ora.shape)
    inf_o = np.isneginf(ora)
    assert np.array_equal(np.isneginf(gpu), inf_o), what + ": -inf pattern differs"
    assert not np.isnan(gpu).any(), what + ": NaN from the GPU"
    fin = ~inf_o
    tol = REL_TOL * np.maximum(np.abs(ora[fin]), 1e-6 * Q)
    if floor is not None:
        tol = np.maximum(tol, np.asarray(floor, dtype=np.float64)[fin])
    err = np.abs(gpu[fin] - ora[fin])
    bad = err > tol
    assert not bad.any(), "%s: %d of %d beyond tolerance, worst rel err %.3e" % (
        what, int(bad.sum()), err.size, float((err / np.maximum(np.abs(ora[fin]), 1e-30)).max()))
    return float((err / np.maximum(np.abs(ora[fin]), 1e-6 * Q)).max()) if err.size else 0.0


def assert_topk_matches(gpu_ids, gpu_scores, ora_all_scores, cand, k: int, Q: int, floor=None):
    """One query.  gpu_ids/gpu_scores: [k] from the HIP path; ora_all_scores: oracle fp64 [K];
    cand: [K] ids.  Ranks whose oracle score is separated from both neighbours by more than twice
    the tolerance must carry exactly the oracle's id; inside a run of near-ties any order is
    accepted as long as every returned id scores within tolerance of the oracle's entry at that
    rank; returned scores must match the oracle's score of the returned id; and the returned list
    must itself be sorted by (score desc, id asc).  floor: [K] from cancellation_floor, or None."""
    gpu_ids = np.asarray(gpu_ids).tolist()
    gpu_scores = np.asarray(gpu_scores, dtype=np.float64).tolist()
    ora = np.asarray(ora_all_scores, dtype=np.float64)
    cand = np.asarray(cand)
    K = cand.shape[0]
    assert len(gpu_ids) == k and len(gpu_scores) == k
    fl = np.zeros(K) if floor is None else np.where(np.isfinite(ora), np.asarray(floor, dtype=np.float64), 0.0)
    order = sorted(range(K), key=lambda j: (-ora[j], int(cand[j])))
    o_sc = [float(ora[j]) for j in order]
    o_id = [int(cand[j]) for j in order]
    o_fl = [float(fl[j]) for j in order]
    by_id, floor_of_id = {}, {}
    for j in range(K):
        by_id.setdefault(int(cand[j]), []).append(float(ora[j]))
        floor_of_id[int(cand[j])] = float(fl[j])

    def separated(a, b, fa=0.0, fb=0.0):
        if math.isinf(a) and math.isinf(b):
            return False
        if math.isinf(a) or math.isinf(b):
            return True
        return abs(a - b) > 2 * max(tol_of(a, Q, fa), tol_of(b, Q, fb))

    used = {}
    for r in range(k):
        gid, gs = gpu_ids[r], gpu_scores[r]
        assert gid in by_id, "rank %d: id %d is not a candidate" % (r, gid)
        used[gid] = used.get(gid, 0) + 1
        assert used[gid] <= len(by_id[gid]), "rank %d: id %d returned more often than listed" % (r, gid)
        own = by_id[gid][0]
        if math.isinf(own):
            assert gs == own, "rank %d: score %r for an empty document" % (r, gs)
        else:
            assert abs(gs - own) <= tol_of(own, Q, floor_of_id[gid]), "rank %d: score %r vs oracle %r" % (r, gs, own)
        pinned = ((r == 0 or separated(o_sc[r - 1], o_sc[r], o_fl[r - 1], o_fl[r])) and
                  (r + 1 >= K or separated(o_sc[r], o_sc[r + 1], o_fl[r], o_fl[r + 1])))
        if pinned:
            assert gid == o_id[r], "rank %d: id %d, oracle %d (score gap is beyond tolerance)" % (r, gid, o_id[r])
        else:
            assert not separated(own, o_sc[r], floor_of_id[gid], o_fl[r]), (
                "rank %d: id %d scores %r, oracle rank holds %r" % (r, gid, own, o_sc[r]))
        if r > 0:
            ps, pi = gpu_scores[r - 1], gpu_ids[r - 1]
            assert ps > gs or (ps == gs and pi <= gid), "rank %d: output not in (score desc, id asc) order" % r
