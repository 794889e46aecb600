"""CPU oracle for the re-ranking path (Eq. 1 MaxSim + ranked top-k), fp64.

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's cpu_baseline leg.  The HIP library and its Python binding never
import this package, and this package imports nothing of theirs.

The arithmetic lives in ``espn_oracle.c`` (plain C, gcc); this file only builds
it and marshals numpy arrays through ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "espn_oracle.c")
_LIB = os.path.join(_HERE, "libespn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile espn_oracle.c into libespn_oracle.so next to it (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_i32, c_i64, c_p = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        lib.espn_oracle_half_to_double.restype = ctypes.c_double
        lib.espn_oracle_half_to_double.argtypes = [ctypes.c_uint16]
        lib.espn_oracle_maxsim_pair.restype = ctypes.c_double
        lib.espn_oracle_maxsim_pair.argtypes = [c_p, c_i32, c_p, c_i64, c_i32]
        lib.espn_oracle_scores.restype = ctypes.c_int
        lib.espn_oracle_scores.argtypes = [c_p, c_p, c_i64, c_i32, c_p, c_p, c_i32, c_i32, c_i32, c_p, c_i32]
        lib.espn_oracle_topk.restype = ctypes.c_int
        lib.espn_oracle_topk.argtypes = [c_p, c_p, c_i32, c_i32, c_i32, c_p, c_p]
        lib.espn_oracle_rerank.restype = ctypes.c_int
        lib.espn_oracle_rerank.argtypes = [c_p, c_p, c_i64, c_i32, c_p, c_p, c_i32, c_i32, c_i32, c_i32,
                                           c_p, c_p, c_p, c_i32]
        lib.espn_oracle_scores_prior.restype = ctypes.c_int
        lib.espn_oracle_scores_prior.argtypes = [c_p, c_p, c_i64, c_i32, c_p, c_p, c_p, ctypes.c_double,
                                                 c_i32, c_i32, c_i32, c_p, c_i32]
        lib.espn_oracle_rerank_partial.restype = ctypes.c_int
        lib.espn_oracle_rerank_partial.argtypes = [c_p, c_p, c_i64, c_i32, c_p, c_p, c_i32, c_i32, c_i32, c_i32,
                                                   c_i32, c_p, c_p, c_i32]
        lib.espn_oracle_merge.restype = ctypes.c_int
        lib.espn_oracle_merge.argtypes = [c_p, c_p, c_i32, c_p, c_p, c_i32, c_i32, c_i32, c_p, c_p]
        lib.espn_oracle_batch_threshold.restype = ctypes.c_double
        lib.espn_oracle_batch_threshold.argtypes = [ctypes.c_double] * 3
        lib.espn_oracle_e4m3_to_double.restype = ctypes.c_double
        lib.espn_oracle_e4m3_to_double.argtypes = [ctypes.c_uint8]
        lib.espn_oracle_scores_e4m3.restype = ctypes.c_int
        lib.espn_oracle_scores_e4m3.argtypes = [c_p, c_p, c_p, c_i64, c_i32, c_p, c_p, c_i32, c_i32, c_i32, c_p, c_i32]
        lib.espn_oracle_max_threads.restype = c_i32
        lib.espn_oracle_max_threads.argtypes = []
        _lib = lib
    return _lib


def _f16_bits(a, shape_tail=None) -> np.ndarray:
    """View an array of binary16 values (float16, or uint16/int16 bit patterns) as uint16."""
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    elif a.dtype == np.int16:
        a = a.view(np.uint16)
    elif a.dtype != np.uint16:
        raise TypeError("binary16 data must be float16 or (u)int16 bit patterns, got %s" % a.dtype)
    return np.ascontiguousarray(a)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def half_to_double(bits: int) -> float:
    """Exact value of one binary16 bit pattern."""
    return float(_load().espn_oracle_half_to_double(int(bits) & 0xFFFF))


def maxsim_pair(q, doc) -> float:
    """Eq. 1 for one query matrix q [Q,d] and one document matrix doc [t,d] (binary16)."""
    qb, db = _f16_bits(q), _f16_bits(doc)
    if qb.ndim != 2 or db.ndim != 2 or (db.shape[0] and qb.shape[1] != db.shape[1]):
        raise ValueError("q must be [Q,d] and doc [t,d]")
    return float(_load().espn_oracle_maxsim_pair(_ptr(qb), qb.shape[0], _ptr(db), db.shape[0], qb.shape[1]))


def _check(emb, offsets, q, cand):
    eb, qb = _f16_bits(emb), _f16_bits(q)
    off = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
    cd = np.ascontiguousarray(np.asarray(cand, dtype=np.int64))
    if eb.ndim != 2 or qb.ndim != 3 or cd.ndim != 2 or off.ndim != 1:
        raise ValueError("expected emb [T,d], offsets [N+1], q [B,Q,d], cand [B,K]")
    if qb.shape[2] != eb.shape[1] or cd.shape[0] != qb.shape[0]:
        raise ValueError("shape mismatch between emb, q and cand")
    if off.shape[0] < 1 or off[0] != 0 or off[-1] != eb.shape[0] or np.any(np.diff(off) < 0):
        raise ValueError("offsets must start at 0, end at the row count and never decrease")
    return eb, off, qb, cd


def scores(emb, offsets, q, cand, threads: int = 0) -> np.ndarray:
    """MaxSim score of every candidate: fp64 [B,K]."""
    eb, off, qb, cd = _check(emb, offsets, q, cand)
    B, Q, d = qb.shape
    K = cd.shape[1]
    out = np.empty((B, K), dtype=np.float64)
    rc = _load().espn_oracle_scores(_ptr(eb), _ptr(off), off.shape[0] - 1, d, _ptr(qb), _ptr(cd),
                                    B, Q, K, _ptr(out), threads)
    if rc != 0:
        raise ValueError("candidate id outside [0, n_docs)")
    return out


def topk(all_scores, cand, k: int):
    """Ranked top-k per query by (score desc, id asc): (ids int64 [B,k], scores fp64 [B,k])."""
    sc = np.ascontiguousarray(np.asarray(all_scores, dtype=np.float64))
    cd = np.ascontiguousarray(np.asarray(cand, dtype=np.int64))
    if sc.shape != cd.shape or sc.ndim != 2:
        raise ValueError("scores and cand must both be [B,K]")
    if np.isnan(sc).any():
        raise ValueError("NaN scores have no rank")
    B, K = sc.shape
    ids = np.empty((B, k), dtype=np.int64)
    out = np.empty((B, k), dtype=np.float64)
    if _load().espn_oracle_topk(_ptr(sc), _ptr(cd), B, K, k, _ptr(ids), _ptr(out)) != 0:
        raise ValueError("k must lie in [0, K]")
    return ids, out


def rerank(emb, offsets, q, cand, k: int, threads: int = 0):
    """Whole path: (top-k ids [B,k], top-k scores [B,k], all scores [B,K])."""
    eb, off, qb, cd = _check(emb, offsets, q, cand)
    B, Q, d = qb.shape
    K = cd.shape[1]
    if not 0 <= k <= K:
        raise ValueError("k must lie in [0, K]")
    ids = np.empty((B, k), dtype=np.int64)
    top = np.empty((B, k), dtype=np.float64)
    allsc = np.empty((B, K), dtype=np.float64)
    rc = _load().espn_oracle_rerank(_ptr(eb), _ptr(off), off.shape[0] - 1, d, _ptr(qb), _ptr(cd),
                                    B, Q, K, k, _ptr(ids), _ptr(top), _ptr(allsc), threads)
    if rc != 0:
        raise ValueError("candidate id outside [0, n_docs)")
    return ids, top, allsc


def max_threads() -> int:
    return int(_load().espn_oracle_max_threads())


def scores_prior(emb, offsets, q, cand, prior, alpha: float, threads: int = 0) -> np.ndarray:
    """MaxSim score plus alpha times the first-stage score (Sec. 3.1): fp64 [B,K]."""
    eb, off, qb, cd = _check(emb, offsets, q, cand)
    pr = np.ascontiguousarray(np.asarray(prior, dtype=np.float32))
    if pr.shape != cd.shape:
        raise ValueError("prior must be [B,K]")
    B, Q, d = qb.shape
    K = cd.shape[1]
    out = np.empty((B, K), dtype=np.float64)
    rc = _load().espn_oracle_scores_prior(_ptr(eb), _ptr(off), off.shape[0] - 1, d, _ptr(qb), _ptr(cd), _ptr(pr),
                                          float(alpha), B, Q, K, _ptr(out), threads)
    if rc != 0:
        raise ValueError("candidate id outside [0, n_docs)")
    return out


def rerank_partial(emb, offsets, q, cand, R: int, k: int, threads: int = 0):
    """Partial re-ranking (Sec. 4.4): (ids [B,k], scores [B,k]); entries beyond the re-ranked R carry NaN."""
    eb, off, qb, cd = _check(emb, offsets, q, cand)
    B, Q, d = qb.shape
    K = cd.shape[1]
    ids = np.empty((B, k), dtype=np.int64)
    top = np.empty((B, k), dtype=np.float64)
    rc = _load().espn_oracle_rerank_partial(_ptr(eb), _ptr(off), off.shape[0] - 1, d, _ptr(qb), _ptr(cd),
                                            B, Q, K, R, k, _ptr(ids), _ptr(top), threads)
    if rc != 0:
        raise ValueError("bad R or k, or candidate id outside [0, n_docs)")
    return ids, top


def merge(ids_a, sc_a, ids_b, sc_b, k: int):
    """First k of the union of two scored lists per query (Sec. 4.3), in ranking order."""
    ia = np.ascontiguousarray(np.asarray(ids_a, dtype=np.int64))
    ib = np.ascontiguousarray(np.asarray(ids_b, dtype=np.int64))
    sa = np.ascontiguousarray(np.asarray(sc_a, dtype=np.float64))
    sb = np.ascontiguousarray(np.asarray(sc_b, dtype=np.float64))
    if ia.shape != sa.shape or ib.shape != sb.shape or ia.ndim != 2 or ib.ndim != 2 or ia.shape[0] != ib.shape[0]:
        raise ValueError("expected [B,ka] and [B,kb] lists")
    if np.isnan(sa).any() or np.isnan(sb).any():
        raise ValueError("NaN scores have no rank")
    B = ia.shape[0]
    ids = np.empty((B, k), dtype=np.int64)
    out = np.empty((B, k), dtype=np.float64)
    if _load().espn_oracle_merge(_ptr(ia), _ptr(sa), ia.shape[1], _ptr(ib), _ptr(sb), ib.shape[1], B, k,
                                 _ptr(ids), _ptr(out)) != 0:
        raise ValueError("k must lie in [0, ka + kb]")
    return ids, out


def batch_threshold(bandwidth_bytes_per_s: float, budget_s: float, bytes_per_query: float) -> float:
    """Eq. 4."""
    return float(_load().espn_oracle_batch_threshold(bandwidth_bytes_per_s, budget_s, bytes_per_query))


def e4m3_to_double(code: int) -> float:
    """Exact value of one E4M3 code (OCP 8-bit floating point)."""
    return float(_load().espn_oracle_e4m3_to_double(int(code) & 0xFF))


def scores_e4m3(codes, doc_scale, offsets, q, cand, threads: int = 0) -> np.ndarray:
    """MaxSim scores on a compressed table: codes uint8 [T,d] (E4M3), one positive fp32 scale per document."""
    cb = np.ascontiguousarray(np.asarray(codes))
    if cb.dtype != np.uint8 or cb.ndim != 2:
        raise TypeError("codes must be uint8 [T,d]")
    qb = _f16_bits(q)
    off = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
    cd = np.ascontiguousarray(np.asarray(cand, dtype=np.int64))
    sc = np.ascontiguousarray(np.asarray(doc_scale, dtype=np.float32))
    if qb.ndim != 3 or cd.ndim != 2 or qb.shape[2] != cb.shape[1] or cd.shape[0] != qb.shape[0]:
        raise ValueError("shape mismatch")
    if off[0] != 0 or off[-1] != cb.shape[0] or np.any(np.diff(off) < 0) or sc.shape != (off.shape[0] - 1,):
        raise ValueError("offsets / scales do not describe the table")
    if not (np.all(sc > 0) and np.all(np.isfinite(sc))):
        raise ValueError("document scales must be positive and finite")
    B, Q, d = qb.shape
    K = cd.shape[1]
    out = np.empty((B, K), dtype=np.float64)
    rc = _load().espn_oracle_scores_e4m3(_ptr(cb), _ptr(sc), _ptr(off), off.shape[0] - 1, d, _ptr(qb), _ptr(cd),
                                         B, Q, K, _ptr(out), threads)
    if rc != 0:
        raise ValueError("candidate id outside [0, n_docs)")
    return out
