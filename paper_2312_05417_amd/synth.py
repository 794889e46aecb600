"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *draws inputs*: token counts, token vectors, query vectors and
candidate lists.  It holds none of the method's arithmetic (no scoring, no
ranking) and is the one piece of code that both the tests' CPU oracle and the
HIP path are fed from.

Shapes follow the paper: 16-bit token vectors of dimension 32 (ColBERTer BOW
vectors, Sec. 3.1) or 128 (uncompressed ColBERT-style, Table 1), a few dozen
token vectors per passage (Table 3: 597.9 M tokens over 8.8 M passages), about
a thousand candidates per query (Sec. 4.4, Sec. 5.4).  The datasets themselves
are not used; every value here is random.

Every array is a pure function of (seed, stream, index): the same call gives the
same bytes again.  Token and query *values* are drawn with torch's generator of
the device they are drawn on, so a table drawn on the GPU differs from one drawn
on the CPU for the same seed; within one run both sides read the same bytes.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np
import torch

DEFAULT_SEED = 20231205

# sub-stream tags
_S_COUNTS, _S_TOKENS, _S_QUERIES, _S_CANDS, _S_PERM = 1, 2, 3, 4, 5


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    n_docs: int
    dim: int
    count_law: str          # "uniform" or "lognormal"
    count_lo: int
    count_hi: int
    count_mean: float       # lognormal only: mean of the unclipped distribution
    B: int                  # queries per batch
    Q: int                  # token vectors per query
    K: int                  # candidates per query
    k: int                  # ranked outputs per query
    cand_law: str           # "uniform" or "zipf"
    zipf_alpha: float = 1.1
    host_resident: bool = False
    count_sigma: float = 0.5
    rerank_top: int = 0     # > 0: partial re-ranking, only the first rerank_top candidates are scored
    codec: str = "f16"      # "f16": binary16 rows; "e4m3": 8-bit codes + one scale per document


WORKLOADS = {
    # small case the CPU oracle finishes in seconds
    "c1": Workload("c1-tiny", 10_000, 32, "uniform", 8, 64, 0.0, 8, 32, 100, 10, "uniform"),
    # ColBERTer-like compressed vectors (d=32), table ~2.6 GB in HBM
    "c2": Workload("c2-colberter-d32", 1_000_000, 32, "lognormal", 4, 128, 40.0, 64, 32, 1000, 10, "uniform"),
    # ColBERTv2-like uncompressed vectors (d=128), table ~36 GB in HBM
    "c3": Workload("c3-colbertv2-d128", 2_000_000, 128, "lognormal", 8, 180, 70.0, 256, 32, 1000, 10, "uniform"),
    # large batch, candidates repeat across queries
    "c4": Workload("c4-overlap-d128", 2_000_000, 128, "lognormal", 8, 180, 70.0, 2048, 32, 1000, 10, "zipf"),
    # table in pinned host memory, streamed over PCIe
    "c5": Workload("c5-host-d128", 8_800_000, 128, "lognormal", 8, 180, 70.0, 1024, 32, 1000, 10, "zipf",
                   host_resident=True),
    # partial re-ranking (Sec. 4.4): only the 64 best-placed of the 1000 candidates are scored, so a
    # batch of the same byte volume holds 16 times as many queries
    "c2p64": Workload("c2-partial64-d32", 1_000_000, 32, "lognormal", 4, 128, 40.0, 1024, 32, 1000, 10, "uniform",
                      rerank_top=64),
    "c3p64": Workload("c3-partial64-d128", 2_000_000, 128, "lognormal", 8, 180, 70.0, 4096, 32, 1000, 10, "uniform",
                      rerank_top=64),
    # the same tables compressed to 8 bits per component (Sec. 6)
    "c2e4m3": Workload("c2-e4m3-d32", 1_000_000, 32, "lognormal", 4, 128, 40.0, 64, 32, 1000, 10, "uniform",
                       codec="e4m3"),
    "c3e4m3": Workload("c3-e4m3-d128", 2_000_000, 128, "lognormal", 8, 180, 70.0, 256, 32, 1000, 10, "uniform",
                       codec="e4m3"),
    # ... and the host-resident table compressed: half the bytes per query cross PCIe (Sec. 6 with Eq. 4)
    "c5e4m3": Workload("c5-host-e4m3-d128", 8_800_000, 128, "lognormal", 8, 180, 70.0, 1024, 32, 1000, 10, "zipf",
                       host_resident=True, codec="e4m3"),
}


def scaled(w: Workload, **changes) -> Workload:
    """A copy of a workload with some fields replaced (smaller n_docs, B, ...)."""
    return dataclasses.replace(w, **changes)


def _np_rng(seed: int, stream: int, index: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, index])))


def _torch_seed(seed: int, stream: int, index: int) -> int:
    # any fixed injective-enough mixing; 63-bit result
    x = (seed * 0x9E3779B97F4A7C15 + stream * 0xBF58476D1CE4E5B9 + index * 0x94D049BB133111EB) & ((1 << 63) - 1)
    return x


def token_counts(w: Workload, seed: int = DEFAULT_SEED) -> np.ndarray:
    """Tokens per document, int64 [n_docs]."""
    rng = _np_rng(seed, _S_COUNTS)
    if w.count_law == "uniform":
        return rng.integers(w.count_lo, w.count_hi + 1, size=w.n_docs, dtype=np.int64)
    if w.count_law == "lognormal":
        mu = math.log(w.count_mean) - 0.5 * w.count_sigma ** 2   # so that E[X] = count_mean
        x = rng.lognormal(mu, w.count_sigma, size=w.n_docs)
        return np.clip(np.rint(x), w.count_lo, w.count_hi).astype(np.int64)
    raise ValueError(w.count_law)


def offsets_from_counts(counts: np.ndarray) -> np.ndarray:
    """CSR row offsets, int64 [n_docs+1], offsets[0] = 0."""
    off = np.zeros(counts.shape[0] + 1, dtype=np.int64)
    np.cumsum(counts, out=off[1:])
    return off


_ROWS_PER_CHUNK = 1 << 21


def unit_rows(n_rows: int, dim: int, seed: int, stream: int, device="cpu", first_chunk: int = 0,
              out: torch.Tensor | None = None) -> torch.Tensor:
    """[n_rows, dim] binary16: each row drawn N(0,1) in fp32, scaled to unit L2 norm in fp32,
    then rounded to nearest-even binary16.  Drawn in fixed chunks of rows, one generator seed per
    chunk.  If `out` is given (any device, e.g. pinned host memory) chunks are copied into it."""
    device = torch.device(device)
    res = out if out is not None else torch.empty((n_rows, dim), dtype=torch.float16, device=device)
    assert res.shape == (n_rows, dim) and res.dtype == torch.float16
    gen = torch.Generator(device=device)
    c = 0
    for r0 in range(0, n_rows, _ROWS_PER_CHUNK):
        r1 = min(n_rows, r0 + _ROWS_PER_CHUNK)
        gen.manual_seed(_torch_seed(seed, stream, first_chunk + c))
        x = torch.randn((r1 - r0, dim), generator=gen, device=device, dtype=torch.float32)
        x /= x.norm(dim=1, keepdim=True).clamp_min_(1e-30)
        res[r0:r1].copy_(x.to(torch.float16))
        c += 1
    return res


def table(w: Workload, seed: int = DEFAULT_SEED, device="cpu", out: torch.Tensor | None = None):
    """(emb [T,dim] binary16 torch tensor, offsets int64 numpy [n_docs+1])."""
    off = offsets_from_counts(token_counts(w, seed))
    emb = unit_rows(int(off[-1]), w.dim, seed, _S_TOKENS, device=device, out=out)
    return emb, off


def queries(w: Workload, seed: int = DEFAULT_SEED, batch: int = 0, device="cpu") -> torch.Tensor:
    """[B, Q, dim] binary16 query token vectors for batch number `batch`."""
    x = unit_rows(w.B * w.Q, w.dim, seed, _S_QUERIES, device=device, first_chunk=batch * 4096)
    return x.view(w.B, w.Q, w.dim)


class _Zipf:
    """Bounded Zipf over ranks 1..n, P(r) ~ r^-alpha, rank -> document id through a seeded
    permutation so that popular documents are scattered over the table."""

    def __init__(self, n: int, alpha: float, seed: int):
        wts = np.arange(1, n + 1, dtype=np.float64) ** (-alpha)
        self.cdf = np.cumsum(wts)
        self.cdf /= self.cdf[-1]
        self.perm = _np_rng(seed, _S_PERM).permutation(n).astype(np.int64)

    def draw(self, rng: np.random.Generator, m: int) -> np.ndarray:
        r = np.searchsorted(self.cdf, rng.random(m), side="left")
        return self.perm[np.minimum(r, self.perm.shape[0] - 1)]


_zipf_cache: dict = {}


def _first_distinct(draw, K: int) -> np.ndarray:
    """First K distinct values of the stream produced by draw(m), in order of first appearance."""
    got = np.empty(0, dtype=np.int64)
    m = K + K // 4 + 16
    while True:
        got = np.concatenate([got, draw(m)])
        _, first = np.unique(got, return_index=True)
        if first.shape[0] >= K:
            return got[np.sort(first)[:K]]
        m *= 2


def candidates(w: Workload, seed: int = DEFAULT_SEED, batch: int = 0) -> np.ndarray:
    """[B, K] int64 candidate document ids, distinct within a query."""
    if w.K > w.n_docs:
        raise ValueError("K exceeds the number of documents")
    out = np.empty((w.B, w.K), dtype=np.int64)
    if w.cand_law == "zipf":
        key = (w.n_docs, w.zipf_alpha, seed)
        if key not in _zipf_cache:
            _zipf_cache.clear()
            _zipf_cache[key] = _Zipf(w.n_docs, w.zipf_alpha, seed)
        z = _zipf_cache[key]
    for b in range(w.B):
        rng = _np_rng(seed, _S_CANDS, batch * 1_000_003 + b)
        if w.cand_law == "uniform":
            out[b] = _first_distinct(lambda m: rng.integers(0, w.n_docs, size=m, dtype=np.int64), w.K)
        elif w.cand_law == "zipf":
            out[b] = _first_distinct(lambda m: z.draw(rng, m), w.K)
        else:
            raise ValueError(w.cand_law)
    return out


def subtable(emb: torch.Tensor, off: np.ndarray, cand: np.ndarray):
    """The part of a table a candidate sample refers to, as a small table of its own:
    (rows [T',dim] binary16 numpy on the host, offsets int64 [U+1], cand remapped into 0..U-1,
    ids int64 [U] = the original id of each local document).  Local ids keep the order of the
    original ids, so ranking ties resolve the same way.  `emb` may live on any device; only the
    needed rows are copied."""
    ids, local = np.unique(np.asarray(cand, dtype=np.int64), return_inverse=True)
    counts = off[ids + 1] - off[ids]
    loc_off = offsets_from_counts(counts)
    total = int(loc_off[-1])
    # row index list: for local doc u, rows off[ids[u]] + 0..counts[u]-1
    start = np.repeat(off[ids] - loc_off[:-1], counts)
    rows = start + np.arange(total, dtype=np.int64)
    idx = torch.from_numpy(rows).to(emb.device)
    sub = emb.index_select(0, idx).cpu().numpy() if total else np.zeros((0, emb.shape[1]), dtype=np.float16 if emb.dtype == torch.float16 else np.uint8)
    return sub, loc_off, local.reshape(np.asarray(cand).shape).astype(np.int64), ids


E4M3_MAX = 448.0


def compress_e4m3(emb: torch.Tensor, off: np.ndarray):
    """An 8-bit copy of a table: (codes uint8 [T,dim] in the OCP E4M3 format, scale float32 numpy [n_docs]).
    Every document gets one scale = (largest magnitude in the document) / 448 (1 for an empty or all-zero
    document); a stored value stands for scale * decode(code).  Rounding is torch's float8_e4m3fn
    conversion (round to nearest even).  Works on the device the table lives on, chunk by chunk."""
    n_docs = off.shape[0] - 1
    dev = emb.device
    counts = torch.from_numpy(np.diff(off)).to(dev)
    doc_of_row = torch.repeat_interleave(torch.arange(n_docs, device=dev), counts)
    amax = torch.zeros(n_docs, dtype=torch.float32, device=dev)
    codes = torch.empty(emb.shape, dtype=torch.uint8, device=dev)
    step = _ROWS_PER_CHUNK
    for r0 in range(0, emb.shape[0], step):
        r1 = min(emb.shape[0], r0 + step)
        row_max = emb[r0:r1].float().abs().amax(dim=1)
        amax.scatter_reduce_(0, doc_of_row[r0:r1], row_max, reduce="amax", include_self=True)
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax))
    for r0 in range(0, emb.shape[0], step):
        r1 = min(emb.shape[0], r0 + step)
        x = emb[r0:r1].float() / scale[doc_of_row[r0:r1]].unsqueeze(1)
        codes[r0:r1] = x.clamp_(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn).view(torch.uint8)
    return codes, scale.cpu().numpy()
