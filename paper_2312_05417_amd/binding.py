"""Thin Python binding of the C-ABI library (include/espn.h): same names, argument marshalling only.

Every step of the path runs in the HIP kernels of libespn.so.  There is no fallback: if the
library has not been built, loading fails with an error that says how to build it.
torch is used for device memory and streams only (data_ptr() and the current stream handle).
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libespn.so")

ESPN_OK = 0
ESPN_ERR_ARG, ESPN_ERR_SHAPE, ESPN_ERR_OFFSETS, ESPN_ERR_ID_RANGE = 1, 2, 3, 4
ESPN_ERR_NOMEM, ESPN_ERR_HIP, ESPN_ERR_UNSUPPORTED = 5, 6, 7
ESPN_RESIDENT_HBM, ESPN_RESIDENT_HOST_PINNED, ESPN_RESIDENT_HOST = 0, 1, 2
ESPN_BATCH_LANES = 3
ESPN_FETCH_AUTO, ESPN_FETCH_STREAMING, ESPN_FETCH_CACHED = 0, 1, 2

_c_i32, _c_i64, _c_p, _c_sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t

# name -> (restype, argtypes); one entry per declaration in include/espn.h
SIGNATURES = {
    "espn_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "espn_last_error": (ctypes.c_char_p, []),
    "espn_table_load": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i32, _c_i32, _c_i32, ctypes.POINTER(_c_p)]),
    "espn_table_load_e4m3": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_i64, _c_i32, _c_i32, _c_i32, ctypes.POINTER(_c_p)]),
    "espn_table_free": (ctypes.c_int, [_c_p]),
    "espn_table_set_fetch": (ctypes.c_int, [_c_p, _c_i32]),
    "espn_table_sample": (ctypes.c_int, [_c_p, _c_p, _c_i32, _c_i32, _c_p]),
    "espn_table_sharing_estimate": (ctypes.c_int, [_c_p, ctypes.POINTER(ctypes.c_float)]),
    "espn_table_info": (ctypes.c_int, [_c_p, ctypes.POINTER(_c_i64), ctypes.POINTER(_c_i64),
                                       ctypes.POINTER(_c_i32), ctypes.POINTER(_c_i32), ctypes.POINTER(_c_i32)]),
    "espn_score": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_p, _c_p]),
    "espn_topk": (ctypes.c_int, [_c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_p, _c_p, _c_p]),
    "espn_workspace_bytes": (_c_sz, [_c_i32, _c_i32]),
    "espn_rerank_plan": (ctypes.c_int, [_c_p, _c_i32, _c_i32, _c_i32, _c_i32, ctypes.POINTER(_c_i32),
                                        ctypes.POINTER(_c_i32), ctypes.POINTER(_c_i32)]),
    "espn_rerank_plan_kernels": (ctypes.c_int, [_c_p, _c_i32, _c_i32, _c_i32, _c_i32, ctypes.c_char_p, _c_sz]),
    "espn_rerank": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_p, _c_p, _c_p, _c_sz, _c_p]),
    "espn_batches_workspace_bytes": (_c_sz, [_c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_i32]),
    "espn_batches_plan": (ctypes.c_int, [_c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_i32, ctypes.POINTER(_c_i32),
                                         ctypes.POINTER(_c_i32), ctypes.POINTER(_c_i32), ctypes.c_char_p, _c_sz]),
    "espn_rerank_batches": (ctypes.c_int, [_c_p, _c_i32, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_p, _c_p, _c_p,
                                           _c_sz, _c_p]),
    "espn_rerank_noalloc": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_p, _c_p, _c_p]),
    "espn_rerank_partial": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_i32, _c_p, _c_p,
                                           _c_p, _c_sz, _c_p]),
    "espn_rerank_prior": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_p, ctypes.c_float, _c_i32, _c_i32, _c_i32, _c_i32,
                                         _c_p, _c_p, _c_p, _c_sz, _c_p]),
    "espn_merge_topk": (ctypes.c_int, [_c_p, _c_p, _c_i32, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_p, _c_p, _c_p]),
    "espn_batch_threshold": (ctypes.c_double, [ctypes.c_double, ctypes.c_double, ctypes.c_double]),
    "espn_table_check": (ctypes.c_int, [_c_p, _c_p]),
    "espn_staging_create": (ctypes.c_int, [_c_p, _c_i64, _c_i64]),
    "espn_staging_create_ring": (ctypes.c_int, [_c_p, _c_i32, _c_i64, _c_i64]),
    "espn_prefetch": (ctypes.c_int, [_c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_p]),
    "espn_prefetch_packed": (ctypes.c_int, [_c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_p]),
    "espn_rerank_staged": (ctypes.c_int, [_c_p, _c_i32, _c_p, _c_p, _c_i32, _c_i32, _c_i32, _c_i32, _c_p, _c_p,
                                          _c_p, _c_sz, _c_p]),
    "espn_staging_counters": (ctypes.c_int, [_c_p, _c_i32, _c_p, ctypes.POINTER(ctypes.c_uint64)]),
}

_lib = None


class EspnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("espn status %d (%s): %s" % (status, status_string(status), message))
        self.status = status


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                "%s is missing: build it with `python -m paper_2312_05417_amd.build` "
                "(or __graft_entry__.build()); there is no non-HIP path" % LIB_PATH)
        handle = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(handle, name)          # AttributeError if the symbol is not exported
            fn.restype, fn.argtypes = res, args
        _lib = handle
    return _lib


def status_string(status: int) -> str:
    return lib().espn_status_string(int(status)).decode()


def last_error() -> str:
    return lib().espn_last_error().decode()


def _check(status: int) -> None:
    if status != ESPN_OK:
        raise EspnError(status, last_error())


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def _workspace(B: int, K: int, device, stream) -> torch.Tensor:
    """Scratch for one call.  It is handed back to torch's allocator as soon as the call returns, while
    the kernels may still be running, so it has to be allocated in the order of the stream they run on:
    a block released in stream order is only reused by work that stream runs later."""
    nbytes = int(lib().espn_workspace_bytes(B, K))
    if isinstance(stream, torch.cuda.Stream):
        with torch.cuda.stream(stream):
            return torch.empty(nbytes, dtype=torch.uint8, device=device)
    if stream is not None:
        raise ValueError("pass a workspace along with a raw stream handle: torch cannot allocate in its order")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError("%s must be a contiguous CUDA tensor of dtype %s" % (name, dtype))
    return t.data_ptr()


class Table:
    """Handle of a loaded table (espn_table_load / espn_table_free).  Keeps `emb` alive."""

    def __init__(self, emb: torch.Tensor, offsets, dim: int | None = None, device: int | None = None,
                 doc_scale=None, pageable: bool = False):
        import numpy as np
        want = torch.float16 if doc_scale is None else torch.uint8
        if emb.dtype != want or emb.dim() != 2 or not emb.is_contiguous():
            raise TypeError("emb must be a contiguous [rows, dim] tensor of %s" % want)
        off = np.ascontiguousarray(np.asarray(offsets, dtype=np.int64))
        if off.ndim != 1 or off.shape[0] < 1:
            raise TypeError("offsets must be a 1-d int64 array of n_docs + 1 entries")
        if int(off[-1]) != emb.shape[0]:
            raise ValueError("offsets[-1] = %d but emb has %d rows" % (int(off[-1]), emb.shape[0]))
        if emb.is_cuda:
            residency, dev = ESPN_RESIDENT_HBM, emb.device.index
        elif emb.is_pinned():
            residency, dev = ESPN_RESIDENT_HOST_PINNED, (torch.cuda.current_device() if device is None else device)
        elif pageable:
            residency, dev = ESPN_RESIDENT_HOST, (torch.cuda.current_device() if device is None else device)
        else:
            raise TypeError("emb must live in device memory or in pinned host memory (ordinary host memory: "
                            "pass pageable=True; only espn_prefetch_packed can then fill staging slots)")
        self.emb, self.n_docs, self.dim = emb, off.shape[0] - 1, emb.shape[1] if dim is None else dim
        self.device = dev
        self._h = _c_p()
        if doc_scale is None:
            _check(lib().espn_table_load(emb.data_ptr(), off.ctypes.data, self.n_docs, self.dim, residency, dev,
                                         ctypes.byref(self._h)))
        else:
            sc = np.ascontiguousarray(np.asarray(doc_scale, dtype=np.float32))
            if sc.shape != (self.n_docs,):
                raise ValueError("doc_scale must hold one value per document")
            _check(lib().espn_table_load_e4m3(emb.data_ptr(), sc.ctypes.data, off.ctypes.data, self.n_docs, self.dim,
                                              residency, dev, ctypes.byref(self._h)))

    def free(self) -> None:
        if self._h:
            lib().espn_table_free(self._h)
            self._h = _c_p()

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    @property
    def handle(self):
        if not self._h:
            raise ValueError("table has been freed")
        return self._h

    def info(self) -> dict:
        n, rows, dim, res, dev = _c_i64(), _c_i64(), _c_i32(), _c_i32(), _c_i32()
        _check(lib().espn_table_info(self.handle, ctypes.byref(n), ctypes.byref(rows), ctypes.byref(dim),
                                     ctypes.byref(res), ctypes.byref(dev)))
        return {"n_docs": n.value, "total_rows": rows.value, "dim": dim.value, "residency": res.value,
                "device": dev.value}


def espn_table_load(emb: torch.Tensor, offsets, device: int | None = None, pageable: bool = False) -> Table:
    return Table(emb, offsets, device=device, pageable=pageable)


def espn_table_load_e4m3(codes: torch.Tensor, doc_scale, offsets, device: int | None = None,
                         pageable: bool = False) -> Table:
    return Table(codes, offsets, device=device, doc_scale=doc_scale, pageable=pageable)


def espn_table_set_fetch(table: Table, mode: int) -> None:
    _check(lib().espn_table_set_fetch(table.handle, mode))


def espn_table_sample(table: Table, cand: torch.Tensor, stream=None) -> float:
    """Samples the batch's candidate lists (synchronous); returns the estimate the table now holds."""
    if cand.dim() != 2:
        raise ValueError("cand must be [B,K]")
    _check(lib().espn_table_sample(table.handle, _dev(cand, torch.int64, "cand"), cand.shape[0], cand.shape[1],
                                   _stream_ptr(stream)))
    return espn_table_sharing_estimate(table)


def espn_table_sharing_estimate(table: Table) -> float:
    out = ctypes.c_float(0.0)
    _check(lib().espn_table_sharing_estimate(table.handle, ctypes.byref(out)))
    return float(out.value)


def espn_table_free(table: Table) -> None:
    table.free()


def espn_workspace_bytes(B: int, K: int) -> int:
    return int(lib().espn_workspace_bytes(B, K))


def espn_rerank_plan(table: Table, B: int, Q: int, K: int, k: int) -> dict:
    """How a batch of this shape would run: slices per query, candidates per slice, kernel launches."""
    slices, slice_, launches = _c_i32(), _c_i32(), _c_i32()
    _check(lib().espn_rerank_plan(table.handle, B, Q, K, k, ctypes.byref(slices), ctypes.byref(slice_),
                                  ctypes.byref(launches)))
    return {"slices": slices.value, "slice": slice_.value, "launches": launches.value}


def espn_rerank_plan_kernels(table: Table, B: int, Q: int, K: int, k: int) -> list:
    """Profiler names of the kernels espn_rerank launches for this shape (scoring, then ranking if separate)."""
    buf = ctypes.create_string_buffer(256)
    _check(lib().espn_rerank_plan_kernels(table.handle, B, Q, K, k, buf, 256))
    text = buf.value.decode()
    return text.split(";") if text else []


def _batch_shape(q: torch.Tensor, cand: torch.Tensor):
    if q.dim() != 3 or cand.dim() != 2 or q.shape[0] != cand.shape[0]:
        raise ValueError("expected q [B,Q,dim] and cand [B,K]")
    return q.shape[0], q.shape[1], cand.shape[1]


def espn_score(table: Table, q: torch.Tensor, cand: torch.Tensor, scores: torch.Tensor | None = None,
               stream=None) -> torch.Tensor:
    B, Q, K = _batch_shape(q, cand)
    if q.shape[2] != table.dim:
        raise ValueError("q has dim %d, table has %d" % (q.shape[2], table.dim))
    if scores is None:
        scores = torch.empty((B, K), dtype=torch.float32, device=q.device)
    if tuple(scores.shape) != (B, K):
        raise ValueError("scores must be [B,K]")
    _check(lib().espn_score(table.handle, _dev(q, torch.float16, "q"), _dev(cand, torch.int64, "cand"), B, Q, K,
                            _dev(scores, torch.float32, "scores"), _stream_ptr(stream)))
    return scores


def espn_topk(scores: torch.Tensor, cand: torch.Tensor, k: int, out_ids: torch.Tensor | None = None,
              out_scores: torch.Tensor | None = None, stream=None):
    if scores.dim() != 2 or scores.shape != cand.shape:
        raise ValueError("scores and cand must both be [B,K]")
    B, K = scores.shape
    if out_ids is None:
        out_ids = torch.empty((B, max(k, 0)), dtype=torch.int64, device=scores.device)
    if out_scores is None:
        out_scores = torch.empty((B, max(k, 0)), dtype=torch.float32, device=scores.device)
    _check(lib().espn_topk(_dev(scores, torch.float32, "scores"), _dev(cand, torch.int64, "cand"), B, K, k,
                           _dev(out_ids, torch.int64, "out_ids"), _dev(out_scores, torch.float32, "out_scores"),
                           _stream_ptr(stream)))
    return out_ids, out_scores


def espn_rerank(table: Table, q: torch.Tensor, cand: torch.Tensor, k: int, out_ids: torch.Tensor | None = None,
                out_scores: torch.Tensor | None = None, workspace: torch.Tensor | None = None, stream=None):
    """Whole hot path.  Returns (out_ids [B,k] int64, out_scores [B,k] float32)."""
    B, Q, K = _batch_shape(q, cand)
    if q.shape[2] != table.dim:
        raise ValueError("q has dim %d, table has %d" % (q.shape[2], table.dim))
    if out_ids is None:
        out_ids = torch.empty((B, max(k, 0)), dtype=torch.int64, device=q.device)
    if out_scores is None:
        out_scores = torch.empty((B, max(k, 0)), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _workspace(B, K, q.device, stream)
    _check(lib().espn_rerank(table.handle, _dev(q, torch.float16, "q"), _dev(cand, torch.int64, "cand"), B, Q, K, k,
                             _dev(out_ids, torch.int64, "out_ids"), _dev(out_scores, torch.float32, "out_scores"),
                             _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream_ptr(stream)))
    return out_ids, out_scores


def espn_batches_workspace_bytes(table: Table, n_batches: int, B: int, Q: int, K: int, k: int) -> int:
    return int(lib().espn_batches_workspace_bytes(table.handle, n_batches, B, Q, K, k))


def espn_batches_plan(table: Table, n_batches: int, B: int, Q: int, K: int, k: int) -> dict:
    """How a queue of this shape would run: batches per launch, launches, streams, kernel names of one chunk."""
    fuse, launches, streams = _c_i32(), _c_i32(), _c_i32()
    buf = ctypes.create_string_buffer(256)
    _check(lib().espn_batches_plan(table.handle, n_batches, B, Q, K, k, ctypes.byref(fuse), ctypes.byref(launches),
                                   ctypes.byref(streams), buf, 256))
    text = buf.value.decode()
    return {"fuse": fuse.value, "launches": launches.value, "streams": streams.value,
            "kernels": text.split(";") if text else []}


def pointer_list(tensors, dtype, name: str):
    """A host array of device pointers (what espn_rerank_batches takes for q, cand, out_ids, out_scores)."""
    return (_c_p * len(tensors))(*[_dev(t, dtype, "%s[%d]" % (name, i)) for i, t in enumerate(tensors)])


def espn_rerank_batches(table: Table, qs, cands, k: int, out_ids=None, out_scores=None,
                        workspace: torch.Tensor | None = None, stream=None):
    """A queue of batches of one shape in one call.  qs, cands: lists of [B,Q,dim] / [B,K] tensors.
    Returns (list of out_ids, list of out_scores)."""
    n = len(qs)
    if n != len(cands):
        raise ValueError("as many query tensors as candidate tensors are needed")
    if n == 0:
        return [], []
    B, Q, K = _batch_shape(qs[0], cands[0])
    for q, c in zip(qs, cands):
        if _batch_shape(q, c) != (B, Q, K) or q.shape[2] != table.dim:
            raise ValueError("all batches of a call must have one shape, with the table's dim")
    dev = qs[0].device
    if out_ids is None:
        out_ids = [torch.empty((B, max(k, 0)), dtype=torch.int64, device=dev) for _ in range(n)]
    if out_scores is None:
        out_scores = [torch.empty((B, max(k, 0)), dtype=torch.float32, device=dev) for _ in range(n)]
    if workspace is None:
        nbytes = espn_batches_workspace_bytes(table, n, B, Q, K, k)
        if isinstance(stream, torch.cuda.Stream):
            with torch.cuda.stream(stream):
                workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        elif stream is None:
            workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        else:
            raise ValueError("pass a workspace along with a raw stream handle: torch cannot allocate in its order")
    _check(lib().espn_rerank_batches(table.handle, n, pointer_list(qs, torch.float16, "q"),
                                     pointer_list(cands, torch.int64, "cand"), B, Q, K, k,
                                     pointer_list(out_ids, torch.int64, "out_ids"),
                                     pointer_list(out_scores, torch.float32, "out_scores"),
                                     _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream_ptr(stream)))
    return out_ids, out_scores


ESPN_NOALLOC_MAX_PAIRS = 4 * 1024 * 1024


def espn_rerank_noalloc(table: Table, q: torch.Tensor, cand: torch.Tensor, k: int, out_ids: torch.Tensor,
                        out_scores: torch.Tensor, stream=None):
    """espn_rerank without a workspace: the library's static scratch holds the scores.  The outputs are the
    caller's (this wrapper allocates nothing either)."""
    B, Q, K = _batch_shape(q, cand)
    if q.shape[2] != table.dim:
        raise ValueError("q has dim %d, table has %d" % (q.shape[2], table.dim))
    _check(lib().espn_rerank_noalloc(table.handle, _dev(q, torch.float16, "q"), _dev(cand, torch.int64, "cand"),
                                     B, Q, K, k, _dev(out_ids, torch.int64, "out_ids"),
                                     _dev(out_scores, torch.float32, "out_scores"), _stream_ptr(stream)))
    return out_ids, out_scores


def espn_table_check(table: Table, stream=None) -> None:
    """Waits for the stream; raises EspnError(ESPN_ERR_ID_RANGE) if a kernel met an id out of range."""
    _check(lib().espn_table_check(table.handle, _stream_ptr(stream)))


def espn_staging_create(table: Table, capacity_rows: int, capacity_docs: int) -> None:
    _check(lib().espn_staging_create(table.handle, capacity_rows, capacity_docs))


def espn_staging_create_ring(table: Table, n_slots: int, capacity_rows: int, capacity_docs: int) -> None:
    _check(lib().espn_staging_create_ring(table.handle, n_slots, capacity_rows, capacity_docs))


def espn_prefetch(table: Table, cand: torch.Tensor, slot: int, side_stream=None) -> None:
    if cand.dim() != 2:
        raise ValueError("cand must be [B,K]")
    _check(lib().espn_prefetch(table.handle, _dev(cand, torch.int64, "cand"), cand.shape[0], cand.shape[1], slot,
                               _stream_ptr(side_stream)))


def espn_prefetch_packed(table: Table, cand_host: torch.Tensor, slot: int, side_stream=None) -> None:
    """The host-side engine: cand_host is a contiguous int64 CPU tensor [B,K]; blocks while it packs."""
    if cand_host.dim() != 2:
        raise ValueError("cand_host must be [B,K]")
    if cand_host.is_cuda or cand_host.dtype != torch.int64 or not cand_host.is_contiguous():
        raise ValueError("cand_host must be a contiguous int64 tensor in host memory")
    _check(lib().espn_prefetch_packed(table.handle, cand_host.data_ptr(), cand_host.shape[0], cand_host.shape[1], slot,
                                      _stream_ptr(side_stream)))


def espn_rerank_staged(table: Table, slot: int, q: torch.Tensor, cand: torch.Tensor, k: int,
                       out_ids: torch.Tensor | None = None, out_scores: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None, stream=None):
    """Returns (out_ids, out_scores, workspace); the workspace starts with all scores, fp32 [B,K]."""
    B, Q, K = _batch_shape(q, cand)
    if q.shape[2] != table.dim:
        raise ValueError("q has dim %d, table has %d" % (q.shape[2], table.dim))
    if out_ids is None:
        out_ids = torch.empty((B, max(k, 0)), dtype=torch.int64, device=q.device)
    if out_scores is None:
        out_scores = torch.empty((B, max(k, 0)), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = _workspace(B, K, q.device, stream)
    _check(lib().espn_rerank_staged(table.handle, slot, _dev(q, torch.float16, "q"), _dev(cand, torch.int64, "cand"),
                                    B, Q, K, k, _dev(out_ids, torch.int64, "out_ids"),
                                    _dev(out_scores, torch.float32, "out_scores"),
                                    _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream_ptr(stream)))
    return out_ids, out_scores, workspace


def espn_staging_counters(table: Table, slot: int, stream=None) -> dict:
    out = (ctypes.c_uint64 * 4)()
    _check(lib().espn_staging_counters(table.handle, slot, _stream_ptr(stream), out))
    return {"distinct_docs": int(out[0]), "rows": int(out[1]), "pcie_bytes": int(out[2]), "capacity_rows": int(out[3])}


def _outputs(B, k, device, out_ids, out_scores):
    if out_ids is None:
        out_ids = torch.empty((B, max(k, 0)), dtype=torch.int64, device=device)
    if out_scores is None:
        out_scores = torch.empty((B, max(k, 0)), dtype=torch.float32, device=device)
    return out_ids, out_scores


def espn_rerank_partial(table: Table, q: torch.Tensor, cand: torch.Tensor, R: int, k: int,
                        out_ids: torch.Tensor | None = None, out_scores: torch.Tensor | None = None,
                        workspace: torch.Tensor | None = None, stream=None):
    B, Q, K = _batch_shape(q, cand)
    if q.shape[2] != table.dim:
        raise ValueError("q has dim %d, table has %d" % (q.shape[2], table.dim))
    out_ids, out_scores = _outputs(B, k, q.device, out_ids, out_scores)
    if workspace is None:
        workspace = _workspace(B, max(R, 0), q.device, stream)
    _check(lib().espn_rerank_partial(table.handle, _dev(q, torch.float16, "q"), _dev(cand, torch.int64, "cand"),
                                     B, Q, K, R, k, _dev(out_ids, torch.int64, "out_ids"),
                                     _dev(out_scores, torch.float32, "out_scores"),
                                     _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream_ptr(stream)))
    return out_ids, out_scores


def espn_rerank_prior(table: Table, q: torch.Tensor, cand: torch.Tensor, prior: torch.Tensor, alpha: float, k: int,
                      out_ids: torch.Tensor | None = None, out_scores: torch.Tensor | None = None,
                      workspace: torch.Tensor | None = None, stream=None):
    """Returns (out_ids, out_scores, workspace); the workspace starts with all totals, fp32 [B,K]."""
    B, Q, K = _batch_shape(q, cand)
    if q.shape[2] != table.dim:
        raise ValueError("q has dim %d, table has %d" % (q.shape[2], table.dim))
    if tuple(prior.shape) != (B, K):
        raise ValueError("prior must be [B,K]")
    out_ids, out_scores = _outputs(B, k, q.device, out_ids, out_scores)
    if workspace is None:
        workspace = _workspace(B, K, q.device, stream)
    _check(lib().espn_rerank_prior(table.handle, _dev(q, torch.float16, "q"), _dev(cand, torch.int64, "cand"),
                                   _dev(prior, torch.float32, "prior"), float(alpha), B, Q, K, k,
                                   _dev(out_ids, torch.int64, "out_ids"), _dev(out_scores, torch.float32, "out_scores"),
                                   _dev(workspace, torch.uint8, "workspace"), workspace.numel(), _stream_ptr(stream)))
    return out_ids, out_scores, workspace


def espn_merge_topk(ids_a: torch.Tensor, scores_a: torch.Tensor, ids_b: torch.Tensor, scores_b: torch.Tensor, k: int,
                    out_ids: torch.Tensor | None = None, out_scores: torch.Tensor | None = None, stream=None):
    if ids_a.dim() != 2 or ids_b.dim() != 2 or ids_a.shape != scores_a.shape or ids_b.shape != scores_b.shape \
            or ids_a.shape[0] != ids_b.shape[0]:
        raise ValueError("expected ids/scores [B,ka] and [B,kb]")
    B = ids_a.shape[0]
    out_ids, out_scores = _outputs(B, k, ids_a.device, out_ids, out_scores)
    _check(lib().espn_merge_topk(_dev(ids_a, torch.int64, "ids_a"), _dev(scores_a, torch.float32, "scores_a"),
                                 ids_a.shape[1], _dev(ids_b, torch.int64, "ids_b"),
                                 _dev(scores_b, torch.float32, "scores_b"), ids_b.shape[1], B, k,
                                 _dev(out_ids, torch.int64, "out_ids"), _dev(out_scores, torch.float32, "out_scores"),
                                 _stream_ptr(stream)))
    return out_ids, out_scores


def espn_batch_threshold(bandwidth_bytes_per_s: float, budget_s: float, bytes_per_query: float) -> float:
    return float(lib().espn_batch_threshold(bandwidth_bytes_per_s, budget_s, bytes_per_query))
