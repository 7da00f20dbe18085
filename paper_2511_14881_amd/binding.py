"""Thin Python face of the C-ABI library (``include/silvertorch.h``): the same entry points,
argument marshalling only.  PyTorch supplies device memory and the stream; every step of the
retrieval path runs inside the library's HIP kernels.  There is no fallback: if the shared
library has not been built, the first call raises."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libsilvertorch.so")
_lib = None

ST_OK, ST_EINVAL, ST_ENOMEM, ST_EHIP, ST_EWORKSPACE = 0, -1, -2, -3, -4

EXPORTS = [
    "st_last_error", "st_version", "st_bloom_build", "st_bloom_free", "st_bloom_bytes",
    "st_bloom_layout_bytes", "st_bloom_n_items", "st_bloom_export_signatures", "st_bloom_mask",
    "st_search_workspace_bytes", "st_search", "st_search_multitask", "st_score_pairs",
    "st_search_plan", "st_set_scoring_path", "st_timing_begin", "st_timing_end",
    "st_search_overflow_flags_offset", "st_bloom_mask_expr", "st_search_expr_workspace_bytes",
    "st_search_expr", "st_search_ivf_workspace_bytes", "st_search_ivf", "st_quantize_global", "st_value_model",
    "st_search_host_plan", "st_stream_read", "st_search_static",
]

ST_OP_LEAF, ST_OP_AND, ST_OP_OR, ST_OP_NOT = 0, 1, 2, 3  # operations of a filter program


class StError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"silvertorch error {code}: {msg}")
        self.code = code


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it first "
                               "(python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.st_last_error.restype = C.c_char_p
        L.st_last_error.argtypes = []
        L.st_version.restype = i32
        L.st_bloom_build.restype = C.c_int
        L.st_bloom_build.argtypes = [p, p, i64, i32, i32, p, C.POINTER(p)]
        L.st_bloom_free.restype = C.c_int
        L.st_bloom_free.argtypes = [p]
        L.st_bloom_bytes.restype = i64
        L.st_bloom_bytes.argtypes = [p]
        L.st_bloom_layout_bytes.restype = i64
        L.st_bloom_layout_bytes.argtypes = [i64, i32]
        L.st_bloom_n_items.restype = i64
        L.st_bloom_n_items.argtypes = [p]
        L.st_bloom_export_signatures.restype = C.c_int
        L.st_bloom_export_signatures.argtypes = [p, p, p]
        L.st_bloom_mask.restype = C.c_int
        L.st_bloom_mask.argtypes = [p, p, p, i32, p, p]
        L.st_search_workspace_bytes.restype = i64
        L.st_search_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
        L.st_search_overflow_flags_offset.restype = i64
        L.st_search_overflow_flags_offset.argtypes = [i64, i32, i32, i32, i32]
        L.st_search.restype = C.c_int
        L.st_search.argtypes = [p, p, p, i64, i32, p, p, i32, p, p, i32, p, p, p, p, i64, p]
        L.st_search_static.restype = C.c_int
        L.st_search_static.argtypes = [p, p, p, i64, i32, p, p, i32, p, p, i32, p, p, p, p]
        L.st_search_multitask.restype = C.c_int
        L.st_search_multitask.argtypes = [p, p, p, i64, i32, p, p, i32, i32, p, p, p, i32, p, p, p, p,
                                          i64, p]
        L.st_score_pairs.restype = C.c_int
        L.st_score_pairs.argtypes = [p, p, i32, p, p, p, p, i64, p, p, p]
        L.st_search_plan.restype = i32
        L.st_search_plan.argtypes = [i64, i32, i32, i32, p, i32, p]
        L.st_set_scoring_path.restype = i32
        L.st_set_scoring_path.argtypes = [i32]
        L.st_timing_begin.restype = C.c_int
        L.st_timing_begin.argtypes = [i32]
        L.st_timing_end.restype = C.c_int
        L.st_timing_end.argtypes = [p, p]
        L.st_bloom_mask_expr.restype = C.c_int
        L.st_bloom_mask_expr.argtypes = [p, p, p, p, i32, p, p]
        L.st_search_expr_workspace_bytes.restype = i64
        L.st_search_expr_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i64]
        L.st_search_expr.restype = C.c_int
        L.st_search_expr.argtypes = [p, p, p, i64, i32, p, p, i32, i32, p, p, p, p, i32, p, p, p, p, i64, p]
        L.st_search_ivf_workspace_bytes.restype = i64
        L.st_search_ivf_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32, i64]
        L.st_search_ivf.restype = C.c_int
        L.st_search_ivf.argtypes = [p, p, p, i64, i32, p, p, p, i32, i32, p, p, i32, p, p, p, i32, p, p, p, p, p,
                                    i64, p]
        L.st_value_model.restype = C.c_int
        L.st_value_model.argtypes = [p, i64, i32, p, p, i32, p, p]
        L.st_search_host_plan.restype = C.c_int
        L.st_search_host_plan.argtypes = [i64, i32, i32, i32, i32, i32, i32, p, p, p]
        L.st_stream_read.restype = C.c_int
        L.st_stream_read.argtypes = [p, i64, p, i32, p]
        L.st_quantize_global.restype = C.c_int
        L.st_quantize_global.argtypes = [p, i64, i32, p, p, p, p, p]
        _lib = L
    return _lib


def last_error() -> str:
    return lib().st_last_error().decode()


def _check(rc: int) -> int:
    if rc < 0:
        raise StError(int(rc), last_error())
    return int(rc)


def _dptr(t: torch.Tensor | None):
    return None if t is None else C.c_void_p(t.data_ptr())


def _hptr(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _stream(stream) -> C.c_void_p:
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def _need(t: torch.Tensor, dtype, name: str):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous CUDA tensor of {dtype}")


def _filters(filt_ids, filt_offsets, n: int):
    ids = np.ascontiguousarray(np.asarray(filt_ids, dtype=np.uint64))
    off = np.ascontiguousarray(np.asarray(filt_offsets, dtype=np.int64))
    if off.size != n + 1:
        raise ValueError("filt_offsets must have one more entry than there are filters")
    if off[-1] != ids.size:
        raise ValueError("filt_offsets[-1] must equal len(filt_ids)")
    return ids, off


class BloomIndex:
    """Owns an ``st_bloom*``."""

    def __init__(self, handle: int, n_items: int, m_bits: int, k_hashes: int):
        self.handle, self.n_items, self.m_bits, self.k_hashes = handle, n_items, m_bits, k_hashes

    @property
    def nbytes(self) -> int:
        return _check(lib().st_bloom_bytes(C.c_void_p(self.handle)))

    def free(self):
        if self.handle:
            _check(lib().st_bloom_free(C.c_void_p(self.handle)))
            self.handle = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def st_bloom_build(feat_offsets, feat_ids, n_items: int, m_bits: int, k_hashes: int,
                   stream=None) -> BloomIndex:
    """feat_offsets int64 [N+1] and feat_ids (int64 bit patterns of uint64) as CUDA tensors or
    numpy arrays."""
    keep = []

    def ptr(x, np_dtype):
        if isinstance(x, torch.Tensor) and x.is_cuda:
            if x.dtype != torch.int64 or not x.is_contiguous():
                raise TypeError("feature tensors must be contiguous int64")
            keep.append(x)
            return _dptr(x)
        a = x.numpy() if isinstance(x, torch.Tensor) else np.asarray(x)
        if a.dtype not in (np.dtype(np.int64), np.dtype(np.uint64)):
            a = a.astype(np_dtype)
        a = np.ascontiguousarray(a).view(np_dtype)
        keep.append(a)
        return _hptr(a)

    out = C.c_void_p()
    _check(lib().st_bloom_build(ptr(feat_offsets, np.int64), ptr(feat_ids, np.uint64), n_items, m_bits,
                                k_hashes, _stream(stream), C.byref(out)))
    return BloomIndex(out.value, n_items, m_bits, k_hashes)


def st_bloom_layout_bytes(n_items: int, m_bits: int) -> int:
    return _check(lib().st_bloom_layout_bytes(n_items, m_bits))


def st_bloom_export_signatures(bloom: BloomIndex, stream=None) -> torch.Tensor:
    words = (bloom.m_bits + 63) // 64
    out = torch.empty((bloom.n_items, words), dtype=torch.int64, device="cuda")
    _check(lib().st_bloom_export_signatures(C.c_void_p(bloom.handle), _dptr(out), _stream(stream)))
    return out


def st_bloom_mask(bloom: BloomIndex, filt_ids, filt_offsets, stream=None) -> torch.Tensor:
    n_f = len(filt_offsets) - 1
    ids, off = _filters(filt_ids, filt_offsets, n_f)
    out = torch.zeros((n_f, (bloom.n_items + 63) // 64), dtype=torch.int64, device="cuda")
    _check(lib().st_bloom_mask(C.c_void_p(bloom.handle), _hptr(ids), _hptr(off), n_f, _dptr(out),
                               _stream(stream)))
    return out


def st_search_workspace_bytes(n_items: int, d: int, batch: int, n_tasks: int, K: int) -> int:
    return _check(lib().st_search_workspace_bytes(n_items, d, batch, n_tasks, K))


def st_search_overflow_flags_offset(n_items: int, d: int, batch: int, n_tasks: int, K: int) -> int:
    return _check(lib().st_search_overflow_flags_offset(n_items, d, batch, n_tasks, K))


def st_search_plan(n_items: int, batch: int, K: int, q_split: int = 1):
    levels = np.zeros((32, 3), dtype=np.int64)
    caps = np.zeros(2, dtype=np.int64)
    n = _check(lib().st_search_plan(n_items, batch, K, q_split, _hptr(levels), 32, _hptr(caps)))
    return levels[:n].copy(), int(caps[0]), int(caps[1])


def st_search_host_plan(n_items: int, d: int, batch: int, n_tasks: int, K: int, m_bits: int, k_hashes: int,
                        filt_ids, filt_offsets) -> dict:
    """The host part of a search alone (no GPU): a summary of the groups and the schedule."""
    ids, off = _filters(filt_ids, filt_offsets, batch)
    out = np.zeros(8, dtype=np.int32)
    _check(lib().st_search_host_plan(n_items, d, batch, n_tasks, K, m_bits, k_hashes, _hptr(ids), _hptr(off),
                                     _hptr(out)))
    keys = ("distinct_filters", "mfma_groups", "dot_groups", "q_split", "waves", "levels", "table_bytes", "seed_pass")
    return {k: int(v) for k, v in zip(keys, out)}


def st_set_scoring_path(path: int) -> int:
    return int(lib().st_set_scoring_path(path))


def st_timing_begin(max_launches: int) -> None:
    _check(lib().st_timing_begin(max_launches))


def st_timing_end():
    """{'scan'|'select'|'rescue'|'expr': (total_ms, launches)}"""
    ms = np.zeros(4, dtype=np.float64)
    n = np.zeros(4, dtype=np.int64)
    _check(lib().st_timing_end(_hptr(ms), _hptr(n)))
    return {k: (float(ms[i]), int(n[i])) for i, k in enumerate(("scan", "select", "rescue", "expr"))}


class SearchBuffers:
    """Workspace and outputs for repeated searches of one shape.  n_expr_entries: room for filter
    programs of that many entries per batch (st_search_expr); None for the plain searches."""

    def __init__(self, n_items: int, d: int, batch: int, n_tasks: int, K: int, n_expr_entries: int | None = None):
        if n_expr_entries is None:
            self.nbytes = st_search_workspace_bytes(n_items, d, batch, n_tasks, K)
        else:
            self.nbytes = _check(lib().st_search_expr_workspace_bytes(n_items, d, batch, n_tasks, K, n_expr_entries))
        self._ovf = (st_search_overflow_flags_offset(n_items, d, batch, n_tasks, K), batch)
        self.workspace = torch.empty(self.nbytes, dtype=torch.uint8, device="cuda")
        self.ids = torch.empty((batch, K), dtype=torch.int64, device="cuda")
        self.scores = torch.empty((batch, K), dtype=torch.float32, device="cuda")
        self.count = torch.empty(batch, dtype=torch.int32, device="cuda")

    def overflow_flags(self):
        """int32 [batch] view: 1 where the last search on these buffers had to recompute the query
        by the slow exact path (read after the stream has synchronised)."""
        off, batch = self._ovf
        return self.workspace[off:off + 4 * batch].view(torch.int32)


def st_search(bloom: BloomIndex, items, item_scale, queries, query_scale, filt_ids, filt_offsets,
              K: int, buffers: SearchBuffers | None = None, stream=None):
    _need(items, torch.int8, "items")
    _need(item_scale, torch.float32, "item_scale")
    _need(queries, torch.int8, "queries")
    _need(query_scale, torch.float32, "query_scale")
    n, d = items.shape
    B = queries.shape[0]
    if queries.dim() != 2 or queries.shape[1] != d or query_scale.numel() != B or item_scale.numel() != n:
        raise ValueError("shape mismatch")
    ids, off = _filters(filt_ids, filt_offsets, B)
    buf = buffers or SearchBuffers(n, d, B, 1, K)
    _check(lib().st_search(C.c_void_p(bloom.handle), _dptr(items), _dptr(item_scale), n, d, _dptr(queries),
                           _dptr(query_scale), B, _hptr(ids), _hptr(off), K, _dptr(buf.ids),
                           _dptr(buf.scores), _dptr(buf.count), _dptr(buf.workspace), buf.nbytes,
                           _stream(stream)))
    return buf.ids, buf.scores, buf.count


ST_STATIC_SCRATCH_BYTES = 80 << 20


def st_search_static(bloom: BloomIndex, items, item_scale, queries, query_scale, filt_ids, filt_offsets,
                     K: int, out=None, stream=None):
    """st_search on the library's own fixed workspace (no allocation inside the call).  out: the
    (ids, scores, count) tensors to fill; allocated here, outside the library, if not given."""
    _need(items, torch.int8, "items")
    _need(item_scale, torch.float32, "item_scale")
    _need(queries, torch.int8, "queries")
    _need(query_scale, torch.float32, "query_scale")
    n, d = items.shape
    B = queries.shape[0]
    if queries.dim() != 2 or queries.shape[1] != d or query_scale.numel() != B or item_scale.numel() != n:
        raise ValueError("shape mismatch")
    ids, off = _filters(filt_ids, filt_offsets, B)
    if out is None:
        out = (torch.empty((B, K), dtype=torch.int64, device="cuda"),
               torch.empty((B, K), dtype=torch.float32, device="cuda"),
               torch.empty(B, dtype=torch.int32, device="cuda"))
    _check(lib().st_search_static(C.c_void_p(bloom.handle), _dptr(items), _dptr(item_scale), n, d, _dptr(queries),
                                  _dptr(query_scale), B, _hptr(ids), _hptr(off), K, _dptr(out[0]), _dptr(out[1]),
                                  _dptr(out[2]), _stream(stream)))
    return out


def st_search_multitask(bloom: BloomIndex, items, item_scale, queries, query_scale, task_weight,
                        filt_ids, filt_offsets, K: int, buffers: SearchBuffers | None = None,
                        stream=None):
    _need(items, torch.int8, "items")
    _need(item_scale, torch.float32, "item_scale")
    _need(queries, torch.int8, "queries")
    _need(query_scale, torch.float32, "query_scale")
    n, d = items.shape
    if queries.dim() != 3 or queries.shape[2] != d:
        raise ValueError("queries must be [B, T, d]")
    B, T = queries.shape[0], queries.shape[1]
    w = np.ascontiguousarray(np.asarray(task_weight, dtype=np.float32))
    if w.size != T or query_scale.numel() != B * T or item_scale.numel() != n:
        raise ValueError("shape mismatch")
    ids, off = _filters(filt_ids, filt_offsets, B)
    buf = buffers or SearchBuffers(n, d, B, T, K)
    _check(lib().st_search_multitask(C.c_void_p(bloom.handle), _dptr(items), _dptr(item_scale), n, d,
                                     _dptr(queries), _dptr(query_scale), B, T, _hptr(w), _hptr(ids),
                                     _hptr(off), K, _dptr(buf.ids), _dptr(buf.scores), _dptr(buf.count),
                                     _dptr(buf.workspace), buf.nbytes, _stream(stream)))
    return buf.ids, buf.scores, buf.count


def _programs(expr_ops, expr_ids, expr_offsets, n: int):
    ops = np.ascontiguousarray(np.asarray(expr_ops, dtype=np.int32))
    ids = np.asarray(expr_ids)
    if ids.dtype != np.dtype(np.uint64):
        ids = ids.astype(np.uint64)
    ids = np.ascontiguousarray(ids)
    off = np.ascontiguousarray(np.asarray(expr_offsets, dtype=np.int64))
    if off.size != n + 1 or ops.size != ids.size or (off.size and ops.size < off[-1]):
        raise ValueError("filter program arrays do not match their offsets")
    return ops, ids, off


def st_bloom_mask_expr(bloom: BloomIndex, expr_ops, expr_ids, expr_offsets, stream=None) -> torch.Tensor:
    n_e = len(expr_offsets) - 1
    ops, ids, off = _programs(expr_ops, expr_ids, expr_offsets, n_e)
    out = torch.zeros((n_e, (bloom.n_items + 63) // 64), dtype=torch.int64, device="cuda")
    _check(lib().st_bloom_mask_expr(C.c_void_p(bloom.handle), _hptr(ops), _hptr(ids), _hptr(off), n_e,
                                    _dptr(out), _stream(stream)))
    return out


def st_search_expr_workspace_bytes(n_items: int, d: int, batch: int, n_tasks: int, K: int,
                                   n_expr_entries: int) -> int:
    return _check(lib().st_search_expr_workspace_bytes(n_items, d, batch, n_tasks, K, n_expr_entries))


def st_search_expr(bloom: BloomIndex, items, item_scale, queries, query_scale, expr_ops, expr_ids,
                   expr_offsets, K: int, task_weight=None, buffers: SearchBuffers | None = None, stream=None):
    """queries [B, d] (task_weight None) or [B, T, d] with T weights; query b's filter is program b."""
    _need(items, torch.int8, "items")
    _need(item_scale, torch.float32, "item_scale")
    _need(queries, torch.int8, "queries")
    _need(query_scale, torch.float32, "query_scale")
    n, d = items.shape
    B = queries.shape[0]
    if task_weight is None:
        if queries.dim() != 2 or queries.shape[1] != d:
            raise ValueError("queries must be [B, d]")
        T, w = 1, None
    else:
        if queries.dim() != 3 or queries.shape[2] != d:
            raise ValueError("queries must be [B, T, d]")
        T = queries.shape[1]
        w = np.ascontiguousarray(np.asarray(task_weight, dtype=np.float32))
        if w.size != T:
            raise ValueError("shape mismatch")
    if query_scale.numel() != B * T or item_scale.numel() != n:
        raise ValueError("shape mismatch")
    ops, ids, off = _programs(expr_ops, expr_ids, expr_offsets, B)
    buf = buffers or SearchBuffers(n, d, B, T, K, n_expr_entries=int(off[-1]))
    _check(lib().st_search_expr(C.c_void_p(bloom.handle), _dptr(items), _dptr(item_scale), n, d, _dptr(queries),
                                _dptr(query_scale), B, T, None if w is None else _hptr(w), _hptr(ops),
                                _hptr(ids), _hptr(off), K, _dptr(buf.ids), _dptr(buf.scores), _dptr(buf.count),
                                _dptr(buf.workspace), buf.nbytes, _stream(stream)))
    return buf.ids, buf.scores, buf.count


def st_search_ivf_workspace_bytes(n_items: int, d: int, batch: int, K: int, n_clusters: int, n_probe: int,
                                  n_expr_entries: int) -> int:
    return _check(lib().st_search_ivf_workspace_bytes(n_items, d, batch, K, n_clusters, n_probe, n_expr_entries))


class IvfBuffers(SearchBuffers):
    """Workspace and outputs of st_search_ivf for one shape."""

    def __init__(self, n_items: int, d: int, batch: int, K: int, n_clusters: int, n_probe: int, n_expr_entries: int):
        super().__init__(n_items, d, batch, 1, K)
        self.nbytes = st_search_ivf_workspace_bytes(n_items, d, batch, K, n_clusters, n_probe, n_expr_entries)
        self.workspace = torch.empty(self.nbytes, dtype=torch.uint8, device="cuda")
        self.probes = torch.empty((batch, n_probe), dtype=torch.int32, device="cuda")


def st_search_ivf(bloom: BloomIndex, items, item_scale, centroids, centroid_scale, cluster_offsets, n_probe: int,
                  queries, query_scale, expr_ops, expr_ids, expr_offsets, K: int,
                  buffers: IvfBuffers | None = None, stream=None):
    """Returns (ids, scores, count, probes); cluster_offsets int64 [n_clusters + 1] on the device."""
    _need(items, torch.int8, "items")
    _need(item_scale, torch.float32, "item_scale")
    _need(centroids, torch.int8, "centroids")
    _need(centroid_scale, torch.float32, "centroid_scale")
    _need(cluster_offsets, torch.int64, "cluster_offsets")
    _need(queries, torch.int8, "queries")
    _need(query_scale, torch.float32, "query_scale")
    n, d = items.shape
    n_c = centroids.shape[0]
    B = queries.shape[0]
    if (queries.dim() != 2 or queries.shape[1] != d or centroids.shape[1] != d or query_scale.numel() != B
            or item_scale.numel() != n or centroid_scale.numel() != n_c or cluster_offsets.numel() != n_c + 1):
        raise ValueError("shape mismatch")
    ops, ids, off = _programs(expr_ops, expr_ids, expr_offsets, B)
    buf = buffers or IvfBuffers(n, d, B, K, n_c, n_probe, int(off[-1]))
    _check(lib().st_search_ivf(C.c_void_p(bloom.handle), _dptr(items), _dptr(item_scale), n, d, _dptr(centroids),
                               _dptr(centroid_scale), _dptr(cluster_offsets), n_c, n_probe, _dptr(queries),
                               _dptr(query_scale), B, _hptr(ops), _hptr(ids), _hptr(off), K, _dptr(buf.ids),
                               _dptr(buf.scores), _dptr(buf.count), _dptr(buf.probes), _dptr(buf.workspace),
                               buf.nbytes, _stream(stream)))
    return buf.ids, buf.scores, buf.count, buf.probes


def st_stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int, stream=None) -> None:
    """Bandwidth probe: reads all of src (any dtype, contiguous) once; sink int32/uint32 [workgroups]."""
    if not (src.is_cuda and src.is_contiguous() and sink.is_cuda and sink.numel() >= workgroups):
        raise TypeError("src must be a contiguous CUDA tensor and sink hold one word per workgroup")
    _check(lib().st_stream_read(_dptr(src), src.numel() * src.element_size(), _dptr(sink), workgroups, _stream(stream)))


def st_quantize_global(x, stream=None):
    """fp32 [N, d] CUDA tensor -> (int8 [N, d], row scales fp32 [N], minmax fp32 [2]) on the device."""
    _need(x, torch.float32, "x")
    if x.dim() != 2:
        raise ValueError("x must be [N, d]")
    n, d = x.shape
    q = torch.empty((n, d), dtype=torch.int8, device="cuda")
    rs = torch.empty(n, dtype=torch.float32, device="cuda")
    mm = torch.empty(2, dtype=torch.float32, device="cuda")
    scratch = torch.empty(2, dtype=torch.int32, device="cuda")
    _check(lib().st_quantize_global(_dptr(x), n, d, _dptr(q), _dptr(rs), _dptr(mm), _dptr(scratch), _stream(stream)))
    return q, rs, mm


def st_value_model(task_scores, ops, consts, out=None, stream=None):
    """task_scores fp32 [n, T] CUDA tensor; postfix formula (ops int32, consts fp32) -> fp32 [n]."""
    _need(task_scores, torch.float32, "task_scores")
    if task_scores.dim() != 2:
        raise ValueError("task_scores must be [n, T]")
    n, T = task_scores.shape
    o = np.ascontiguousarray(np.asarray(ops, dtype=np.int32))
    c = np.ascontiguousarray(np.asarray(consts, dtype=np.float32))
    if o.size != c.size:
        raise ValueError("ops and consts differ in length")
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device="cuda")
    _check(lib().st_value_model(_dptr(task_scores), n, T, _hptr(o), _hptr(c), o.size, _dptr(out), _stream(stream)))
    return out


def st_score_pairs(items, item_scale, queries, query_scale, pair_item, pair_query, stream=None):
    _need(items, torch.int8, "items")
    _need(queries, torch.int8, "queries")
    _need(pair_item, torch.int64, "pair_item")
    _need(pair_query, torch.int32, "pair_query")
    d = items.shape[1]
    q2 = queries.reshape(-1, d)
    n = pair_item.numel()
    dots = torch.empty(n, dtype=torch.int32, device="cuda")
    scores = torch.empty(n, dtype=torch.float32, device="cuda")
    _check(lib().st_score_pairs(_dptr(items), _dptr(item_scale), d, _dptr(q2), _dptr(query_scale.reshape(-1)),
                                _dptr(pair_item), _dptr(pair_query), n, _dptr(dots), _dptr(scores),
                                _stream(stream)))
    return dots, scores
