"""ctypes front end of the CPU oracle (``st_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module; the GPU library never does, and nothing in
here imports the GPU package.  All arrays are numpy, host memory.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "st_oracle.c")
_LIB = os.path.join(_HERE, "libst_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No contraction, no fast-math: the fp32
    rounding order is part of the definition."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.check_call(cmd)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        p = C.c_void_p
        L.sto_splitmix64.restype = C.c_uint64
        L.sto_splitmix64.argtypes = [C.c_uint64]
        L.sto_bit_index.restype = C.c_int64
        L.sto_bit_index.argtypes = [C.c_uint64, C.c_int32, C.c_int32]
        L.sto_signature.restype = None
        L.sto_signature.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p]
        L.sto_bloom_build.restype = None
        L.sto_bloom_build.argtypes = [p, p, C.c_int64, C.c_int32, C.c_int32, p]
        L.sto_bloom_mask.restype = None
        L.sto_bloom_mask.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p, C.c_int64, p]
        L.sto_exact_mask.restype = None
        L.sto_exact_mask.argtypes = [p, p, C.c_int64, p, C.c_int64, p]
        L.sto_dot.restype = C.c_int32
        L.sto_dot.argtypes = [p, p, C.c_int32]
        L.sto_rescale.restype = C.c_float
        L.sto_rescale.argtypes = [C.c_int32, C.c_float, C.c_float]
        L.sto_search.restype = C.c_int
        L.sto_search.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p, p, C.c_int32, p, p,
                                 C.c_int32, C.c_int32, p, p, p, C.c_int32, p, p, p]
        L.sto_expr_depth.restype = C.c_int32
        L.sto_expr_depth.argtypes = [p, C.c_int64]
        L.sto_expr_mask.restype = C.c_int
        L.sto_expr_mask.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p, p, C.c_int64, p]
        L.sto_search_expr.restype = C.c_int
        L.sto_search_expr.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p, p, C.c_int32, p, p,
                                      C.c_int32, C.c_int32, p, p, p, p, C.c_int32, p, p, p]
        L.sto_search_ivf.restype = C.c_int
        L.sto_search_ivf.argtypes = [p, C.c_int64, C.c_int32, C.c_int32, p, p, C.c_int32, p, p, p, C.c_int32,
                                     C.c_int32, p, p, C.c_int32, p, p, p, C.c_int32, p, p, p, p]
        L.sto_quantize_global.restype = None
        L.sto_quantize_global.argtypes = [p, C.c_int64, C.c_int32, p, p, p]
        L.sto_vm_depth.restype = C.c_int32
        L.sto_vm_depth.argtypes = [p, C.c_int32, C.c_int32]
        L.sto_value_model.restype = C.c_int
        L.sto_value_model.argtypes = [p, C.c_int64, C.c_int32, p, p, C.c_int32, p]
        L.sto_num_threads.restype = C.c_int32
        L.sto_num_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=dtype))


def splitmix64(x: int) -> int:
    return int(lib().sto_splitmix64(C.c_uint64(x & 0xFFFFFFFFFFFFFFFF)))


def bit_index(f: int, j: int, m: int) -> int:
    return int(lib().sto_bit_index(C.c_uint64(f & 0xFFFFFFFFFFFFFFFF), j, m))


def sig_words(m: int) -> int:
    return (m + 63) // 64


def signature(ids, m: int, k: int) -> np.ndarray:
    ids = _arr(ids, np.uint64)
    out = np.zeros(sig_words(m), dtype=np.uint64)
    lib().sto_signature(_ptr(ids), ids.size, m, k, _ptr(out))
    return out


def bloom_build(feat_offsets, feat_ids, m: int, k: int) -> np.ndarray:
    """Item-major signatures, shape [n_items, ceil(m/64)] uint64."""
    off = _arr(feat_offsets, np.int64)
    ids = _arr(feat_ids, np.uint64)
    n = off.size - 1
    sigs = np.zeros((n, sig_words(m)), dtype=np.uint64)
    lib().sto_bloom_build(_ptr(off), _ptr(ids), n, m, k, _ptr(sigs))
    return sigs


def bloom_mask(sigs: np.ndarray, m: int, k: int, filt_ids) -> np.ndarray:
    """1 bit per item, ceil(N/64) uint64 words, LSB first."""
    n = sigs.shape[0]
    f = _arr(filt_ids, np.uint64)
    mask = np.zeros((n + 63) // 64, dtype=np.uint64)
    lib().sto_bloom_mask(_ptr(sigs), n, m, k, _ptr(f), f.size, _ptr(mask))
    return mask


def exact_mask(feat_offsets, feat_ids, filt_ids) -> np.ndarray:
    off = _arr(feat_offsets, np.int64)
    ids = _arr(feat_ids, np.uint64)
    f = _arr(filt_ids, np.uint64)
    n = off.size - 1
    mask = np.zeros((n + 63) // 64, dtype=np.uint64)
    lib().sto_exact_mask(_ptr(off), _ptr(ids), n, _ptr(f), f.size, _ptr(mask))
    return mask


def mask_to_bool(mask: np.ndarray, n: int) -> np.ndarray:
    bits = np.unpackbits(mask.view(np.uint8), bitorder="little")
    return bits[:n].astype(bool)


def dot(q, e) -> int:
    q = _arr(q, np.int8)
    e = _arr(e, np.int8)
    return int(lib().sto_dot(_ptr(q), _ptr(e), q.size))


def rescale(d: int, s_q: float, s_i: float) -> np.float32:
    return np.float32(lib().sto_rescale(int(d), C.c_float(s_q), C.c_float(s_i)))


def search(sigs, m, k, items, item_scale, queries, query_scale, filt_ids, filt_offsets, K,
           task_weight=None):
    """Filtered top-K.  queries [B,d] (task_weight None) or [B,T,d].
    Returns (ids int64 [B,K], scores float32 [B,K], count int32 [B])."""
    items = _arr(items, np.int8)
    item_scale = _arr(item_scale, np.float32)
    queries = _arr(queries, np.int8)
    query_scale = _arr(query_scale, np.float32)
    fid = _arr(filt_ids, np.uint64)
    foff = _arr(filt_offsets, np.int64)
    n, d = items.shape
    if task_weight is None:
        assert queries.ndim == 2 and queries.shape[1] == d
        B, T, w = queries.shape[0], 1, None
    else:
        assert queries.ndim == 3 and queries.shape[2] == d
        B, T = queries.shape[0], queries.shape[1]
        w = _arr(task_weight, np.float32)
        assert w.size == T
    assert query_scale.size == B * T and foff.size == B + 1 and sigs.shape[0] == n
    ids = np.empty((B, K), dtype=np.int64)
    scores = np.empty((B, K), dtype=np.float32)
    count = np.empty(B, dtype=np.int32)
    sigs = _arr(sigs, np.uint64)
    rc = lib().sto_search(_ptr(sigs), n, m, k, _ptr(items), _ptr(item_scale), d, _ptr(queries),
                          _ptr(query_scale), B, T, _ptr(w), _ptr(fid), _ptr(foff), K,
                          _ptr(ids), _ptr(scores), _ptr(count))
    if rc != 0:
        raise MemoryError("oracle ran out of memory")
    return ids, scores, count


LEAF, AND, OR, NOT = 0, 1, 2, 3  # operation codes of a filter program (postfix order)


def expr_depth(ops) -> int:
    """Deepest stack a program reaches, -1 if it is ill-formed."""
    ops = _arr(ops, np.int32)
    return int(lib().sto_expr_depth(_ptr(ops), ops.size))


def expr_mask(sigs: np.ndarray, m: int, k: int, ops, ids) -> np.ndarray:
    """1 bit per item for one filter program (ops, ids in postfix order)."""
    n = sigs.shape[0]
    ops = _arr(ops, np.int32)
    ids = _arr(ids, np.uint64)
    assert ops.size == ids.size
    mask = np.zeros((n + 63) // 64, dtype=np.uint64)
    sigs = _arr(sigs, np.uint64)
    if lib().sto_expr_mask(_ptr(sigs), n, m, k, _ptr(ops), _ptr(ids), ops.size, _ptr(mask)) != 0:
        raise ValueError("ill-formed filter program")
    return mask


def search_expr(sigs, m, k, items, item_scale, queries, query_scale, expr_ops, expr_ids, expr_offsets, K,
                task_weight=None):
    """Filtered top-K with one filter program per query; otherwise as ``search``."""
    items = _arr(items, np.int8)
    item_scale = _arr(item_scale, np.float32)
    queries = _arr(queries, np.int8)
    query_scale = _arr(query_scale, np.float32)
    eops = _arr(expr_ops, np.int32)
    eids = _arr(expr_ids, np.uint64)
    eoff = _arr(expr_offsets, np.int64)
    n, d = items.shape
    if task_weight is None:
        assert queries.ndim == 2 and queries.shape[1] == d
        B, T, w = queries.shape[0], 1, None
    else:
        assert queries.ndim == 3 and queries.shape[2] == d
        B, T = queries.shape[0], queries.shape[1]
        w = _arr(task_weight, np.float32)
        assert w.size == T
    assert query_scale.size == B * T and eoff.size == B + 1 and sigs.shape[0] == n
    assert eops.size == eids.size == eoff[-1]
    ids = np.empty((B, K), dtype=np.int64)
    scores = np.empty((B, K), dtype=np.float32)
    count = np.empty(B, dtype=np.int32)
    sigs = _arr(sigs, np.uint64)
    rc = lib().sto_search_expr(_ptr(sigs), n, m, k, _ptr(items), _ptr(item_scale), d, _ptr(queries),
                               _ptr(query_scale), B, T, _ptr(w), _ptr(eops), _ptr(eids), _ptr(eoff), K,
                               _ptr(ids), _ptr(scores), _ptr(count))
    if rc == -2:
        raise ValueError("ill-formed filter program")
    if rc != 0:
        raise MemoryError("oracle ran out of memory")
    return ids, scores, count


def search_ivf(sigs, m, k, items, item_scale, centroids, centroid_scale, cluster_offsets, n_probe,
               queries, query_scale, expr_ops, expr_ids, expr_offsets, K):
    """Probe the n_probe best clusters per query, filter and score inside them, top-K.
    Returns (ids [B,K], scores [B,K], count [B], probes int32 [B,n_probe])."""
    items = _arr(items, np.int8)
    item_scale = _arr(item_scale, np.float32)
    cent = _arr(centroids, np.int8)
    cs = _arr(centroid_scale, np.float32)
    coff = _arr(cluster_offsets, np.int64)
    queries = _arr(queries, np.int8)
    query_scale = _arr(query_scale, np.float32)
    eops = _arr(expr_ops, np.int32)
    eids = _arr(expr_ids, np.uint64)
    eoff = _arr(expr_offsets, np.int64)
    n, d = items.shape
    n_c = cent.shape[0]
    B = queries.shape[0]
    assert queries.ndim == 2 and queries.shape[1] == d and cent.shape[1] == d
    assert cs.size == n_c and coff.size == n_c + 1 and coff[0] == 0 and coff[-1] == n
    assert query_scale.size == B and eoff.size == B + 1 and eops.size == eids.size == eoff[-1]
    ids = np.empty((B, K), dtype=np.int64)
    scores = np.empty((B, K), dtype=np.float32)
    count = np.empty(B, dtype=np.int32)
    probes = np.empty((B, n_probe), dtype=np.int32)
    sigs = _arr(sigs, np.uint64)
    rc = lib().sto_search_ivf(_ptr(sigs), n, m, k, _ptr(items), _ptr(item_scale), d, _ptr(cent), _ptr(cs),
                              _ptr(coff), n_c, n_probe, _ptr(queries), _ptr(query_scale), B, _ptr(eops),
                              _ptr(eids), _ptr(eoff), K, _ptr(ids), _ptr(scores), _ptr(count), _ptr(probes))
    if rc == -2:
        raise ValueError("ill-formed filter program")
    if rc != 0:
        raise MemoryError("oracle ran out of memory")
    return ids, scores, count, probes


def quantize_global(x):
    """fp32 [N, d] -> (int8 [N, d], row scales fp32 [N], (min, max))."""
    x = _arr(x, np.float32)
    assert x.ndim == 2
    q = np.empty(x.shape, dtype=np.int8)
    rs = np.empty(x.shape[0], dtype=np.float32)
    mm = np.empty(2, dtype=np.float32)
    lib().sto_quantize_global(_ptr(x), x.shape[0], x.shape[1], _ptr(q), _ptr(rs), _ptr(mm))
    return q, rs, (float(mm[0]), float(mm[1]))


VM_TASK, VM_CONST, VM_ADD, VM_SUB, VM_MUL, VM_MIN, VM_MAX, VM_GT, VM_SELECT = range(9)


def vm_task(t: int) -> int:
    """Program entry that pushes the score of task t."""
    return VM_TASK | (t << 8)


def vm_depth(ops, n_tasks: int) -> int:
    ops = _arr(ops, np.int32)
    return int(lib().sto_vm_depth(_ptr(ops), ops.size, n_tasks))


def value_model(scores, ops, consts) -> np.ndarray:
    """scores fp32 [n, T]; postfix program (ops int32, consts fp32, same length) -> fp32 [n]."""
    scores = _arr(scores, np.float32)
    ops = _arr(ops, np.int32)
    consts = _arr(consts, np.float32)
    assert scores.ndim == 2 and ops.size == consts.size
    out = np.empty(scores.shape[0], dtype=np.float32)
    if lib().sto_value_model(_ptr(scores), scores.shape[0], scores.shape[1], _ptr(ops), _ptr(consts), ops.size,
                             _ptr(out)) != 0:
        raise ValueError("ill-formed value model program")
    return out


def num_threads() -> int:
    return int(lib().sto_num_threads())
