"""CPU oracle for batched top-k maximum-inner-product retrieval (ctypes front of
``ann_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``; never by the product package, and
it imports nothing from it.  All arrays are host numpy arrays; fp16 / bf16
inputs are passed as their raw 16-bit patterns (``uint16`` or ``float16``), so
the oracle sees exactly the bits the GPU reads.

Paper passages: exact vs approximate retrieval, Section 2.1 "Retrieval
Mechanism"; candidate list with best and worst element and the natural stop,
Section 3.3; search range = candidate-list size, up to 32 neighbours per node,
Appendix B.3.  Recall of an approximate result is measured against exact
retrieval (Appendix B.2 quotes such recall values without a formula; the usual
definition is used: mean over queries of |approx ids ∩ exact ids| / k).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ann_oracle.c")
# ANN_ORACLE_LIBRARY_PATH: use a build of ann_oracle.c made elsewhere (e.g. with sanitizers) instead
_LIB = os.environ.get("ANN_ORACLE_LIBRARY_PATH", os.path.join(_HERE, "libann_oracle.so"))

F16, BF16, F32 = 0, 1, 2
_lib = None


def build(force: bool = False) -> str:
    """Compile ann_oracle.c with gcc into oracle/libann_oracle.so."""
    if "ANN_ORACLE_LIBRARY_PATH" in os.environ:
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.oracle_threads.restype = c.c_int
        lib.oracle_threads.argtypes = [c.c_int]
        lib.oracle_score.restype = c.c_double
        lib.oracle_score.argtypes = [c.c_void_p, c.c_int32, c.c_int, c.c_int64, c.c_void_p, c.c_int32]
        lib.oracle_flat_search.restype = c.c_int
        lib.oracle_flat_search.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int, c.c_void_p,
                                           c.c_int32, c.c_int32, c.c_void_p, c.c_void_p,
                                           c.c_void_p, c.c_void_p, c.c_void_p, c.c_int]
        lib.oracle_graph_search.restype = c.c_int
        lib.oracle_graph_search.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int, c.c_void_p, c.c_int32,
                                            c.c_int32, c.c_void_p, c.c_int32, c.c_void_p, c.c_int32, c.c_int32, c.c_int32,
                                            c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int]
        lib.oracle_graph_search_nonstall.restype = c.c_int
        lib.oracle_graph_search_nonstall.argtypes = [c.c_void_p, c.c_int64, c.c_int32, c.c_int, c.c_void_p, c.c_int32,
                                                     c.c_int32, c.c_void_p, c.c_int32, c.c_void_p, c.c_int32, c.c_int32, c.c_int32,
                                                     c.c_float, c.c_int32, c.c_int, c.c_int64, c.c_int64,
                                                     c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int]
        lib.oracle_priority_order.restype = c.c_int
        lib.oracle_priority_order.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int32, c.c_int32,
                                              c.c_void_p, c.c_void_p]
        _lib = lib
    return _lib


def _code(a: np.ndarray, dtype: Optional[str]) -> int:
    if dtype is not None:
        return {"f16": F16, "bf16": BF16, "f32": F32}[dtype]
    if a.dtype == np.float16:
        return F16
    if a.dtype == np.float32:
        return F32
    raise ValueError("pass dtype='bf16' (or 'f16') for raw uint16 storage")


def _prep(corpus, queries, dtype):
    corpus = np.ascontiguousarray(corpus)
    queries = np.ascontiguousarray(queries)
    if corpus.ndim != 2 or queries.ndim != 2 or corpus.shape[1] != queries.shape[1]:
        raise ValueError("corpus [N,d] and queries [B,d] expected")
    if corpus.dtype.itemsize != queries.dtype.itemsize:
        raise ValueError("corpus and queries must share the storage type")
    return corpus, queries, _code(corpus, dtype)


def threads(n: int = 0) -> int:
    return _load().oracle_threads(n)


def score(corpus, queries, b: int, row: int, dtype: Optional[str] = None) -> float:
    corpus, queries, code = _prep(corpus, queries, dtype)
    return _load().oracle_score(corpus.ctypes.data, corpus.shape[1], code, row, queries.ctypes.data, b)


def flat_search(corpus, queries, k: int, *, after=None, dtype: Optional[str] = None,
                n_threads: int = 0) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Exact top-k.  Returns (ids int32 [B,k], scores fp32 [B,k], scores fp64 [B,k]).
    after = (scores fp64 [B], ids int32 [B]): only rows that come strictly after that pair in the order
    (score descending, id ascending) are candidates: the continuation of an earlier answer (pass the
    binary64 scores this function returned)."""
    corpus, queries, code = _prep(corpus, queries, dtype)
    N, d = corpus.shape
    B = queries.shape[0]
    ids = np.empty((B, k), np.int32)
    sc = np.empty((B, k), np.float32)
    sc64 = np.empty((B, k), np.float64)
    a_s = a_i = None
    if after is not None:
        a_s = np.ascontiguousarray(after[0], dtype=np.float64)
        a_i = np.ascontiguousarray(after[1], dtype=np.int32)
        if a_s.shape != (B,) or a_i.shape != (B,):
            raise ValueError("after = (scores [B], ids [B]) expected")
    rc = _load().oracle_flat_search(corpus.ctypes.data, N, d, code, queries.ctypes.data, B, k,
                                    a_s.ctypes.data if a_s is not None else None,
                                    a_i.ctypes.data if a_i is not None else None,
                                    ids.ctypes.data, sc.ctypes.data, sc64.ctypes.data, n_threads)
    if rc != 0:
        raise ValueError("oracle_flat_search: bad arguments")
    return ids, sc, sc64


def _entries(entries, B: int):
    """None, or the per-query entry nodes as a contiguous int32 [B, E] array."""
    if entries is None:
        return None, 0, 0
    e = np.ascontiguousarray(entries, dtype=np.int32)
    if e.ndim == 1:
        e = e.reshape(B, 1)
    if e.ndim != 2 or e.shape[0] != B or e.shape[1] < 1:
        raise ValueError("entries [B] or [B, E] expected")
    return e, e.ctypes.data, e.shape[1]


RQ_FORMS = {"node": 0, "expansion": 1}


def graph_search(corpus, graph, entry: int, queries, k: int, ef: int, *, entries=None,
                 dtype: Optional[str] = None, n_threads: int = 0):
    """Best-first graph search from the node `entry`, or, with `entries` ([B] or [B, E]), from
    each query's own entry nodes.  Returns (ids, scores fp32, scores fp64, n_dist, n_expand)."""
    corpus, queries, code = _prep(corpus, queries, dtype)
    graph = np.ascontiguousarray(graph, dtype=np.int32)
    N, d = corpus.shape
    if graph.ndim != 2 or graph.shape[0] != N:
        raise ValueError("graph [N,R] expected")
    B = queries.shape[0]
    ids = np.empty((B, k), np.int32)
    sc = np.empty((B, k), np.float32)
    sc64 = np.empty((B, k), np.float64)
    nd = np.empty(B, np.int64)
    ne = np.empty(B, np.int64)
    keep, e_ptr, E = _entries(entries, B)
    rc = _load().oracle_graph_search(corpus.ctypes.data, N, d, code, graph.ctypes.data, graph.shape[1],
                                     entry, e_ptr, E, queries.ctypes.data, B, k, ef, ids.ctypes.data,
                                     sc.ctypes.data, sc64.ctypes.data, nd.ctypes.data, ne.ctypes.data,
                                     n_threads)
    if rc != 0:
        raise ValueError("oracle_graph_search: bad arguments")
    return ids, sc, sc64, nd, ne


def graph_search_nonstall(corpus, graph, entry: int, queries, k: int, ef: int, *, tau: float = 0.9,
                          window: int = 500, form: str = "expansion", ready_from: int = 0, max_expand: int = 0,
                          entries=None, dtype: Optional[str] = None, n_threads: int = 0):
    """Best-first graph search with the maturity (non-stall) exit of Section 3.3.
    form "node": best / worst of the candidate list as it stands when each node is scored (binary64);
    form "expansion": as it stands when the expansion starts, binary32 decision (the form a search that
    scores a node's neighbours together computes; the GPU library is compared with this one).
    Returns (ids, scores fp32, scores fp64, stats int32 [B,3] = (early, n_dist, n_expand), ema fp32 [B])."""
    corpus, queries, code = _prep(corpus, queries, dtype)
    graph = np.ascontiguousarray(graph, dtype=np.int32)
    N, d = corpus.shape
    if graph.ndim != 2 or graph.shape[0] != N:
        raise ValueError("graph [N,R] expected")
    B = queries.shape[0]
    ids = np.empty((B, k), np.int32)
    sc = np.empty((B, k), np.float32)
    sc64 = np.empty((B, k), np.float64)
    stats = np.empty((B, 3), np.int32)
    ema = np.empty(B, np.float32)
    keep, e_ptr, E = _entries(entries, B)
    rc = _load().oracle_graph_search_nonstall(corpus.ctypes.data, N, d, code, graph.ctypes.data, graph.shape[1], entry,
                                              e_ptr, E, queries.ctypes.data, B, k, ef, tau, window, RQ_FORMS[form],
                                              ready_from, max_expand,
                                              ids.ctypes.data, sc.ctypes.data, sc64.ctypes.data, stats.ctypes.data,
                                              ema.ctypes.data, n_threads)
    if rc != 0:
        raise ValueError("oracle_graph_search_nonstall: bad arguments")
    return ids, sc, sc64, stats, ema


def priority_order(R, W, C, Wcur, G: int):
    """Scheduler priority levels (Section 3.2, Eq. 1-2) and execution order.
    R, C int32 [n]; W, Wcur float64 [n].  Returns (level int32 [n], order int32 [n])."""
    R = np.ascontiguousarray(R, dtype=np.int32)
    C = np.ascontiguousarray(C, dtype=np.int32)
    W = np.ascontiguousarray(W, dtype=np.float64)
    Wcur = np.ascontiguousarray(Wcur, dtype=np.float64)
    n = R.shape[0]
    if not (W.shape == C.shape == Wcur.shape == (n,)):
        raise ValueError("R, W, C, Wcur must have the same length")
    level = np.empty(n, np.int32)
    order = np.empty(n, np.int32)
    rc = _load().oracle_priority_order(R.ctypes.data, W.ctypes.data, C.ctypes.data, Wcur.ctypes.data, n, G,
                                       level.ctypes.data, order.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_priority_order: bad arguments")
    return level, order


def recall_at_k(approx_ids: np.ndarray, exact_ids: np.ndarray) -> float:
    """Mean over queries of |approx ∩ exact| / k; padding ids (-1) never match."""
    B, k = exact_ids.shape
    hit = 0
    for b in range(B):
        hit += len(set(int(i) for i in approx_ids[b] if i >= 0) & set(int(i) for i in exact_ids[b]))
    return hit / (B * k)
