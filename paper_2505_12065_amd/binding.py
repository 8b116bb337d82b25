"""ctypes binding of libann.so: the same entry points as include/ann.h, taking
torch device tensors.  Argument marshalling only — shapes, pointers, the current
HIP stream; every step of the search runs in the library's kernels.  There is no
fallback: if the library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("ANN_LIBRARY_PATH", os.path.join(_HERE, "libann.so"))

ANN_OK, ANN_ERR_INVALID, ANN_ERR_ALIGNMENT, ANN_ERR_UNKNOWN_CORPUS, ANN_ERR_LAUNCH, ANN_ERR_NOMEM = 0, -1, -2, -3, -4, -5
ANN_F16, ANN_BF16, ANN_F32 = 0, 1, 2
ANN_K_MAX, ANN_EF_MAX, ANN_R_MAX, ANN_D_MAX = 16, 16384, 256, 4096
ANN_ENTRIES_MAX = 32

_DTYPES = {torch.float16: ANN_F16, torch.bfloat16: ANN_BF16, torch.float32: ANN_F32}

EXPORTS = ("ann_version", "ann_last_error", "ann_flat_search_typed", "ann_flat_search",
           "ann_graph_search_typed", "ann_graph_search", "ann_register_corpus", "ann_unregister_corpus",
           "ann_set_default_dtype", "ann_flat_workspace_bytes", "ann_release_workspace",
           "ann_graph_search_nonstall_typed", "ann_graph_nonstall_workspace_bytes",
           "ann_graph_search_entries_typed", "ann_gather_ids", "ann_timing_enable", "ann_timing_read",
           "ann_measure_mfma_rate", "ann_priority_order", "ann_flat_search_static",
           "ann_graph_search_multi_typed", "ann_timing_read_each",
           "ann_set_workspace", "ann_flat_search_after_typed")


class AnnError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libann error {code}: {message}")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2505_12065_amd.build` "
                "(or __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        vp, i32, i64 = c.c_void_p, c.c_int32, c.c_int64
        L.ann_version.restype = c.c_int
        L.ann_last_error.restype = c.c_char_p
        L.ann_flat_search_typed.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, vp, vp]
        L.ann_flat_search.argtypes = [vp, i64, i32, vp, i32, i32, vp, vp, vp]
        L.ann_flat_search_after_typed.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, vp, vp, vp, vp]
        L.ann_flat_search_static.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, vp, vp]
        L.ann_graph_search_typed.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, i32, i32, i32, vp, vp, vp]
        L.ann_graph_search.argtypes = [vp, vp, i32, i32, vp, i32, i32, i32, vp, vp, vp]
        L.ann_register_corpus.argtypes = [vp, i64, i32, i32]
        L.ann_unregister_corpus.argtypes = [vp]
        L.ann_set_default_dtype.argtypes = [i32]
        L.ann_flat_workspace_bytes.argtypes = [i64, i32, i32, i32, i32]
        L.ann_flat_workspace_bytes.restype = i64
        L.ann_graph_search_nonstall_typed.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, i32, i32, i32, vp, i32,
                                                      c.c_float, i32, vp, vp, vp, vp, vp, vp]
        L.ann_graph_search_multi_typed.argtypes = [vp, i64, i32, i32, vp, i32, vp, i32, vp, i32, i32, i32, vp, vp, vp]
        L.ann_graph_search_entries_typed.argtypes = [vp, i64, i32, i32, vp, i32, vp, vp, i32, i32, i32, vp, vp, vp]
        L.ann_gather_ids.argtypes = [vp, i64, vp, i64, vp, vp]
        L.ann_measure_mfma_rate.argtypes = [i32, i32, c.POINTER(c.c_double)]
        L.ann_priority_order.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp]
        L.ann_set_workspace.argtypes = [vp, i64]
        L.ann_timing_enable.argtypes = [i32]
        L.ann_timing_read.argtypes = [i32, c.POINTER(i32), c.POINTER(c.c_double)]
        L.ann_timing_read_each.argtypes = [i32, i32, c.POINTER(i32), c.POINTER(c.c_float)]
        L.ann_graph_nonstall_workspace_bytes.argtypes = [i64, i32]
        L.ann_graph_nonstall_workspace_bytes.restype = i64
        for name in EXPORTS:
            if name not in ("ann_last_error", "ann_flat_workspace_bytes", "ann_graph_nonstall_workspace_bytes"):
                getattr(L, name).restype = c.c_int
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != ANN_OK:
        raise AnnError(rc, lib().ann_last_error().decode())


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _outputs(B: int, k: int, device, ids, scores):
    if ids is None:
        ids = torch.empty(B, k, dtype=torch.int32, device=device)
    if scores is None:
        scores = torch.empty(B, k, dtype=torch.float32, device=device)
    if ids.shape != (B, k) or ids.dtype != torch.int32 or not ids.is_contiguous() or not ids.is_cuda:
        raise ValueError("ids must be a contiguous int32 [B, k] device tensor")
    if scores.shape != (B, k) or scores.dtype != torch.float32 or not scores.is_contiguous() or not scores.is_cuda:
        raise ValueError("scores must be a contiguous float32 [B, k] device tensor")
    return ids, scores


def _matrix(t: torch.Tensor, name: str) -> torch.Tensor:
    if t.dim() != 2 or not t.is_cuda or not t.is_contiguous() or t.dtype not in _DTYPES:
        raise ValueError(f"{name} must be a contiguous 2-D fp16/bf16/fp32 device tensor")
    return t


def ann_version() -> int:
    return lib().ann_version()


def ann_last_error() -> str:
    return lib().ann_last_error().decode()


def ann_flat_search_typed(corpus: torch.Tensor, queries: torch.Tensor, k: int, *, after=None, ids=None, scores=None,
                          stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Exact top-k of every query over the corpus; element type taken from the tensors.
    after = (scores float32 [B], ids int32 [B]) device tensors: the continuation entry point, the k best rows
    that come strictly after that pair in the order."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    with torch.cuda.device(corpus.device):
        if after is None:
            _check(lib().ann_flat_search_typed(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], queries.data_ptr(), B, k,
                                               ids.data_ptr(), scores.data_ptr(), _stream(stream)))
        else:
            a_s, a_i = after
            if a_s.dtype != torch.float32 or a_i.dtype != torch.int32 or tuple(a_s.shape) != (B,) or tuple(a_i.shape) != (B,) \
                    or not (a_s.is_cuda and a_i.is_cuda and a_s.is_contiguous() and a_i.is_contiguous()):
                raise ValueError("after must be (float32 [B], int32 [B]) contiguous device tensors")
            _check(lib().ann_flat_search_after_typed(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], queries.data_ptr(),
                                                     B, k, a_s.data_ptr(), a_i.data_ptr(), ids.data_ptr(),
                                                     scores.data_ptr(), _stream(stream)))
    return ids, scores


ANN_STATIC_WORKSPACE_BYTES = 8 * 1024 * 1024


def ann_flat_search_static(corpus: torch.Tensor, queries: torch.Tensor, k: int, *, ids: torch.Tensor,
                           scores: torch.Tensor, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Exact top-k through the entry point that allocates nothing: the caller brings ids and
    scores, the workspace is the library's static array."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    with torch.cuda.device(corpus.device):
        _check(lib().ann_flat_search_static(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], queries.data_ptr(), B, k,
                                            ids.data_ptr(), scores.data_ptr(), _stream(stream)))
    return ids, scores


def ann_flat_search(corpus: torch.Tensor, queries: torch.Tensor, k: int, *, ids=None, scores=None,
                    stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Exact top-k through the short entry point, which assumes the library's default
    element type (fp16 unless ann_set_default_dtype changed it)."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    with torch.cuda.device(corpus.device):
        _check(lib().ann_flat_search(corpus.data_ptr(), N, d, queries.data_ptr(), B, k, ids.data_ptr(),
                                     scores.data_ptr(), _stream(stream)))
    return ids, scores


def _graph(graph: torch.Tensor, N: int) -> torch.Tensor:
    if graph.dim() != 2 or graph.dtype != torch.int32 or not graph.is_cuda or not graph.is_contiguous() \
            or graph.shape[0] != N:
        raise ValueError("graph must be a contiguous int32 [N, R] device tensor")
    return graph


def ann_graph_search_typed(corpus: torch.Tensor, graph: torch.Tensor, entry: int, queries: torch.Tensor, k: int,
                           ef: int, *, ids=None, scores=None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Best-first graph search with a candidate list of ef entries."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    _graph(graph, N)
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    with torch.cuda.device(corpus.device):
        _check(lib().ann_graph_search_typed(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], graph.data_ptr(),
                                            graph.shape[1], int(entry), queries.data_ptr(), B, k, ef,
                                            ids.data_ptr(), scores.data_ptr(), _stream(stream)))
    return ids, scores


def ann_graph_search_nonstall_typed(corpus: torch.Tensor, graph: torch.Tensor, entry: int, queries: torch.Tensor,
                                    k: int, ef: int, *, entries: Optional[torch.Tensor] = None, tau: float = 0.9,
                                    window: int = 500, engine_ready: Optional[torch.Tensor] = None, ids=None, scores=None,
                                    stats=None, ema=None, stream=None):
    """Graph search with the maturity (non-stall) exit.  `engine_ready` is an int32 tensor of one
    element on the device or in pinned host memory (None = always ready).  Returns
    (ids, scores, stats [B,3] = (early, scored, expansions), ema [B])."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    _graph(graph, N)
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    if stats is None:
        stats = torch.empty(B, 3, dtype=torch.int32, device=corpus.device)
    if ema is None:
        ema = torch.empty(B, dtype=torch.float32, device=corpus.device)
    if stats.dtype != torch.int32 or tuple(stats.shape) != (B, 3) or not stats.is_contiguous() or not stats.is_cuda:
        raise ValueError("stats must be a contiguous int32 [B, 3] device tensor")
    if ema.dtype != torch.float32 or tuple(ema.shape) != (B,) or not ema.is_contiguous() or not ema.is_cuda:
        raise ValueError("ema must be a contiguous float32 [B] device tensor")
    entries_ptr, n_entries = 0, 0
    if entries is not None:
        entries_ptr, n_entries = _entries(entries, B).data_ptr(), (1 if entries.dim() == 1 else entries.shape[1])
    ready_ptr = 0
    if engine_ready is not None:
        if engine_ready.dtype != torch.int32 or engine_ready.numel() != 1 or \
                not (engine_ready.is_cuda or engine_ready.is_pinned()):
            raise ValueError("engine_ready must be one int32 on the device or in pinned host memory")
        ready_ptr = engine_ready.data_ptr()
    with torch.cuda.device(corpus.device):
        _check(lib().ann_graph_search_nonstall_typed(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], graph.data_ptr(),
                                                     graph.shape[1], int(entry), queries.data_ptr(), B, k, ef,
                                                     entries_ptr, n_entries, float(tau), int(window), ready_ptr, ids.data_ptr(),
                                                     scores.data_ptr(), stats.data_ptr(), ema.data_ptr(),
                                                     _stream(stream)))
    return ids, scores, stats, ema


def _entries(entries: torch.Tensor, B: int) -> torch.Tensor:
    ok_shape = tuple(entries.shape) == (B,) or (entries.dim() == 2 and entries.shape[0] == B and entries.shape[1] >= 1)
    if entries.dtype != torch.int32 or not ok_shape or not entries.is_contiguous() or not entries.is_cuda:
        raise ValueError("entries must be a contiguous int32 [B] or [B, E] device tensor")
    return entries


def ann_graph_search_multi_typed(corpus: torch.Tensor, graph: torch.Tensor, entries: torch.Tensor,
                                 queries: torch.Tensor, k: int, ef: int, *, ids=None, scores=None,
                                 stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Graph search with entries[B, E] entry nodes per query."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    _graph(graph, N)
    _entries(entries, B)
    if entries.dim() != 2:
        raise ValueError("entries must be [B, E]")
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    with torch.cuda.device(corpus.device):
        _check(lib().ann_graph_search_multi_typed(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], graph.data_ptr(),
                                                  graph.shape[1], entries.data_ptr(), entries.shape[1],
                                                  queries.data_ptr(), B, k, ef, ids.data_ptr(), scores.data_ptr(),
                                                  _stream(stream)))
    return ids, scores


def ann_graph_search_entries_typed(corpus: torch.Tensor, graph: torch.Tensor, entries: torch.Tensor,
                                   queries: torch.Tensor, k: int, ef: int, *, ids=None, scores=None,
                                   stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Graph search with one entry node per query."""
    _matrix(corpus, "corpus"), _matrix(queries, "queries")
    if queries.dtype != corpus.dtype or queries.shape[1] != corpus.shape[1]:
        raise ValueError("queries must have the corpus' element type and dimension")
    (N, d), B = corpus.shape, queries.shape[0]
    _graph(graph, N)
    if _entries(entries, B).dim() != 1:
        raise ValueError("entries must be [B]")
    ids, scores = _outputs(B, k, corpus.device, ids, scores)
    with torch.cuda.device(corpus.device):
        _check(lib().ann_graph_search_entries_typed(corpus.data_ptr(), N, d, _DTYPES[corpus.dtype], graph.data_ptr(),
                                                    graph.shape[1], entries.data_ptr(), queries.data_ptr(), B, k, ef,
                                                    ids.data_ptr(), scores.data_ptr(), _stream(stream)))
    return ids, scores


def ann_gather_ids(table: torch.Tensor, idx: torch.Tensor, *, out=None, stream=None) -> torch.Tensor:
    """out[i] = table[idx[i]] (-1 where idx[i] is out of range); int32 device tensors."""
    for t in (table, idx):
        if t.dtype != torch.int32 or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("table and idx must be contiguous int32 device tensors")
    if out is None:
        out = torch.empty_like(idx)
    if out.dtype != torch.int32 or out.shape != idx.shape or not out.is_contiguous() or not out.is_cuda:
        raise ValueError("out must be a contiguous int32 device tensor shaped like idx")
    with torch.cuda.device(table.device):
        _check(lib().ann_gather_ids(table.data_ptr(), table.numel(), idx.data_ptr(), idx.numel(), out.data_ptr(),
                                    _stream(stream)))
    return out


KERNEL_FLAT_STREAM, KERNEL_FLAT_WIDE, KERNEL_FLAT_F32, KERNEL_GRAPH = 0, 1, 2, 3


def ann_priority_order(R: torch.Tensor, W: torch.Tensor, C: torch.Tensor, Wcur: torch.Tensor, G: int = 6, *,
                       stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Scheduler priority levels and execution order.  R, C int32 [n]; W, Wcur float64 [n]; device tensors."""
    n = R.numel()
    for t, dt in ((R, torch.int32), (C, torch.int32), (W, torch.float64), (Wcur, torch.float64)):
        if t.dtype != dt or t.numel() != n or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("R, C must be int32 and W, Wcur float64 contiguous device tensors of one length")
    level = torch.empty(n, dtype=torch.int32, device=R.device)
    order = torch.empty(n, dtype=torch.int32, device=R.device)
    with torch.cuda.device(R.device):
        _check(lib().ann_priority_order(R.data_ptr(), W.data_ptr(), C.data_ptr(), Wcur.data_ptr(), n, int(G),
                                        level.data_ptr(), order.data_ptr(), _stream(stream)))
    return level, order


def ann_measure_mfma_rate(random_operands: bool, iters: int = 100000) -> float:
    """Dense fp16 MFMA rate (TFLOP/s) the current device sustains on register operands."""
    out = ctypes.c_double(0.0)
    _check(lib().ann_measure_mfma_rate(1 if random_operands else 0, int(iters), ctypes.byref(out)))
    return out.value


def ann_timing_enable(on: bool) -> None:
    _check(lib().ann_timing_enable(1 if on else 0))


def ann_timing_read(kernel: int) -> Tuple[int, float]:
    """(launches, total milliseconds) of the main kernel `kernel` since timing was switched on."""
    n, ms = ctypes.c_int32(0), ctypes.c_double(0.0)
    _check(lib().ann_timing_read(kernel, ctypes.byref(n), ctypes.byref(ms)))
    return n.value, ms.value


def ann_timing_read_each(kernel: int):
    """Durations (ms) of the recorded launches of the main kernel `kernel`, in call order."""
    n = ctypes.c_int32(0)
    _check(lib().ann_timing_read_each(kernel, 0, ctypes.byref(n), None))
    buf = (ctypes.c_float * max(1, n.value))()
    _check(lib().ann_timing_read_each(kernel, n.value, ctypes.byref(n), buf))
    return [buf[i] for i in range(n.value)]


def ann_graph_nonstall_workspace_bytes(N: int, B: int) -> int:
    return int(lib().ann_graph_nonstall_workspace_bytes(N, B))


def ann_graph_search(corpus: torch.Tensor, graph: torch.Tensor, entry: int, queries: torch.Tensor, k: int, ef: int,
                     *, ids=None, scores=None, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Graph search through the short entry point: the corpus must have been registered."""
    _matrix(queries, "queries")
    B = queries.shape[0]
    ids, scores = _outputs(B, k, queries.device, ids, scores)
    with torch.cuda.device(queries.device):
        _check(lib().ann_graph_search(corpus.data_ptr(), graph.data_ptr(), graph.shape[1], int(entry),
                                      queries.data_ptr(), B, k, ef, ids.data_ptr(), scores.data_ptr(),
                                      _stream(stream)))
    return ids, scores


def ann_register_corpus(corpus: torch.Tensor) -> None:
    _matrix(corpus, "corpus")
    _check(lib().ann_register_corpus(corpus.data_ptr(), corpus.shape[0], corpus.shape[1], _DTYPES[corpus.dtype]))


def ann_unregister_corpus(corpus: torch.Tensor) -> None:
    _check(lib().ann_unregister_corpus(corpus.data_ptr()))


def ann_set_default_dtype(dtype: torch.dtype) -> None:
    _check(lib().ann_set_default_dtype(_DTYPES[dtype]))


def ann_flat_workspace_bytes(N: int, d: int, dtype: torch.dtype, B: int, k: int) -> int:
    return int(lib().ann_flat_workspace_bytes(N, d, _DTYPES[dtype], B, k))


def ann_set_workspace(buf: Optional[torch.Tensor]) -> None:
    """Use `buf` (a contiguous uint8 device tensor the caller keeps alive) as the workspace of its device;
    None hands the workspace back to the library."""
    if buf is None:
        _check(lib().ann_set_workspace(None, 0))
        return
    if buf.dtype != torch.uint8 or not buf.is_cuda or not buf.is_contiguous():
        raise ValueError("the workspace must be a contiguous uint8 device tensor")
    with torch.cuda.device(buf.device):
        _check(lib().ann_set_workspace(buf.data_ptr(), buf.numel()))


def ann_release_workspace() -> None:
    _check(lib().ann_release_workspace())
