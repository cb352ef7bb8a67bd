"""ctypes binding of include/tsdg_ann.h.  Same names as the C entry points;
torch is used for device memory and streams only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

ANN_F32, ANN_U8, ANN_F16 = 0, 1, 2
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtsdg_ann.so")
_lib = None

_STATUS = {1: "ANN_EINVAL", 2: "ANN_ENOMEM", 3: "ANN_EDEVICE", 4: "ANN_EUNSUPPORTED"}


class AnnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


_PROGRESS_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_char_p, C.c_int64, C.c_int64)


class _BuildStats(C.Structure):
    _fields_ = [("knn_ms", C.c_float), ("stage1_ms", C.c_float), ("reverse_ms", C.c_float), ("stage2_ms", C.c_float),
                ("stage1_rows", C.c_uint64), ("stage2_rows", C.c_uint64), ("reverse_edges", C.c_uint64),
                ("gather_row_bytes", C.c_int), ("knn_contraction", C.c_int), ("knn_plain_scan_rows", C.c_uint32)]

    def as_dict(self):
        return {name: getattr(self, name) for name, _ in self._fields_}


class _BuildParams(C.Structure):
    _fields_ = [("dtype", C.c_int), ("alpha", C.c_float), ("lambda0", C.c_int), ("rev_cap", C.c_int),
                ("stream", C.c_void_p), ("metric", C.c_int), ("knn_mode", C.c_int), ("descent_S", C.c_int),
                ("descent_iters", C.c_int), ("descent_delta", C.c_float), ("descent_seed", C.c_uint64),
                ("knn_filter", C.c_int), ("knn_row_block", C.c_int64), ("progress", _PROGRESS_FN),
                ("progress_user", C.c_void_p), ("stats", C.POINTER(_BuildStats))]


class _SearchParams(C.Structure):
    _fields_ = [("dtype", C.c_int), ("mode", C.c_int), ("lambda_visit", C.c_int), ("n_seeds", C.c_int),
                ("seed", C.c_uint64), ("max_hops", C.c_int), ("visited_slots", C.c_int),
                ("waves_per_query", C.c_int), ("qi_offset", C.c_int64), ("stream", C.c_void_p),
                ("metric", C.c_int)]


ANN_L2, ANN_COSINE = 0, 1
_METRICS = {"l2": ANN_L2, "cosine": ANN_COSINE, ANN_L2: ANN_L2, ANN_COSINE: ANN_COSINE}


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built library; builds it first only when no built file exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build(force=True)
    L = C.CDLL(_LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int, C.c_int64, C.c_uint64
    L.ann_last_error.restype = C.c_char_p
    L.ann_build_params_default.argtypes = [C.POINTER(_BuildParams)]
    L.ann_search_params_default.argtypes = [C.POINTER(_SearchParams)]
    L.ann_build_graph.argtypes = [vp, i64, i32, i32, C.POINTER(vp)]
    L.ann_build_graph_ex.argtypes = [vp, i64, i32, i32, C.POINTER(_BuildParams), C.POINTER(vp)]
    L.ann_knn.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp]
    L.ann_knn_ex.argtypes = [vp, i64, i32, i32, C.POINTER(_BuildParams), vp, vp]
    L.ann_bruteforce.argtypes = [vp, i64, i32, i32, vp, i32, i32, vp, vp, vp]
    L.ann_search.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    L.ann_search_ex.argtypes = [vp, vp, vp, i32, i32, i32, C.POINTER(_SearchParams), vp, vp, vp]
    L.ann_search_multi.argtypes = [vp, vp, vp, i32, i32, i32, C.POINTER(_SearchParams), vp, C.c_size_t, vp, vp, vp]
    L.ann_search_multi_static.argtypes = [vp, vp, vp, i32, i32, i32, C.POINTER(_SearchParams), vp, vp, vp]
    L.ann_search_multi_workspace_bytes.argtypes = [i32, i32]
    L.ann_search_multi_workspace_bytes.restype = C.c_size_t
    L.ann_search_alg2.argtypes = [vp, vp, vp, i32, i32, C.c_float, i32, i32, C.POINTER(_SearchParams), vp, vp, vp]
    L.ann_graph_export.argtypes = [vp, vp, vp, vp]
    L.ann_graph_import.argtypes = [vp, vp, i64, i32, i32, vp, C.POINTER(vp)]
    L.ann_graph_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32)]
    L.ann_graph_free.argtypes = [vp]
    L.ann_probe_gather.argtypes = [vp, i64, i32, vp, i64, vp, vp]
    L.ann_probe_mfma.argtypes = [i32, i32, i32, vp, vp]
    L.ann_normalize_rows.argtypes = [vp, i64, i32, vp, vp]
    L.ann_max_row_norm.argtypes = [vp, i64, i32, vp, C.POINTER(C.c_float)]
    L.ann_ip_augment_rows.argtypes = [vp, i64, i32, C.c_float, i32, vp, vp]
    L.ann_knn_descent.argtypes = [vp, i64, i32, i32, i32, i32, i32, C.c_float, u64, vp, vp, vp, vp,
                                  C.POINTER(i32), C.POINTER(i64)]
    L.ann_graph_free.restype = None
    for name in ("ann_build_graph", "ann_build_graph_ex", "ann_knn", "ann_knn_ex", "ann_bruteforce", "ann_search",
                 "ann_search_ex", "ann_search_multi", "ann_search_multi_static", "ann_search_alg2", "ann_graph_export", "ann_graph_import", "ann_graph_info", "ann_probe_gather", "ann_probe_mfma", "ann_normalize_rows", "ann_knn_descent", "ann_max_row_norm", "ann_ip_augment_rows"):
        getattr(L, name).restype = C.c_int
    del u64
    _lib = L
    return L


def ann_last_error() -> str:
    return load_library().ann_last_error().decode()


def _check(status: int):
    if status != 0:
        raise AnnError(status, ann_last_error())


def _stream_ptr(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise TypeError(f"{name}: need a contiguous CUDA tensor of {dtype}")
    return t.data_ptr()


def _base_ptr(base: torch.Tensor):
    if base.dtype == torch.float32:
        return _dev(base, torch.float32, "base"), ANN_F32
    if base.dtype == torch.uint8:
        return _dev(base, torch.uint8, "base"), ANN_U8
    if base.dtype == torch.float16:      # storage type of the search calls
        return _dev(base, torch.float16, "base"), ANN_F16
    raise TypeError("base: float32, float16 or uint8 rows")


class Graph:
    """Owner of an ann_graph*; freed on deletion or with ann_graph_free."""

    def __init__(self, ptr: int):
        self.ptr = ptr

    def __del__(self):
        try:
            ann_graph_free(self)
        except Exception:
            pass


@dataclass
class QueryStats:
    hops: torch.Tensor
    dist_evals: torch.Tensor
    dedup_hits: torch.Tensor


def ann_build_graph(base: torch.Tensor, K: int) -> Graph:
    p, dt = _base_ptr(base)
    if dt != ANN_F32:
        raise TypeError("ann_build_graph takes fp32 rows; use ann_build_graph_ex for uint8")
    out = C.c_void_p()
    _check(load_library().ann_build_graph(p, base.shape[0], base.shape[1], K, C.byref(out)))
    return Graph(out.value)


def _build_params(L, dt, stream, *, alpha=1.2, lambda0=9, rev_cap=0, metric="l2", knn_mode=0, descent_S=0,
                  descent_iters=0, descent_delta=0.0, descent_seed=0, knn_filter=0, knn_row_block=0, progress=None,
                  want_stats=False):
    """Fills an ann_build_params; returns it with the objects that must outlive the call."""
    prm = _BuildParams()
    L.ann_build_params_default(C.byref(prm))
    prm.dtype, prm.alpha, prm.lambda0, prm.rev_cap, prm.stream = dt, alpha, lambda0, rev_cap, _stream_ptr(stream)
    prm.metric = _METRICS[metric]
    prm.knn_mode, prm.descent_S, prm.descent_iters = knn_mode, descent_S, descent_iters
    prm.descent_delta, prm.descent_seed = descent_delta, descent_seed
    prm.knn_filter, prm.knn_row_block = knn_filter, knn_row_block
    keep = []
    if progress is not None:
        cb = _PROGRESS_FN(lambda user, step, done, total: progress(step.decode(), done, total))
        prm.progress = cb
        keep.append(cb)
    stats = None
    if want_stats:
        stats = _BuildStats()
        prm.stats = C.pointer(stats)
    return prm, stats, keep


def ann_build_graph_ex(base: torch.Tensor, K: int, alpha: float = 1.2, lambda0: int = 9, rev_cap: int = 0,
                       stream=None, metric="l2", knn_mode: int = 0, descent_S: int = 0, descent_iters: int = 0,
                       descent_delta: float = 0.0, descent_seed: int = 0, knn_filter: int = 0, knn_row_block: int = 0,
                       progress=None, want_stats: bool = False):
    """Returns the graph, or (graph, stats dict) with want_stats.  progress(step, done, total) is called
    between launches of a long build."""
    L = load_library()
    p, dt = _base_ptr(base)
    prm, stats, keep = _build_params(L, dt, stream, alpha=alpha, lambda0=lambda0, rev_cap=rev_cap, metric=metric,
                                     knn_mode=knn_mode, descent_S=descent_S, descent_iters=descent_iters,
                                     descent_delta=descent_delta, descent_seed=descent_seed, knn_filter=knn_filter,
                                     knn_row_block=knn_row_block, progress=progress, want_stats=want_stats)
    out = C.c_void_p()
    _check(L.ann_build_graph_ex(p, base.shape[0], base.shape[1], K, C.byref(prm), C.byref(out)))
    del keep
    g = Graph(out.value)
    return (g, stats.as_dict()) if want_stats else g


def ann_knn(base: torch.Tensor, K: int, stream=None, knn_filter: int = 0, knn_row_block: int = 0, progress=None,
            want_stats: bool = False):
    """Exact K nearest neighbours of every row: (ids, dists) or (ids, dists, stats dict)."""
    L = load_library()
    p, dt = _base_ptr(base)
    N, d = base.shape
    ids = torch.empty((N, K), dtype=torch.int32, device=base.device)
    s = torch.empty((N, K), dtype=torch.float32, device=base.device)
    prm, stats, keep = _build_params(L, dt, stream, knn_filter=knn_filter, knn_row_block=knn_row_block,
                                     progress=progress, want_stats=want_stats)
    _check(L.ann_knn_ex(p, N, d, K, C.byref(prm), ids.data_ptr(), s.data_ptr()))
    del keep
    return (ids, s, stats.as_dict()) if want_stats else (ids, s)


def ann_knn_descent(base: torch.Tensor, K: int, S: int = 8, max_iters: int = 12, delta: float = 0.001, seed: int = 0,
                    init_ids: torch.Tensor = None, stream=None):
    """Approximate k-NN lists by neighbourhood propagation.  Returns (ids, dists, iterations, last_changed)."""
    p, dt = _base_ptr(base)
    N, d = base.shape
    ids = torch.empty((N, K), dtype=torch.int32, device=base.device)
    s = torch.empty((N, K), dtype=torch.float32, device=base.device)
    done, changed = C.c_int(0), C.c_int64(0)
    init = _dev(init_ids, torch.int32, "init_ids") if init_ids is not None else None
    _check(load_library().ann_knn_descent(p, N, d, K, dt, S, max_iters, C.c_float(delta), C.c_uint64(seed), init,
                                          _stream_ptr(stream), ids.data_ptr(), s.data_ptr(), C.byref(done),
                                          C.byref(changed)))
    return ids, s, done.value, changed.value


def ann_bruteforce(base: torch.Tensor, queries: torch.Tensor, k: int, stream=None):
    p, dt = _base_ptr(base)
    N, d = base.shape
    q = _dev(queries, torch.float32, "queries")
    if queries.shape[1] != d:
        raise ValueError("queries: wrong row length")
    nq = queries.shape[0]
    ids = torch.empty((nq, k), dtype=torch.int32, device=base.device)
    s = torch.empty((nq, k), dtype=torch.float32, device=base.device)
    _check(load_library().ann_bruteforce(p, N, d, dt, q, nq, k, _stream_ptr(stream), ids.data_ptr(), s.data_ptr()))
    return ids, s


def ann_search(graph: Graph, base: torch.Tensor, queries: torch.Tensor, k: int, L: int):
    p, dt = _base_ptr(base)
    if dt != ANN_F32:
        raise TypeError("ann_search takes fp32 rows; use ann_search_ex for uint8")
    q = _dev(queries, torch.float32, "queries")
    nq = queries.shape[0]
    ids = torch.empty((nq, k), dtype=torch.int32, device=base.device)
    s = torch.empty((nq, k), dtype=torch.float32, device=base.device)
    _check(load_library().ann_search(graph.ptr, p, q, nq, k, L, ids.data_ptr(), s.data_ptr()))
    return ids, s


def ann_search_ex(graph: Graph, base: torch.Tensor, queries: torch.Tensor, k: int, L: int, *, mode: int = 0,
                  lambda_visit: int = 0, n_seeds: int = 32, seed: int = 0, max_hops: int = 0,
                  visited_slots: int = 0, waves_per_query: int = 0, qi_offset: int = 0, stream=None,
                  want_stats: bool = False, out=None, metric="l2"):
    """Returns (ids, dists) or (ids, dists, QueryStats).  `out=(ids, dists)` reuses output tensors."""
    lib = load_library()
    p, dt = _base_ptr(base)
    q = _dev(queries, torch.float32, "queries")
    nq = queries.shape[0]
    if out is None:
        ids = torch.empty((nq, k), dtype=torch.int32, device=base.device)
        s = torch.empty((nq, k), dtype=torch.float32, device=base.device)
    else:
        ids, s = out
        _dev(ids, torch.int32, "out ids")
        _dev(s, torch.float32, "out dists")
    prm = _SearchParams()
    lib.ann_search_params_default(C.byref(prm))
    prm.dtype, prm.mode, prm.lambda_visit, prm.n_seeds, prm.seed = dt, mode, lambda_visit, n_seeds, seed
    prm.max_hops, prm.visited_slots, prm.waves_per_query = max_hops, visited_slots, waves_per_query
    prm.qi_offset, prm.stream, prm.metric = qi_offset, _stream_ptr(stream), _METRICS[metric]
    st = torch.zeros((nq, 3), dtype=torch.int32, device=base.device) if want_stats else None
    _check(lib.ann_search_ex(graph.ptr, p, q, nq, k, L, C.byref(prm), ids.data_ptr(), s.data_ptr(),
                             st.data_ptr() if st is not None else None))
    if want_stats:
        return ids, s, QueryStats(st[:, 0], st[:, 1], st[:, 2])
    return ids, s


def ann_search_multi_workspace_bytes(nq: int, t0: int) -> int:
    return int(load_library().ann_search_multi_workspace_bytes(nq, t0))


def ann_search_multi(graph: Graph, base: torch.Tensor, queries: torch.Tensor, k: int, t0: int, *,
                     lambda_visit: int = 0, seed: int = 0, max_hops: int = 0, qi_offset: int = 0, stream=None,
                     want_stats: bool = False, out=None, metric="l2", workspace: torch.Tensor = None, _static=False):
    """Small-batch multi-search (Alg. 1).  Returns (ids, dists) or (ids, dists, QueryStats).
    `workspace`: a uint8 device tensor of at least ann_search_multi_workspace_bytes(nq, t0) bytes that the
    caller keeps for its calls; without one this wrapper takes one from torch's allocator for the call."""
    lib = load_library()
    p, dt = _base_ptr(base)
    q = _dev(queries, torch.float32, "queries")
    nq = queries.shape[0]
    if out is None:
        ids = torch.empty((nq, k), dtype=torch.int32, device=base.device)
        s = torch.empty((nq, k), dtype=torch.float32, device=base.device)
    else:
        ids, s = out
        _dev(ids, torch.int32, "out ids")
        _dev(s, torch.float32, "out dists")
    prm = _SearchParams()
    lib.ann_search_params_default(C.byref(prm))
    prm.dtype, prm.lambda_visit, prm.seed, prm.max_hops = dt, lambda_visit, seed, max_hops
    prm.qi_offset, prm.stream, prm.metric = qi_offset, _stream_ptr(stream), _METRICS[metric]
    st = torch.zeros((nq, 3), dtype=torch.int32, device=base.device) if want_stats else None
    stp = st.data_ptr() if st is not None else None
    if _static:
        _check(lib.ann_search_multi_static(graph.ptr, p, q, nq, k, t0, C.byref(prm), ids.data_ptr(), s.data_ptr(), stp))
    else:
        if workspace is None:
            need = int(lib.ann_search_multi_workspace_bytes(nq, max(t0, 1))) if nq > 0 else 0
            workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=base.device)
            if stream is not None:          # the block must not be handed out again before that stream is done with it
                workspace.record_stream(stream)
        _dev(workspace, torch.uint8, "workspace")
        _check(lib.ann_search_multi(graph.ptr, p, q, nq, k, t0, C.byref(prm), workspace.data_ptr(), workspace.numel(),
                                    ids.data_ptr(), s.data_ptr(), stp))
    if want_stats:
        return ids, s, QueryStats(st[:, 0], st[:, 1], st[:, 2])
    return ids, s


def ann_search_multi_static(graph: Graph, base: torch.Tensor, queries: torch.Tensor, k: int, t0: int, **kw):
    """ann_search_multi on the library's own scratch: the C call allocates nothing (nq * t0 <= 2048).
    Pass `out=(ids, dists)` to keep this wrapper from allocating the outputs too."""
    return ann_search_multi(graph, base, queries, k, t0, _static=True, **kw)


def ann_search_alg2(graph: Graph, base: torch.Tensor, queries: torch.Tensor, k: int, delta: float, *, m_c: int = 16,
                    m_v: int = 16, lambda_visit: int = 0, seed: int = 0, max_hops: int = 0, qi_offset: int = 0,
                    stream=None, want_stats: bool = False, out=None, metric="l2"):
    """Search with the paper's own R / C / V structures (Alg. 2)."""
    lib = load_library()
    p, dt = _base_ptr(base)
    q = _dev(queries, torch.float32, "queries")
    nq = queries.shape[0]
    if out is None:
        ids = torch.empty((nq, k), dtype=torch.int32, device=base.device)
        s = torch.empty((nq, k), dtype=torch.float32, device=base.device)
    else:
        ids, s = out
        _dev(ids, torch.int32, "out ids")
        _dev(s, torch.float32, "out dists")
    prm = _SearchParams()
    lib.ann_search_params_default(C.byref(prm))
    prm.dtype, prm.lambda_visit, prm.seed, prm.max_hops = dt, lambda_visit, seed, max_hops
    prm.qi_offset, prm.stream, prm.metric = qi_offset, _stream_ptr(stream), _METRICS[metric]
    st = torch.zeros((nq, 3), dtype=torch.int32, device=base.device) if want_stats else None
    _check(lib.ann_search_alg2(graph.ptr, p, q, nq, k, C.c_float(delta), m_c, m_v, C.byref(prm), ids.data_ptr(),
                               s.data_ptr(), st.data_ptr() if st is not None else None))
    if want_stats:
        return ids, s, QueryStats(st[:, 0], st[:, 1], st[:, 2])
    return ids, s


def ann_graph_export(graph: Graph, stream=None):
    N, K, _ = ann_graph_info(graph)
    adj = torch.empty((N, K), dtype=torch.int32, device="cuda")
    lam = torch.empty((N, K), dtype=torch.uint8, device="cuda")
    _check(load_library().ann_graph_export(graph.ptr, adj.data_ptr(), lam.data_ptr(), _stream_ptr(stream)))
    return adj, lam


def ann_graph_import(adj: torch.Tensor, lam: torch.Tensor, d: int, stream=None) -> Graph:
    a = _dev(adj, torch.int32, "adj")
    l = _dev(lam, torch.uint8, "lam")
    if adj.shape != lam.shape or adj.dim() != 2:
        raise ValueError("adj and lam must both be [N,K]")
    out = C.c_void_p()
    _check(load_library().ann_graph_import(a, l, adj.shape[0], adj.shape[1], d, _stream_ptr(stream), C.byref(out)))
    return Graph(out.value)


def ann_graph_info(graph: Graph):
    N, K, d = C.c_int64(), C.c_int(), C.c_int()
    _check(load_library().ann_graph_info(graph.ptr, C.byref(N), C.byref(K), C.byref(d)))
    return N.value, K.value, d.value


def ann_normalize_rows(x: torch.Tensor, out: torch.Tensor = None, stream=None) -> torch.Tensor:
    """Unit rows for the cosine metric; `out` may be `x` itself."""
    src = _dev(x, torch.float32, "x")
    if out is None:
        out = torch.empty_like(x)
    _check(load_library().ann_normalize_rows(src, x.shape[0], x.shape[1], _dev(out, torch.float32, "out"),
                                             _stream_ptr(stream)))
    return out


def ann_max_row_norm(x: torch.Tensor, stream=None) -> float:
    M = C.c_float(0.0)
    _check(load_library().ann_max_row_norm(_dev(x, torch.float32, "x"), x.shape[0], x.shape[1], _stream_ptr(stream),
                                           C.byref(M)))
    return M.value


def ann_ip_augment_rows(x: torch.Tensor, M: float = 0.0, is_query: bool = False, stream=None) -> torch.Tensor:
    """Rows for the inner-product measure by its reduction to L2 (d + 4 columns)."""
    out = torch.empty((x.shape[0], x.shape[1] + 4), dtype=torch.float32, device=x.device)
    _check(load_library().ann_ip_augment_rows(_dev(x, torch.float32, "x"), x.shape[0], x.shape[1], C.c_float(M),
                                              int(bool(is_query)), out.data_ptr(), _stream_ptr(stream)))
    return out


def ann_probe_gather(base: torch.Tensor, ids: torch.Tensor, out: torch.Tensor = None, stream=None) -> torch.Tensor:
    """Measurement probe: gathers base[ids] row by row and returns one xor-folded word per row."""
    if not (base.is_cuda and base.is_contiguous() and base.dim() == 2):
        raise ValueError("base must be a contiguous [N,d] device tensor")
    row_bytes = base.shape[1] * base.element_size()
    i = _dev(ids, torch.int32, "ids")
    if out is None:
        out = torch.empty(ids.numel(), dtype=torch.int32, device=base.device)
    _check(load_library().ann_probe_gather(base.data_ptr(), base.shape[0], row_bytes, i, ids.numel(),
                                           _dev(out, torch.int32, "out"), _stream_ptr(stream)))
    return out


def ann_probe_mfma(kind: int, blocks: int, iters: int, out: torch.Tensor = None, stream=None) -> torch.Tensor:
    """Measurement probe: 4 * iters matrix-core instructions per wavefront on register operands
    (kind 0 int8 32x32x32, kind 1 bf16 32x32x16, on fragments of ones; kinds 2 and 3 the same on
    pseudo-random fragments); returns one float per wavefront."""
    if out is None:
        out = torch.empty(4 * blocks, dtype=torch.float32, device="cuda")
    if out.numel() < 4 * blocks:
        raise ValueError("out must hold 4 * blocks floats")
    _check(load_library().ann_probe_mfma(int(kind), int(blocks), int(iters), _dev(out, torch.float32, "out"),
                                         _stream_ptr(stream)))
    return out


def ann_graph_free(graph: Graph) -> None:
    if graph is not None and getattr(graph, "ptr", None):
        load_library().ann_graph_free(graph.ptr)
        graph.ptr = None
