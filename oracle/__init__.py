"""ctypes front end of the CPU oracle (oracle/tsdg_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg.  The product package never imports this
module and this module never imports the product package.

Every function takes and returns numpy arrays in host memory.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

F32, U8, F16 = 0, 1, 2
_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.orc_sqdist.restype = C.c_float
        L.orc_sqdist.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.orc_seed_id.restype = C.c_int64
        L.orc_seed_id.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_int64]
        L.orc_recall.restype = C.c_double
        L.orc_recall.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int]
        L.orc_max_threads.restype = C.c_int
        L.orc_descent_slot.restype = C.c_uint32
        L.orc_descent_slot.argtypes = [C.c_uint32, C.c_int]
        L.orc_alg2_stop.restype = C.c_int
        L.orc_alg2_stop.argtypes = [C.c_float, C.c_float, C.c_float, C.c_int]
        _lib = L
    return _lib


def _dtype_code(base: np.ndarray) -> int:
    if base.dtype == np.float32:
        return F32
    if base.dtype == np.uint8:
        return U8
    if base.dtype == np.float16:
        return F16
    raise TypeError("base must be float32, float16 or uint8")


def _c(a: np.ndarray, dt=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def max_threads() -> int:
    return int(lib().orc_max_threads())


def sqdist(a: np.ndarray, b: np.ndarray) -> np.float32:
    a = _c(a, np.float32)
    b = _c(b, np.float32)
    assert a.shape == b.shape and a.ndim == 1
    return np.float32(lib().orc_sqdist(_p(a), _p(b), a.shape[0]))


def seed_id(seed: int, qi: int, j: int, N: int) -> int:
    return int(lib().orc_seed_id(seed, qi, j, N))


def alg2_stop(s_u: float, s_f: float, delta: float, metric="l2") -> bool:
    """Stop test of Alg. 2 on squared distances s_u (popped candidate), s_f (furthest of R)."""
    return bool(lib().orc_alg2_stop(s_u, s_f, delta, METRICS[metric]))


def bruteforce(base, queries, k, threads=0):
    base = _c(base)
    queries = _c(queries, np.float32)
    N, d = base.shape
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.int32)
    s = np.empty((nq, k), np.float32)
    rc = lib().orc_bruteforce(_p(base), _dtype_code(base), C.c_int64(N), d, _p(queries),
                              C.c_int64(nq), k, 0, _p(ids), _p(s), threads)
    _check(rc, "bruteforce")
    return ids, s


def knn(base, K, threads=0):
    base = _c(base)
    N, d = base.shape
    ids = np.empty((N, K), np.int32)
    s = np.empty((N, K), np.float32)
    rc = lib().orc_knn(_p(base), _dtype_code(base), C.c_int64(N), d, K, _p(ids), _p(s), threads)
    _check(rc, "knn")
    return ids, s


METRICS = {"l2": 0, "cosine": 1}


def normalize_rows(x):
    """Unit rows for the cosine metric (fp64 sum of squares, norm and quotient rounded to fp32)."""
    x = _c(x, np.float32)
    out = np.empty_like(x)
    _check(lib().orc_normalize_rows(_p(x), C.c_int64(x.shape[0]), x.shape[1], _p(out)), "normalize_rows")
    return out


def ip_augment_rows(x, M=0.0, is_query=False):
    """Rows for the inner-product measure by its reduction to L2: [x, sqrt(M^2 - |x|^2), 0, 0, 0] for
    base rows (M >= every base norm), [q, 0, 0, 0, 0] for queries."""
    x = _c(x, np.float32)
    out = np.empty((x.shape[0], x.shape[1] + 4), np.float32)
    _check(lib().orc_ip_augment_rows(_p(x), C.c_int64(x.shape[0]), x.shape[1], C.c_float(M), int(bool(is_query)),
                                     _p(out)), "ip_augment_rows")
    return out


def stage1(base, knn_id, knn_s, alpha, threads=0, metric="l2"):
    base = _c(base)
    knn_id = _c(knn_id, np.int32)
    knn_s = _c(knn_s, np.float32)
    N, d = base.shape
    K = knn_id.shape[1]
    g1_id = np.empty((N, K), np.int32)
    g1_s = np.empty((N, K), np.float32)
    g1_deg = np.empty((N,), np.int32)
    rc = lib().orc_stage1_m(_p(base), _dtype_code(base), C.c_int64(N), d, K, _p(knn_id), _p(knn_s),
                            C.c_float(alpha), METRICS[metric], _p(g1_id), _p(g1_s), _p(g1_deg), threads)
    _check(rc, "stage1")
    return g1_id, g1_s, g1_deg


def reverse(base, g1_id, g1_deg, rev_cap, threads=0):
    base = _c(base)
    g1_id = _c(g1_id, np.int32)
    g1_deg = _c(g1_deg, np.int32)
    N, d = base.shape
    K = g1_id.shape[1]
    g2_id = np.empty((N, rev_cap), np.int32)
    g2_s = np.empty((N, rev_cap), np.float32)
    g2_deg = np.empty((N,), np.int32)
    rc = lib().orc_reverse(_p(base), _dtype_code(base), C.c_int64(N), d, K, _p(g1_id), _p(g1_deg),
                           rev_cap, _p(g2_id), _p(g2_s), _p(g2_deg), threads)
    _check(rc, "reverse")
    return g2_id, g2_s, g2_deg


def stage2(base, g2_id, g2_s, g2_deg, lambda0, K, threads=0):
    base = _c(base)
    g2_id = _c(g2_id, np.int32)
    g2_s = _c(g2_s, np.float32)
    g2_deg = _c(g2_deg, np.int32)
    N, d = base.shape
    rev_cap = g2_id.shape[1]
    adj = np.empty((N, K), np.int32)
    lam = np.empty((N, K), np.uint8)
    rc = lib().orc_stage2(_p(base), _dtype_code(base), C.c_int64(N), d, rev_cap, _p(g2_id), _p(g2_s),
                          _p(g2_deg), lambda0, K, _p(adj), _p(lam), threads)
    _check(rc, "stage2")
    return adj, lam


def build_graph(base, K, alpha=1.2, lambda0=9, rev_cap=None, threads=0, stages=False, metric="l2"):
    """Exact k-NN -> stage 1 -> reverse edges -> stage 2.  Returns (adj, lam),
    plus a dict of the intermediate arrays when stages=True.  metric="cosine" expects unit rows
    (normalize_rows) and applies Eq. 2 to m = 1 - cos = s/2; the distances in `stages` stay s."""
    base = _c(base)
    N, d = base.shape
    if rev_cap is None:
        rev_cap = 2 * K
    adj = np.empty((N, K), np.int32)
    lam = np.empty((N, K), np.uint8)
    st = None
    args = [None] * 7
    if stages:
        st = dict(knn_id=np.empty((N, K), np.int32), knn_s=np.empty((N, K), np.float32),
                  g1_id=np.empty((N, K), np.int32), g1_deg=np.empty((N,), np.int32),
                  g2_id=np.empty((N, rev_cap), np.int32), g2_s=np.empty((N, rev_cap), np.float32),
                  g2_deg=np.empty((N,), np.int32))
        args = [st["knn_id"], st["knn_s"], st["g1_id"], st["g1_deg"], st["g2_id"], st["g2_s"],
                st["g2_deg"]]
    rc = lib().orc_build_m(_p(base), _dtype_code(base), C.c_int64(N), d, K, C.c_float(alpha), METRICS[metric],
                           lambda0, rev_cap, _p(adj), _p(lam), *[_p(a) for a in args], threads)
    _check(rc, "build")
    return (adj, lam, st) if stages else (adj, lam)


def search(adj, lam, base, queries, k, L, lambda_visit, n_seeds=32, seed=0, max_hops=0,
           visited_cap=0, reverse_hop=False, qi_offset=0, threads=0, want_stats=False,
           trace_cap=0, metric="l2"):
    """metric="cosine": base rows and queries are unit vectors; the walk is the same (m = s/2 orders
    like s) and the distances returned are m = 1 - cos = s/2 (halving is exact in fp32)."""
    adj = _c(adj, np.int32)
    lam = _c(lam, np.uint8)
    base = _c(base)
    queries = _c(queries, np.float32)
    N, d = base.shape
    K = adj.shape[1]
    nq = queries.shape[0]
    assert adj.shape[0] == N and lam.shape == adj.shape and queries.shape[1] == d
    ids = np.empty((nq, k), np.int32)
    s = np.empty((nq, k), np.float32)
    stats = np.zeros((nq, 3), np.uint32) if want_stats else None
    trace = np.full((nq, trace_cap), -1, np.int32) if trace_cap else None
    rc = lib().orc_search(_p(adj), _p(lam), C.c_int64(N), K, _p(base), _dtype_code(base), d,
                          _p(queries), C.c_int64(nq), k, L, lambda_visit, n_seeds,
                          C.c_uint64(seed), max_hops, visited_cap, int(bool(reverse_hop)),
                          C.c_int64(qi_offset), _p(ids), _p(s), _p(stats), _p(trace), trace_cap,
                          threads)
    _check(rc, "search")
    if METRICS[metric] == 1:
        s = s * np.float32(0.5)
    out = [ids, s]
    if want_stats:
        out.append(stats)
    if trace_cap:
        out.append(trace)
    return tuple(out)


def search_multi(adj, lam, base, queries, k, t0, max_hops=16, lambda_visit=10, seed=0, qi_offset=0, threads=0,
                 want_stats=False, metric="l2"):
    """Small-batch multi-search (Alg. 1): t0 greedy searches per query, merged.  metric="cosine":
    unit rows, distances returned as m = s/2."""
    adj = _c(adj, np.int32)
    lam = _c(lam, np.uint8)
    base = _c(base)
    queries = _c(queries, np.float32)
    N, d = base.shape
    K = adj.shape[1]
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.int32)
    s = np.empty((nq, k), np.float32)
    stats = np.zeros((nq, 3), np.uint32) if want_stats else None
    rc = lib().orc_search_multi(_p(adj), _p(lam), C.c_int64(N), K, _p(base), _dtype_code(base), d, _p(queries),
                                C.c_int64(nq), k, t0, max_hops, lambda_visit, C.c_uint64(seed),
                                C.c_int64(qi_offset), _p(ids), _p(s), _p(stats), threads)
    _check(rc, "search_multi")
    if METRICS[metric] == 1:
        s = s * np.float32(0.5)
    return (ids, s, stats) if want_stats else (ids, s)


def search_alg2(adj, lam, base, queries, k, delta, m_c=16, m_v=16, max_hops=0, lambda_visit=5, seed=0, qi_offset=0,
                threads=0, want_stats=False, metric="l2"):
    """Large-batch search with the paper's own R / C / V structures and the Delta stop (Alg. 2).
    delta is in units of the measure m: the L2 distance sqrt(s) for metric="l2", 1 - cos = s/2 for
    metric="cosine" (unit rows; the distances returned are then m = s/2)."""
    adj = _c(adj, np.int32)
    lam = _c(lam, np.uint8)
    base = _c(base)
    queries = _c(queries, np.float32)
    N, d = base.shape
    K = adj.shape[1]
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.int32)
    s = np.empty((nq, k), np.float32)
    stats = np.zeros((nq, 3), np.uint32) if want_stats else None
    rc = lib().orc_search_alg2(_p(adj), _p(lam), C.c_int64(N), K, _p(base), _dtype_code(base), d, _p(queries),
                               C.c_int64(nq), k, m_c, m_v, C.c_float(delta), METRICS[metric], max_hops, lambda_visit,
                               C.c_uint64(seed), C.c_int64(qi_offset), _p(ids), _p(s), _p(stats), threads)
    _check(rc, "search_alg2")
    if METRICS[metric] == 1:
        s = s * np.float32(0.5)
    return (ids, s, stats) if want_stats else (ids, s)


def descent_slot(u: int, S: int) -> int:
    """Cell of source u in a reverse-sample table of S cells (neighbourhood propagation)."""
    return int(lib().orc_descent_slot(u, S.bit_length() - 1))


def knn_descent(base, K, S=8, max_iters=10, delta=0.001, seed=0, init_ids=None, threads=0):
    """Approximate k-NN lists by neighbourhood propagation (pull form, deterministic).
    Returns (ids [N,K], s [N,K], iterations done, entries changed per iteration)."""
    base = _c(base)
    N, d = base.shape
    ids = np.empty((N, K), np.int32)
    s = np.empty((N, K), np.float32)
    done = C.c_int32(0)
    changed = np.zeros((max(max_iters, 1),), np.int64)
    init = _c(init_ids, np.int32) if init_ids is not None else None
    rc = lib().orc_knn_descent(_p(base), _dtype_code(base), C.c_int64(N), d, K, S, max_iters, C.c_float(delta),
                               C.c_uint64(seed), _p(init), _p(ids), _p(s), C.byref(done), _p(changed), threads)
    _check(rc, "knn_descent")
    return ids, s, done.value, changed[:done.value]


def recall(found, truth) -> float:
    found = _c(found, np.int32)
    truth = _c(truth, np.int32)
    assert found.shape == truth.shape
    return float(lib().orc_recall(_p(found), _p(truth), C.c_int64(found.shape[0]), found.shape[1]))
