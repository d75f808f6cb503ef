"""ctypes front end of the CPU oracle (oracle/cagra_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of the benchmark.  The product package never imports it, and
it never imports the product package.  It computes in numpy arrays on the
host; nothing here touches a GPU.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cagra_oracle.c")
_LIB = os.path.join(_HERE, "libcagra_oracle.so")

L2 = 0
IP = 1
INVALID_ID = 0xFFFFFFFF
FLT_MAX = float(np.finfo(np.float32).max)

_lib = None


def build_lib(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off keeps the compiler from
    fusing or splitting any floating-point operation the source does not spell
    out; -mfma only lets fmaf() map to the hardware instruction."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-mfma", "-mavx2", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_lib()
        lib = C.CDLL(_LIB)
        u32p, f32p, i64p = C.POINTER(C.c_uint32), C.POINTER(C.c_float), C.POINTER(C.c_int64)
        i32, i64, u64 = C.c_int32, C.c_int64, C.c_uint64
        lib.oracle_distance.restype = C.c_float
        lib.oracle_distance.argtypes = [f32p, f32p, i32, i32]
        lib.oracle_exact_search.argtypes = [f32p, i64, i32, i32, f32p, i64, i32, u32p, f32p]
        lib.oracle_knn_graph.argtypes = [f32p, i64, i32, i32, i64p, i64, i32, u32p, f32p]
        lib.oracle_detour_count.argtypes = [u32p, i64, i32, i64p, i64, u32p]
        lib.oracle_detour_count_distance.argtypes = [u32p, f32p, i64, i32, i64p, i64, u32p]
        lib.oracle_optimize_ex.argtypes = [u32p, f32p, i64, i32, i32, u32p]
        lib.oracle_build_ex.argtypes = [f32p, i64, i32, i32, i32, i32, i32, u32p]
        lib.oracle_nn_descent.argtypes = [f32p, i64, i32, i32, i32, i32, i32, u64, u32p, f32p]
        lib.oracle_two_hop_counts.argtypes = [u32p, i64, i32, u32p]
        lib.oracle_strong_components.restype = i64
        lib.oracle_strong_components.argtypes = [u32p, i64, i32]
        lib.oracle_weak_components.restype = i64
        lib.oracle_weak_components.argtypes = [u32p, i64, i32]
        lib.oracle_prune.argtypes = [u32p, u32p, i64, i32, i32, u32p]
        lib.oracle_reverse.argtypes = [u32p, i64, i32, u32p, u32p]
        lib.oracle_merge.argtypes = [u32p, u32p, u32p, i64, i32, u32p]
        lib.oracle_optimize.argtypes = [u32p, i64, i32, i32, u32p]
        lib.oracle_build.argtypes = [f32p, i64, i32, i32, i32, i32, u32p]
        lib.oracle_splitmix_fin.restype = u64
        lib.oracle_splitmix_fin.argtypes = [u64]
        lib.oracle_seed_id.restype = C.c_uint32
        lib.oracle_seed_id.argtypes = [u64, u64, u64, u64]
        lib.oracle_auto_max_iterations.restype = i32
        lib.oracle_auto_max_iterations.argtypes = [i32, i32]
        lib.oracle_search.argtypes = [u32p, i64, i32, f32p, i32, i32, f32p, i64, i32, i32, i32,
                                      u64, i32, i32, i32, u32p, f32p, u32p]
        lib.oracle_search_multi.argtypes = [u32p, i64, i32, f32p, i32, i32, f32p, i64, i32, i32,
                                            i32, u64, i32, i32, u32p, f32p, u32p]
        lib.oracle_search_multi_lists.argtypes = [u32p, i64, i32, f32p, i32, i32, f32p, i64, i32, i32,
                                                  i32, u64, i32, i32, u32p, f32p, u32p, u32p]
        lib.oracle_num_threads.restype = i32
        _lib = lib
    return _lib


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _u32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint32)


def _p(a: Optional[np.ndarray], ct):
    return None if a is None else a.ctypes.data_as(C.POINTER(ct))


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} rejected its arguments (code {rc})")


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def distance(x, y, metric: int = L2) -> float:
    x, y = _f32(x), _f32(y)
    return float(_load().oracle_distance(_p(x, C.c_float), _p(y, C.c_float), x.shape[0], metric))


def exact_search(base, queries, k: int, metric: int = L2):
    """Eq. 1: ids and distances of the k nearest base rows per query."""
    base, queries = _f32(base), _f32(queries)
    B = queries.shape[0]
    ids = np.empty((B, k), np.uint32)
    dists = np.empty((B, k), np.float32)
    _check(_load().oracle_exact_search(_p(base, C.c_float), base.shape[0], base.shape[1], metric,
                                       _p(queries, C.c_float), B, k,
                                       _p(ids, C.c_uint32), _p(dists, C.c_float)), "exact_search")
    return ids, dists


def recall(found_ids, true_ids) -> float:
    """Eq. 2 averaged over the batch: |found ∩ true| / |true| with sets per query."""
    found_ids, true_ids = np.asarray(found_ids), np.asarray(true_ids)
    hit = 0
    for f, t in zip(found_ids, true_ids):
        hit += len(set(int(v) for v in f if int(v) != INVALID_ID) & set(int(v) for v in t))
    return hit / float(true_ids.size)


def knn_graph(base, d_init: int, metric: int = L2, rows=None, return_dists: bool = False):
    base = _f32(base)
    N, dim = base.shape
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n = N if rows_a is None else rows_a.shape[0]
    g0 = np.empty((n, d_init), np.uint32)
    gd = np.empty((n, d_init), np.float32) if return_dists else None
    _check(_load().oracle_knn_graph(_p(base, C.c_float), N, dim, metric, _p(rows_a, C.c_int64), n,
                                    d_init, _p(g0, C.c_uint32), _p(gd, C.c_float)), "knn_graph")
    return (g0, gd) if return_dists else g0


def nn_descent(base, k: int, rounds: int, sample: int, metric: int = L2, seed: int = 0):
    """Approximate k-NN graph by NN-descent in synchronous rounds: (ids[N, k], dists[N, k]), rows sorted."""
    base = _f32(base)
    N = base.shape[0]
    ids = np.empty((N, k), np.uint32)
    dists = np.empty((N, k), np.float32)
    _check(_load().oracle_nn_descent(_p(base, C.c_float), N, base.shape[1], metric, k, rounds, sample, seed,
                                     _p(ids, C.c_uint32), _p(dists, C.c_float)), "nn_descent")
    return ids, dists


def detour_count(g0, rows=None):
    """Eq. 3 counts for every node, or for the listed nodes only (same values, fewer rows)."""
    g0 = _u32(g0)
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n = g0.shape[0] if rows_a is None else rows_a.shape[0]
    cnt = np.empty((n, g0.shape[1]), np.uint32)
    _check(_load().oracle_detour_count(_p(g0, C.c_uint32), g0.shape[0], g0.shape[1],
                                       _p(rows_a, C.c_int64), n, _p(cnt, C.c_uint32)), "detour_count")
    return cnt


def detour_count_distance(g0, g0_dist, rows=None):
    """Eq. 3 with the stored distances as weights (distance-based reordering)."""
    g0, g0_dist = _u32(g0), _f32(g0_dist)
    rows_a = None if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    n = g0.shape[0] if rows_a is None else rows_a.shape[0]
    cnt = np.empty((n, g0.shape[1]), np.uint32)
    _check(_load().oracle_detour_count_distance(_p(g0, C.c_uint32), _p(g0_dist, C.c_float), g0.shape[0],
                                                g0.shape[1], _p(rows_a, C.c_int64), n,
                                                _p(cnt, C.c_uint32)), "detour_count_distance")
    return cnt


def prune(g0, count, d: int):
    g0, count = _u32(g0), _u32(count)
    out = np.empty((g0.shape[0], d), np.uint32)
    _check(_load().oracle_prune(_p(g0, C.c_uint32), _p(count, C.c_uint32), g0.shape[0],
                                g0.shape[1], d, _p(out, C.c_uint32)), "prune")
    return out


def reverse(pruned):
    pruned = _u32(pruned)
    N, d = pruned.shape
    rev = np.full((N, d), INVALID_ID, np.uint32)
    rev_len = np.zeros(N, np.uint32)
    _check(_load().oracle_reverse(_p(pruned, C.c_uint32), N, d, _p(rev, C.c_uint32),
                                  _p(rev_len, C.c_uint32)), "reverse")
    return rev, rev_len


def merge(pruned, rev, rev_len):
    pruned, rev, rev_len = _u32(pruned), _u32(rev), _u32(rev_len)
    N, d = pruned.shape
    out = np.empty((N, d), np.uint32)
    _check(_load().oracle_merge(_p(pruned, C.c_uint32), _p(rev, C.c_uint32),
                                _p(rev_len, C.c_uint32), N, d, _p(out, C.c_uint32)), "merge")
    return out


RANK = 0       # reordering by ranks (what CAGRA adopts)
DISTANCE = 1   # reordering by the stored distances


def optimize(g0, d: int, g0_dist=None):
    """g0_dist given: distance-based reordering, else rank-based."""
    g0 = _u32(g0)
    gd = None if g0_dist is None else _f32(g0_dist)
    out = np.empty((g0.shape[0], d), np.uint32)
    _check(_load().oracle_optimize_ex(_p(g0, C.c_uint32), _p(gd, C.c_float), g0.shape[0], g0.shape[1], d,
                                      _p(out, C.c_uint32)), "optimize")
    return out


def build(base, degree: int, init_degree: int = 0, metric: int = L2, reorder: int = RANK):
    base = _f32(base)
    out = np.empty((base.shape[0], degree), np.uint32)
    _check(_load().oracle_build_ex(_p(base, C.c_float), base.shape[0], base.shape[1], metric, degree,
                                   init_degree, reorder, _p(out, C.c_uint32)), "build")
    return out


def two_hop_counts(graph) -> np.ndarray:
    """Sec. III-A: per node, the number of other nodes reachable in one or two steps."""
    graph = _u32(graph)
    out = np.empty(graph.shape[0], np.uint32)
    _check(_load().oracle_two_hop_counts(_p(graph, C.c_uint32), graph.shape[0], graph.shape[1],
                                         _p(out, C.c_uint32)), "two_hop_counts")
    return out


def strong_components(graph) -> int:
    graph = _u32(graph)
    n = int(_load().oracle_strong_components(_p(graph, C.c_uint32), graph.shape[0], graph.shape[1]))
    if n < 0:
        raise ValueError("oracle strong_components failed")
    return n


def weak_components(graph) -> int:
    graph = _u32(graph)
    n = int(_load().oracle_weak_components(_p(graph, C.c_uint32), graph.shape[0], graph.shape[1]))
    if n < 0:
        raise ValueError("oracle weak_components failed")
    return n


def splitmix_fin(z: int) -> int:
    return int(_load().oracle_splitmix_fin(C.c_uint64(z & 0xFFFFFFFFFFFFFFFF)))


def seed_id(seed: int, query: int, slot: int, N: int) -> int:
    return int(_load().oracle_seed_id(seed, query, slot, N))


def auto_max_iterations(itopk: int, search_width: int) -> int:
    return int(_load().oracle_auto_max_iterations(itopk, search_width))


def search(graph, base, queries, k: int, itopk: int, search_width: int = 1, metric: int = L2,
           seed: int = 0, max_iterations: int = 0, reset_interval: int = 0, n_threads: int = 0,
           return_stats: bool = False):
    """Single-CTA search.  stats columns: passes, parents, distances computed, hit I_max."""
    graph, base, queries = _u32(graph), _f32(base), _f32(queries)
    B = queries.shape[0]
    ids = np.empty((B, k), np.uint32)
    dists = np.empty((B, k), np.float32)
    stats = np.zeros((B, 4), np.uint32)
    _check(_load().oracle_search(_p(graph, C.c_uint32), base.shape[0], graph.shape[1],
                                 _p(base, C.c_float), base.shape[1], metric,
                                 _p(queries, C.c_float), B, k, itopk, search_width, seed,
                                 max_iterations, reset_interval, n_threads,
                                 _p(ids, C.c_uint32), _p(dists, C.c_float),
                                 _p(stats, C.c_uint32)), "search")
    return (ids, dists, stats) if return_stats else (ids, dists)


def search_multi(graph, base, queries, k: int, local_topk: int, n_workers: int, metric: int = L2,
                 seed: int = 0, max_iterations: int = 64, n_threads: int = 0,
                 return_stats: bool = False, return_lists: bool = False):
    """Multi-CTA search, workers simulated in lock step.  return_lists: also every worker's final
    list of ids, [B, n_workers, local_topk] (appended to the returned tuple)."""
    graph, base, queries = _u32(graph), _f32(base), _f32(queries)
    B = queries.shape[0]
    ids = np.empty((B, k), np.uint32)
    dists = np.empty((B, k), np.float32)
    stats = np.zeros((B, 4), np.uint32)
    if return_lists:
        lists = np.empty((B, n_workers, local_topk), np.uint32)
        _check(_load().oracle_search_multi_lists(_p(graph, C.c_uint32), base.shape[0], graph.shape[1],
                                                 _p(base, C.c_float), base.shape[1], metric,
                                                 _p(queries, C.c_float), B, k, local_topk, n_workers, seed,
                                                 max_iterations, n_threads, _p(ids, C.c_uint32),
                                                 _p(dists, C.c_float), _p(stats, C.c_uint32),
                                                 _p(lists, C.c_uint32)), "search_multi_lists")
        return (ids, dists, stats, lists) if return_stats else (ids, dists, lists)
    _check(_load().oracle_search_multi(_p(graph, C.c_uint32), base.shape[0], graph.shape[1],
                                       _p(base, C.c_float), base.shape[1], metric,
                                       _p(queries, C.c_float), B, k, local_topk, n_workers, seed,
                                       max_iterations, n_threads, _p(ids, C.c_uint32),
                                       _p(dists, C.c_float), _p(stats, C.c_uint32)),
           "search_multi")
    return (ids, dists, stats) if return_stats else (ids, dists)
