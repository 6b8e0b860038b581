"""ctypes access to the CPU oracle (vamana_oracle.c, hnsw_oracle.c, hcnng_oracle.c).

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's CPU
baseline leg may import this package; the HIP library and its Python binding
never do, and this package never imports them.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("vamana_oracle.c", "hnsw_oracle.c", "hcnng_oracle.c")]
_HDRS = [os.path.join(_HERE, f) for f in ("vamana_oracle.h", "hnsw_oracle.h", "hcnng_oracle.h")]
_LIB = os.path.join(_HERE, "libvamana_oracle.so")

NONE = 0xFFFFFFFF
U8, I8, F32 = 0, 1, 2
L2SQ, MIPS = 0, 1

_NP_DTYPE = {U8: np.uint8, I8: np.int8, F32: np.float32}


def dtype_code(arr: np.ndarray) -> int:
    if arr.dtype == np.uint8:
        return U8
    if arr.dtype == np.int8:
        return I8
    if arr.dtype == np.float32:
        return F32
    raise TypeError(f"unsupported dtype {arr.dtype}")


def build_oracle(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math, no contraction)."""
    stale = (
        force
        or not os.path.exists(_LIB)
        or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS + _HDRS)
    )
    if stale:
        cmd = [
            "gcc", "-std=c11", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
            "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, *_SRCS, "-lm",
        ]
        subprocess.run(cmd, check=True)
    return _LIB


class _Data(C.Structure):
    _fields_ = [
        ("points", C.c_void_p),
        ("n", C.c_uint64),
        ("d", C.c_uint32),
        ("dtype", C.c_int),
        ("metric", C.c_int),
    ]


class _Hnsw(C.Structure):
    _fields_ = [
        ("n", C.c_uint64),
        ("m", C.c_uint32),
        ("top", C.c_uint32),
        ("entry", C.c_uint32),
        ("level", C.POINTER(C.c_uint32)),
        ("rows", C.POINTER(C.POINTER(C.c_uint32))),
    ]


class HcnngStats(C.Structure):
    _fields_ = [("leaves", C.c_uint64), ("tree_edges", C.c_uint64), ("neighbours", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in (
        "searches", "hops", "evals", "prunes", "reprunes", "appends", "edges",
        "prune_cand", "prune_evals", "rounds")]

    def as_dict(self):
        return {k: int(getattr(self, k)) for k, _ in self._fields_}


_lib = None


def lib():
    global _lib
    if _lib is None:
        build_oracle()
        L = C.CDLL(_LIB)
        L.vo_distance.restype = C.c_double
        L.vo_distance.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_int, C.c_int]
        L.vo_greedy_search.restype = C.c_int
        L.vo_greedy_search.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint32,
            C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64), C.c_void_p,
            C.c_void_p, C.POINTER(Stats)]
        L.vo_greedy_search_eps.restype = C.c_int
        L.vo_greedy_search_eps.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint32,
            C.c_uint32, C.c_double, C.c_void_p, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64),
            C.c_void_p, C.c_void_p, C.POINTER(Stats)]
        L.vo_search_batch_eps.restype = C.c_int
        L.vo_search_batch_eps.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint64,
            C.c_uint32, C.c_uint32, C.c_double, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(Stats)]
        L.vo_prune.restype = C.c_uint32
        L.vo_prune.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64, C.c_uint32,
            C.c_double, C.c_void_p, C.POINTER(Stats)]
        L.vo_start_vertex.restype = C.c_uint32
        L.vo_start_vertex.argtypes = [C.POINTER(_Data)]
        L.vo_insertion_order.restype = None
        L.vo_insertion_order.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_void_p]
        L.vo_schedule.restype = C.c_uint64
        L.vo_schedule.argtypes = [C.c_uint64, C.c_uint64, C.c_void_p]
        L.vo_insert.restype = C.c_int
        L.vo_insert.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
            C.c_double, C.POINTER(Stats)]
        L.vo_batch_insert.restype = C.c_int
        L.vo_batch_insert.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint64,
            C.c_uint32, C.c_double, C.c_int, C.POINTER(Stats)]
        L.vo_build.restype = C.c_int
        L.vo_build.argtypes = [
            C.POINTER(_Data), C.c_uint32, C.c_uint32, C.c_double, C.c_uint64, C.c_uint64,
            C.c_uint32, C.c_void_p, C.c_uint64, C.c_int, C.c_void_p, C.POINTER(C.c_uint32),
            C.POINTER(Stats)]
        L.vo_insert_points.restype = C.c_int
        L.vo_insert_points.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint32,
            C.c_double, C.c_uint64, C.c_uint64, C.c_void_p, C.c_uint64, C.c_int, C.POINTER(Stats)]
        L.vo_new_points_order.restype = None
        L.vo_new_points_order.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_void_p]
        L.vo_schedule_from.restype = C.c_uint64
        L.vo_schedule_from.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, C.c_void_p]
        L.vo_build_sequential.restype = C.c_int
        L.vo_build_sequential.argtypes = [
            C.POINTER(_Data), C.c_uint32, C.c_uint32, C.c_double, C.c_uint32, C.c_void_p,
            C.c_uint64, C.c_void_p, C.POINTER(Stats)]
        L.vo_search_batch.restype = C.c_int
        L.vo_search_batch.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_uint64,
            C.c_uint32, C.c_uint32, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(Stats)]
        L.vo_brute_force.restype = C.c_int
        L.vo_brute_force.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint64, C.c_uint32, C.c_int, C.c_void_p,
            C.c_void_p]
        L.vo_batch_insert_from.restype = C.c_int
        L.vo_batch_insert_from.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64,
            C.c_uint32, C.c_double, C.c_int, C.c_void_p, C.POINTER(Stats)]
        L.vo_search_batch_from.restype = C.c_int
        L.vo_search_batch_from.argtypes = [
            C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p, C.c_uint64,
            C.c_uint32, C.c_uint32, C.c_double, C.c_int, C.c_void_p, C.c_void_p, C.POINTER(Stats)]
        L.vo_hnsw_level.restype = C.c_uint32
        L.vo_hnsw_level.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32]
        L.vo_hnsw_build.restype = C.c_int
        L.vo_hnsw_build.argtypes = [
            C.POINTER(_Data), C.c_uint32, C.c_uint32, C.c_double, C.c_uint64, C.c_uint64, C.c_void_p,
            C.c_void_p, C.c_uint64, C.c_int, C.POINTER(C.POINTER(_Hnsw)), C.POINTER(Stats)]
        L.vo_hnsw_insert_batch.restype = C.c_int
        L.vo_hnsw_insert_batch.argtypes = [
            C.POINTER(_Data), C.POINTER(_Hnsw), C.c_void_p, C.c_uint64, C.c_uint32, C.c_double, C.c_int,
            C.POINTER(Stats)]
        L.vo_hnsw_free.restype = None
        L.vo_hnsw_free.argtypes = [C.POINTER(_Hnsw)]
        L.vo_hnsw_search_batch.restype = C.c_int
        L.vo_hnsw_search_batch.argtypes = [
            C.POINTER(_Data), C.POINTER(_Hnsw), C.c_void_p, C.c_uint64, C.c_uint32, C.c_uint32,
            C.c_double, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Stats)]
        L.vo_hcnng_tree.restype = C.c_int
        L.vo_hcnng_tree.argtypes = [C.POINTER(_Data), C.c_uint32, C.c_uint64, C.c_uint32, C.c_void_p,
                                    C.c_void_p, C.POINTER(C.c_uint64)]
        L.vo_hcnng_leaf.restype = C.c_int
        L.vo_hcnng_leaf.argtypes = [C.POINTER(_Data), C.c_void_p, C.c_uint32, C.c_uint32, C.c_uint32,
                                    C.c_void_p, C.c_void_p, C.POINTER(C.c_uint64)]
        L.vo_hcnng_build.restype = C.c_int
        L.vo_hcnng_build.argtypes = [C.POINTER(_Data), C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32,
                                     C.c_uint32, C.c_double, C.c_uint64, C.c_int, C.c_void_p,
                                     C.POINTER(HcnngStats)]
        L.vo_threads.restype = C.c_int
        L.vo_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


@dataclass
class Dataset:
    """Row-major points plus metric, kept alive for the C struct."""
    points: np.ndarray
    metric: int = L2SQ

    def __post_init__(self):
        self.points = np.ascontiguousarray(self.points)
        assert self.points.ndim == 2
        self._c = _Data(self.points.ctypes.data, self.points.shape[0], self.points.shape[1],
                        dtype_code(self.points), int(self.metric))

    @property
    def n(self):
        return self.points.shape[0]

    @property
    def d(self):
        return self.points.shape[1]

    @property
    def dtype(self):
        return dtype_code(self.points)

    def c(self):
        return C.byref(self._c)


def distance(a: np.ndarray, b: np.ndarray, metric: int = L2SQ) -> float:
    a = np.ascontiguousarray(a)
    b = np.ascontiguousarray(b)
    assert a.dtype == b.dtype and a.shape == b.shape and a.ndim == 1
    return float(lib().vo_distance(_ptr(a), _ptr(b), a.shape[0], dtype_code(a), int(metric)))


def greedy_search(ds: Dataset, graph: np.ndarray, start: int, query: np.ndarray, L: int, k: int,
                  stats: Stats | None = None, check: bool = True, eps: float = -1.0):
    """Alg. 1, with the (1 + eps) rule of Sec. 4.5 when eps >= 0.
    Returns (V_ids, V_dists, K_ids, K_dists)."""
    graph = np.ascontiguousarray(graph, dtype=np.uint32)
    query = np.ascontiguousarray(query, dtype=ds.points.dtype)
    R = graph.shape[1]
    cap = ds.n
    v_ids = np.empty(cap, np.uint32)
    v_d = np.empty(cap, np.float64)
    k_ids = np.empty(k, np.uint32)
    k_d = np.empty(k, np.float64)
    nv = C.c_uint64(0)
    rc = lib().vo_greedy_search_eps(ds.c(), _ptr(graph), R, start, _ptr(query), L, k, float(eps),
                                    _ptr(v_ids), _ptr(v_d), cap, C.byref(nv), _ptr(k_ids), _ptr(k_d),
                                    C.byref(stats) if stats is not None else None)
    if check and rc != 0:
        raise RuntimeError(f"vo_greedy_search rc={rc}")
    n = nv.value
    return v_ids[:n].copy(), v_d[:n].copy(), k_ids, k_d


def prune(ds: Dataset, p_vec: np.ndarray, p_id: int, cand: np.ndarray, R: int, alpha: float,
          stats: Stats | None = None) -> np.ndarray:
    """prune(p, C, R) of Sec. 4.1; returns the selected ids in selection order."""
    cand = np.ascontiguousarray(cand, dtype=np.uint32)
    p_vec = np.ascontiguousarray(p_vec, dtype=ds.points.dtype)
    out = np.empty(R, np.uint32)
    cnt = lib().vo_prune(ds.c(), _ptr(p_vec), p_id, _ptr(cand), cand.shape[0], R, float(alpha),
                         _ptr(out), C.byref(stats) if stats is not None else None)
    return out[:cnt].copy()


def start_vertex(ds: Dataset) -> int:
    return int(lib().vo_start_vertex(ds.c()))


def insertion_order(n: int, start: int, seed: int) -> np.ndarray:
    order = np.empty(max(n - 1, 0), np.uint32)
    lib().vo_insertion_order(n, start, seed, _ptr(order))
    return order


def schedule(m: int, theta: int) -> np.ndarray:
    rounds = lib().vo_schedule(m, theta, None)
    bounds = np.empty(rounds + 1, np.uint64)
    lib().vo_schedule(m, theta, _ptr(bounds))
    return bounds


def empty_graph(n: int, R: int) -> np.ndarray:
    return np.full((n, R), NONE, np.uint32)


def insert(ds: Dataset, graph: np.ndarray, start: int, p: int, L: int, alpha: float,
           stats: Stats | None = None) -> None:
    assert graph.dtype == np.uint32 and graph.flags.c_contiguous
    rc = lib().vo_insert(ds.c(), _ptr(graph), graph.shape[1], start, p, L, float(alpha),
                         C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_insert rc={rc}")


def batch_insert(ds: Dataset, graph: np.ndarray, start: int, batch: np.ndarray, L: int,
                 alpha: float, threads: int = 1, stats: Stats | None = None) -> None:
    assert graph.dtype == np.uint32 and graph.flags.c_contiguous
    batch = np.ascontiguousarray(batch, dtype=np.uint32)
    rc = lib().vo_batch_insert(ds.c(), _ptr(graph), graph.shape[1], start, _ptr(batch),
                               batch.shape[0], L, float(alpha), threads,
                               C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_batch_insert rc={rc}")


def build(ds: Dataset, R: int, L: int, alpha: float, seed: int = 1, theta: int = 0,
          start: int | None = None, order: np.ndarray | None = None, max_rounds: int = 0,
          threads: int = 1, stats: Stats | None = None):
    """Alg. 3.  Returns (graph[n,R] uint32, start)."""
    graph = np.empty((ds.n, R), np.uint32)
    s_out = C.c_uint32(0)
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.uint32)
        assert order.shape[0] == ds.n - 1
    rc = lib().vo_build(ds.c(), R, L, float(alpha), seed, theta,
                        NONE if start is None else start,
                        _ptr(order) if order is not None else None, max_rounds, threads,
                        _ptr(graph), C.byref(s_out),
                        C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_build rc={rc}")
    return graph, int(s_out.value)


def new_points_order(first: int, count: int, seed: int) -> np.ndarray:
    order = np.empty(count, np.uint32)
    lib().vo_new_points_order(first, count, seed, _ptr(order))
    return order


def schedule_from(present: int, m: int, theta: int) -> np.ndarray:
    rounds = lib().vo_schedule_from(present, m, theta, None)
    bounds = np.empty(rounds + 1, np.uint64)
    lib().vo_schedule_from(present, m, theta, _ptr(bounds))
    return bounds


def insert_points(ds: Dataset, graph_old: np.ndarray, start: int, L: int, alpha: float,
                  seed: int = 1, theta: int = 0, order: np.ndarray | None = None,
                  max_rounds: int = 0, threads: int = 1, stats: Stats | None = None) -> np.ndarray:
    """Streams the points graph_old.shape[0]..ds.n-1 into the graph; returns the grown graph."""
    n_old, R = graph_old.shape
    assert graph_old.dtype == np.uint32 and n_old <= ds.n
    graph = np.full((ds.n, R), NONE, np.uint32)
    graph[:n_old] = graph_old
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.uint32)
        assert order.shape[0] == ds.n - n_old
    rc = lib().vo_insert_points(ds.c(), _ptr(graph), R, start, n_old, L, float(alpha), seed, theta,
                                _ptr(order) if order is not None else None, max_rounds, threads,
                                C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_insert_points rc={rc}")
    return graph


def build_sequential(ds: Dataset, R: int, L: int, alpha: float, start: int, order: np.ndarray,
                     stats: Stats | None = None) -> np.ndarray:
    graph = np.empty((ds.n, R), np.uint32)
    order = np.ascontiguousarray(order, dtype=np.uint32)
    rc = lib().vo_build_sequential(ds.c(), R, L, float(alpha), start, _ptr(order),
                                   order.shape[0], _ptr(graph),
                                   C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_build_sequential rc={rc}")
    return graph


def _dist_out(ds: Dataset, shape):
    return np.empty(shape, np.float32 if ds.dtype == F32 else np.int32)


def search_batch(ds: Dataset, graph: np.ndarray, start: int, queries: np.ndarray, k: int, L: int,
                 threads: int = 1, stats: Stats | None = None, eps: float = -1.0):
    graph = np.ascontiguousarray(graph, dtype=np.uint32)
    queries = np.ascontiguousarray(queries, dtype=ds.points.dtype)
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.uint32)
    dists = _dist_out(ds, (nq, k))
    rc = lib().vo_search_batch_eps(ds.c(), _ptr(graph), graph.shape[1], start, _ptr(queries), nq, k,
                                   L, float(eps), threads, _ptr(ids), _ptr(dists),
                                   C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_search_batch rc={rc}")
    return ids, dists


def brute_force(ds: Dataset, queries: np.ndarray, k: int, threads: int = 0):
    queries = np.ascontiguousarray(queries, dtype=ds.points.dtype)
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.uint32)
    dists = _dist_out(ds, (nq, k))
    rc = lib().vo_brute_force(ds.c(), _ptr(queries), nq, k, threads, _ptr(ids), _ptr(dists))
    if rc:
        raise RuntimeError(f"vo_brute_force rc={rc}")
    return ids, dists


def threads(t: int = 0) -> int:
    return int(lib().vo_threads(t))


# ---------------------------------------------------------------------------------------------
# layered index (hnsw_oracle.c)
# ---------------------------------------------------------------------------------------------
def batch_insert_from(ds: Dataset, graph: np.ndarray, starts: np.ndarray, batch: np.ndarray, L: int,
                      alpha: float, threads: int = 1, stats: Stats | None = None) -> np.ndarray:
    """BatchInsert with one start vertex per batch point; returns, per point, the closest
    vertex its search visited."""
    assert graph.dtype == np.uint32 and graph.flags.c_contiguous
    batch = np.ascontiguousarray(batch, dtype=np.uint32)
    starts = np.ascontiguousarray(starts, dtype=np.uint32)
    assert starts.shape == batch.shape
    near = np.empty(batch.shape[0], np.uint32)
    rc = lib().vo_batch_insert_from(ds.c(), _ptr(graph), graph.shape[1], 0, _ptr(starts), _ptr(batch),
                                    batch.shape[0], L, float(alpha), threads, _ptr(near),
                                    C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_batch_insert_from rc={rc}")
    return near


def search_batch_from(ds: Dataset, graph: np.ndarray, starts: np.ndarray, queries: np.ndarray, k: int,
                      L: int, eps: float = -1.0, threads: int = 1, stats: Stats | None = None):
    queries = np.ascontiguousarray(queries)
    starts = np.ascontiguousarray(starts, dtype=np.uint32)
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.uint32)
    dists = _dist_out(ds, (nq, k))
    rc = lib().vo_search_batch_from(ds.c(), _ptr(graph), graph.shape[1], 0, _ptr(starts), _ptr(queries),
                                    nq, k, L, float(eps), threads, _ptr(ids), _ptr(dists),
                                    C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_search_batch_from rc={rc}")
    return ids, dists


def hnsw_level(seed: int, i: int, m: int) -> int:
    return int(lib().vo_hnsw_level(seed, i, m))


class Hnsw:
    """A layered index: `level` (n), `layers[l]` = n x (2m if l == 0 else m) rows of global ids,
    `entry`, `m`.  Either built by the oracle or put together by hand (for pins of the search)."""

    def __init__(self, m: int, level: np.ndarray, layers: list, entry: int):
        self.m = int(m)
        self.level = np.ascontiguousarray(level, dtype=np.uint32)
        self.layers = [np.ascontiguousarray(a, dtype=np.uint32) for a in layers]
        self.entry = int(entry)
        for l, a in enumerate(self.layers):
            assert a.shape == (self.level.shape[0], 2 * self.m if l == 0 else self.m)

    @property
    def top(self):
        return len(self.layers) - 1

    def c(self):
        arr = (C.POINTER(C.c_uint32) * len(self.layers))(
            *[a.ctypes.data_as(C.POINTER(C.c_uint32)) for a in self.layers])
        self._keep = arr
        return _Hnsw(self.level.shape[0], self.m, self.top, self.entry,
                     self.level.ctypes.data_as(C.POINTER(C.c_uint32)), arr)


def hnsw_build(ds: Dataset, m: int, efc: int, alpha: float, seed: int = 1, theta: int = 0,
               level: np.ndarray | None = None, order: np.ndarray | None = None, max_rounds: int = 0,
               threads: int = 1, stats: Stats | None = None) -> Hnsw:
    if level is not None:
        level = np.ascontiguousarray(level, dtype=np.uint32)
        assert level.shape == (ds.n,)
    if order is not None:
        order = np.ascontiguousarray(order, dtype=np.uint32)
        assert order.shape == (ds.n - 1,)
    hp = C.POINTER(_Hnsw)()
    rc = lib().vo_hnsw_build(ds.c(), m, efc, float(alpha), seed, theta,
                             _ptr(level) if level is not None else None,
                             _ptr(order) if order is not None else None, max_rounds, threads,
                             C.byref(hp), C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_hnsw_build rc={rc}")
    h = hp.contents
    n = int(h.n)
    lev = np.ctypeslib.as_array(h.level, shape=(n,)).copy()
    layers = [np.ctypeslib.as_array(h.rows[l], shape=(n, 2 * m if l == 0 else m)).copy()
              for l in range(int(h.top) + 1)]
    out = Hnsw(m, lev, layers, int(h.entry))
    lib().vo_hnsw_free(hp)
    return out


def hnsw_insert_batch(ds: Dataset, h: Hnsw, batch: np.ndarray, efc: int, alpha: float, threads: int = 1,
                      stats: Stats | None = None) -> None:
    """One batch into an existing index (its layer arrays are modified in place)."""
    batch = np.ascontiguousarray(batch, dtype=np.uint32)
    hc = h.c()
    rc = lib().vo_hnsw_insert_batch(ds.c(), C.byref(hc), _ptr(batch), batch.shape[0], efc, float(alpha),
                                    threads, C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_hnsw_insert_batch rc={rc}")


def hnsw_insert_points(ds: Dataset, h: Hnsw, efc: int, alpha: float, seed: int = 1, level_seed: int = 1,
                       theta: int = 0, order: np.ndarray | None = None, level: np.ndarray | None = None,
                       max_rounds: int = 0, threads: int = 1) -> Hnsw:
    """Streams the points h.n .. ds.n-1 into the index: levels by the index's rule (or given),
    capped at its highest layer; order and batches as insert_points; one hnsw_insert_batch per
    batch.  Returns the grown index."""
    n_old, n = h.level.shape[0], ds.n
    m_new = n - n_old
    if level is None:
        level = np.array([hnsw_level(level_seed, i, h.m) for i in range(n_old, n)], np.uint32)
    level = np.minimum(np.asarray(level, np.uint32), h.top).astype(np.uint32)
    layers = []
    for l, a in enumerate(h.layers):
        b = np.full((n, a.shape[1]), NONE, np.uint32)
        b[:n_old] = a
        layers.append(b)
    out = Hnsw(h.m, np.concatenate([h.level, level]), layers, h.entry)
    if order is None:
        order = new_points_order(n_old, m_new, seed)
    order = np.ascontiguousarray(order, dtype=np.uint32)
    assert sorted(order.tolist()) == list(range(n_old, n))
    bounds = schedule_from(n_old - 1, m_new, theta if theta else max(1, n // 50)).astype(np.int64)
    for r in range(len(bounds) - 1):
        if max_rounds and r >= max_rounds:
            break
        hnsw_insert_batch(ds, out, order[bounds[r]:bounds[r + 1]], efc, alpha, threads=threads)
    return out


def hnsw_search_batch(ds: Dataset, h: Hnsw, queries: np.ndarray, k: int, L: int, eps: float = -1.0,
                      threads: int = 1, stats: Stats | None = None):
    """Returns (ids, dists, layer-0 start vertex of every query)."""
    queries = np.ascontiguousarray(queries)
    nq = queries.shape[0]
    ids = np.empty((nq, k), np.uint32)
    dists = _dist_out(ds, (nq, k))
    entry = np.empty(nq, np.uint32)
    hc = h.c()
    rc = lib().vo_hnsw_search_batch(ds.c(), C.byref(hc), _ptr(queries), nq, k, L, float(eps), threads,
                                    _ptr(ids), _ptr(dists), _ptr(entry),
                                    C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_hnsw_search_batch rc={rc}")
    return ids, dists, entry


# ---------------------------------------------------------------------------------------------
# clustering-based builder (hcnng_oracle.c)
# ---------------------------------------------------------------------------------------------
def hcnng_tree(ds: Dataset, Ls: int, seed: int, tree: int):
    """One cluster tree: (perm, leaf_off): the point ids leaf after leaf and the leaf boundaries."""
    perm = np.empty(ds.n, np.uint32)
    off = np.empty(ds.n + 1, np.uint64)
    nl = C.c_uint64(0)
    rc = lib().vo_hcnng_tree(ds.c(), Ls, seed, tree, _ptr(perm), _ptr(off), C.byref(nl))
    if rc:
        raise RuntimeError(f"vo_hcnng_tree rc={rc}")
    return perm, off[:nl.value + 1].astype(np.int64)


def hcnng_leaf(ds: Dataset, ids: np.ndarray, s: int, l: int) -> np.ndarray:
    """The degree-bounded tree of one leaf: accepted pairs (u < v) in acceptance order."""
    ids = np.ascontiguousarray(ids, dtype=np.uint32)
    cnt = ids.shape[0]
    eu = np.empty(max(cnt - 1, 1), np.uint32)
    ev = np.empty(max(cnt - 1, 1), np.uint32)
    ne = C.c_uint64(0)
    rc = lib().vo_hcnng_leaf(ds.c(), _ptr(ids), cnt, s, l, _ptr(eu), _ptr(ev), C.byref(ne))
    if rc:
        raise RuntimeError(f"vo_hcnng_leaf rc={rc}")
    return np.stack([eu[:ne.value], ev[:ne.value]], axis=1)


def hcnng_build(ds: Dataset, T: int, Ls: int, s: int, l: int, R: int, alpha: float, seed: int = 1,
                threads: int = 1, stats: HcnngStats | None = None) -> np.ndarray:
    graph = np.empty((ds.n, R), np.uint32)
    rc = lib().vo_hcnng_build(ds.c(), T, Ls, s, l, R, float(alpha), seed, threads, _ptr(graph),
                              C.byref(stats) if stats is not None else None)
    if rc:
        raise RuntimeError(f"vo_hcnng_build rc={rc}")
    return graph
