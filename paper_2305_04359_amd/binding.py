"""Thin ctypes binding of the C ABI in include/ann.h.

Argument marshalling only: every step of the path runs in the HIP kernels of libannmi.so.
PyTorch (ROCm) tensors serve as device allocations and give the current stream.  There is no
CPU fallback: if the library has not been built, loading fails with an error.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

NONE = 0xFFFFFFFF
U8, I8, F32 = 0, 1, 2
L2SQ, MIPS = 0, 1


class AnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"ann error {code}: {msg}")
        self.code = code


class BuildOpts(C.Structure):
    _fields_ = [
        ("batch_cap", C.c_uint64),
        ("start", C.c_uint32),
        ("use_start", C.c_uint32),
        ("order", C.c_void_p),
        ("visited_cap", C.c_uint32),
        ("spill_cap", C.c_uint64),
        ("hash_bits", C.c_uint32),
        ("max_rounds", C.c_uint64),
        ("collect_stats", C.c_uint32),
        ("alloc", C.c_void_p),
        ("free", C.c_void_p),
        ("alloc_user", C.c_void_p),
        ("step1_parts", C.c_uint32),
    ]


class GraphInfo(C.Structure):
    _fields_ = [("n", C.c_uint64), ("d", C.c_uint32), ("R", C.c_uint32), ("dtype", C.c_uint32),
                ("metric", C.c_uint32), ("start", C.c_uint32), ("rounds", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [(k, C.c_uint64) for k in ("searches", "hops", "evals", "prunes", "reprunes", "appends",
                                           "edges", "prune_evals", "redone", "restarts", "rounds", "passes", "survivors",
                                           "insert_hops")] + \
               [(k, C.c_double) for k in ("ms_search", "ms_prune", "ms_sort", "ms_merge", "ms_total")] + \
               [("search_launches", C.c_uint64), ("ms_search_launches", C.c_double)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class HnswOpts(C.Structure):
    _fields_ = [("batch_cap", C.c_uint64), ("order", C.c_void_p), ("level", C.c_void_p),
                ("max_rounds", C.c_uint64), ("collect_stats", C.c_uint32),
                ("alloc", C.c_void_p), ("free", C.c_void_p), ("alloc_user", C.c_void_p)]


class HnswInfo(C.Structure):
    _fields_ = [("n", C.c_uint64), ("d", C.c_uint32), ("m", C.c_uint32), ("dtype", C.c_uint32),
                ("metric", C.c_uint32), ("top", C.c_uint32), ("entry", C.c_uint32), ("rounds", C.c_uint64)]


EXPORTS = [
    "ann_build", "ann_insert_batch", "ann_insert_points", "ann_graph_reserve", "ann_search", "ann_search_eps", "ann_search_noalloc", "ann_start_vertex", "ann_graph_from_host",
    "ann_graph_copy_neighbors", "ann_graph_device_rows", "ann_graph_info", "ann_get_stats", "ann_graph_set_stats", "ann_graph_set_filter_bits",
    "ann_graph_free", "ann_sort_edges", "ann_last_error",
    "ann_hnsw_build", "ann_hnsw_insert_points", "ann_hnsw_from_host", "ann_hnsw_search", "ann_hnsw_info", "ann_hnsw_copy_levels", "ann_hnsw_layer_size",
    "ann_hnsw_copy_layer", "ann_hnsw_get_stats", "ann_hnsw_free",
    "ann_hcnng_build", "ann_hcnng_tree_edges", "ann_hcnng_leaf_knn",
]

_lib = None


def lib():
    """Load libannmi.so (built in-tree by build.build_library); raise if it is missing."""
    global _lib
    if _lib is None:
        path = _build.library_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} not found: run __graft_entry__.build() "
                              "(or paper_2305_04359_amd/build.py) first")
        # PyTorch ships its own HIP runtime (same SONAME as the one hipcc links against).  Load it
        # first so that this library binds to that copy: two runtimes in one process do not
        # share a device context.
        import torch  # noqa: F401
        L = C.CDLL(path)
        vp, u64, u32 = C.c_void_p, C.c_uint64, C.c_uint32
        L.ann_build.restype = C.c_int
        L.ann_build.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, u32, C.c_float, u64,
                                C.POINTER(BuildOpts), vp, C.POINTER(vp)]
        L.ann_insert_batch.restype = C.c_int
        L.ann_insert_batch.argtypes = [vp, vp, vp, u64, u32, C.c_float, vp]
        L.ann_insert_points.restype = C.c_int
        L.ann_insert_points.argtypes = [vp, vp, u64, u32, C.c_float, u64, C.POINTER(BuildOpts), vp]
        L.ann_graph_reserve.restype = C.c_int
        L.ann_graph_reserve.argtypes = [vp, u64, vp]
        L.ann_search.restype = C.c_int
        L.ann_search.argtypes = [vp, vp, vp, u64, u32, u32, vp, vp, vp]
        L.ann_search_eps.restype = C.c_int
        L.ann_search_eps.argtypes = [vp, vp, vp, u64, u32, u32, C.c_float, vp, vp, vp]
        L.ann_search_noalloc.restype = C.c_int
        L.ann_search_noalloc.argtypes = [vp, vp, vp, u64, u32, u32, C.c_float, vp, vp, vp]
        L.ann_start_vertex.restype = C.c_int
        L.ann_start_vertex.argtypes = [vp, u64, u32, C.c_int, vp, C.POINTER(u32)]
        L.ann_graph_from_host.restype = C.c_int
        L.ann_graph_from_host.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, u32, C.POINTER(vp)]
        L.ann_graph_copy_neighbors.restype = C.c_int
        L.ann_graph_copy_neighbors.argtypes = [vp, vp]
        L.ann_graph_device_rows.restype = vp
        L.ann_graph_device_rows.argtypes = [vp]
        L.ann_graph_info.restype = C.c_int
        L.ann_graph_info.argtypes = [vp, C.POINTER(GraphInfo)]
        L.ann_get_stats.restype = C.c_int
        L.ann_get_stats.argtypes = [vp, C.POINTER(Stats)]
        L.ann_graph_set_stats.restype = C.c_int
        L.ann_graph_set_stats.argtypes = [vp, C.c_int]
        L.ann_graph_set_filter_bits.restype = C.c_int
        L.ann_graph_set_filter_bits.argtypes = [vp, u32]
        L.ann_graph_free.restype = None
        L.ann_graph_free.argtypes = [vp]
        L.ann_sort_edges.restype = C.c_int
        L.ann_sort_edges.argtypes = [vp, u64, u32, vp]
        L.ann_hnsw_build.restype = C.c_int
        L.ann_hnsw_build.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, u32, C.c_float, u64,
                                     C.POINTER(HnswOpts), vp, C.POINTER(vp)]
        L.ann_hnsw_insert_points.restype = C.c_int
        L.ann_hnsw_insert_points.argtypes = [vp, vp, u64, u32, C.c_float, u64, C.POINTER(HnswOpts), vp]
        L.ann_hnsw_from_host.restype = C.c_int
        L.ann_hnsw_from_host.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, vp, u32, C.POINTER(vp), vp,
                                         C.POINTER(vp)]
        L.ann_hnsw_search.restype = C.c_int
        L.ann_hnsw_search.argtypes = [vp, vp, vp, u64, u32, u32, C.c_float, vp, vp, vp]
        L.ann_hnsw_info.restype = C.c_int
        L.ann_hnsw_info.argtypes = [vp, C.POINTER(HnswInfo)]
        L.ann_hnsw_copy_levels.restype = C.c_int
        L.ann_hnsw_copy_levels.argtypes = [vp, vp]
        L.ann_hnsw_layer_size.restype = C.c_int
        L.ann_hnsw_layer_size.argtypes = [vp, u32, C.POINTER(u64)]
        L.ann_hnsw_copy_layer.restype = C.c_int
        L.ann_hnsw_copy_layer.argtypes = [vp, u32, vp, vp]
        L.ann_hnsw_get_stats.restype = C.c_int
        L.ann_hnsw_get_stats.argtypes = [vp, u32, C.POINTER(Stats)]
        L.ann_hnsw_free.restype = None
        L.ann_hnsw_free.argtypes = [vp]
        L.ann_hcnng_build.restype = C.c_int
        L.ann_hcnng_build.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, u32, u32, u32, u32, C.c_float, u64, vp,
                                      C.POINTER(vp)]
        L.ann_hcnng_tree_edges.restype = C.c_int
        L.ann_hcnng_tree_edges.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, u32, u32, u64, u32, vp, vp, vp,
                                           C.POINTER(u64), vp, C.POINTER(u64)]
        L.ann_hcnng_leaf_knn.restype = C.c_int
        L.ann_hcnng_leaf_knn.argtypes = [vp, u64, u32, C.c_int, C.c_int, u32, u32, u64, u32, vp, vp, vp,
                                         C.POINTER(u64), vp, vp]
        L.ann_last_error.restype = C.c_char_p
        L.ann_last_error.argtypes = []
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise AnnError(rc, lib().ann_last_error().decode())


def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.uint8:
        return U8
    if t.dtype == torch.int8:
        return I8
    if t.dtype == torch.float32:
        return F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


ALLOC_FN = C.CFUNCTYPE(C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p)
FREE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_void_p)


class TorchAllocator:
    """The `alloc` / `free` callbacks of ann_build_opts / ann_hnsw_opts served by PyTorch's caching
    allocator, so that the graph and every scratch buffer of a call are PyTorch's memory.  One
    instance serves any number of calls; it must outlive every object built with it (the
    objects made by this module keep a reference)."""

    def __init__(self):
        torch = _torch()
        self.calls = 0
        self.bytes = 0
        self.live = 0

        def _alloc(nbytes, stream, user):
            try:
                p = torch.cuda.caching_allocator_alloc(int(nbytes), stream=int(stream or 0))
            except Exception:  # out of memory: the library reports ANN_ENOMEM
                return None
            self.calls += 1
            self.bytes += int(nbytes)
            self.live += 1
            return p

        def _free(ptr, user):
            try:
                torch.cuda.caching_allocator_delete(ptr)
                self.live -= 1
            except Exception:  # (interpreter shutting down: the process is about to end)
                pass

        self.alloc = ALLOC_FN(_alloc)
        self.free = FREE_FN(_free)

    def fill(self, opts):
        opts.alloc = C.cast(self.alloc, C.c_void_p)
        opts.free = C.cast(self.free, C.c_void_p)
        opts.alloc_user = None


_torch_allocator = None


def torch_allocator() -> TorchAllocator:
    """The shared TorchAllocator of this process."""
    global _torch_allocator
    if _torch_allocator is None:
        _torch_allocator = TorchAllocator()
    return _torch_allocator


def _use_allocator(opts, allocator):
    """Puts the callbacks of `allocator` into `opts`: "torch" = the process's TorchAllocator, None
    = the library's own hipMalloc / hipFree, or any object with a fill(opts) method."""
    if allocator is None:
        return None
    a = torch_allocator() if isinstance(allocator, str) and allocator == "torch" else allocator
    a.fill(opts)
    return a


def _dev2d(t, name):
    if not t.is_cuda or t.dim() != 2 or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous 2-D device tensor")
    return t


class Graph:
    """Owner of an ann_graph handle."""

    def __init__(self, handle, allocator=None):
        self._h = C.c_void_p(handle)
        self._allocator = allocator  # its callbacks are called when the graph is freed

    def close(self):
        if self._h:
            lib().ann_graph_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def info(self) -> GraphInfo:
        gi = GraphInfo()
        _check(lib().ann_graph_info(self._h, C.byref(gi)))
        return gi

    def stats(self) -> dict:
        st = Stats()
        _check(lib().ann_get_stats(self._h, C.byref(st)))
        return st.as_dict()

    def set_stats(self, on: bool) -> None:
        _check(lib().ann_graph_set_stats(self._h, 1 if on else 0))

    def set_filter_bits(self, hash_bits: int) -> None:
        _check(lib().ann_graph_set_filter_bits(self._h, int(hash_bits)))

    def neighbors(self) -> np.ndarray:
        gi = self.info()
        out = np.empty((gi.n, gi.R), np.uint32)
        _check(lib().ann_graph_copy_neighbors(self._h, out.ctypes.data_as(C.c_void_p)))
        return out


def ann_build(points, R, L, alpha, seed=1, metric=L2SQ, batch_cap=0, start=None, order=None,
              visited_cap=0, hash_bits=0, max_rounds=0, collect_stats=False, spill_cap=0,
              allocator="torch", step1_parts=0) -> Graph:
    """batchBuild of Alg. 3 over a device tensor of points (n x d; uint8, int8 or float32).
    The graph and the build's scratch are PyTorch's memory unless allocator=None."""
    points = _dev2d(points, "points")
    o = BuildOpts()
    al = _use_allocator(o, allocator)
    o.batch_cap = batch_cap
    o.step1_parts = step1_parts
    o.use_start = 0 if start is None else 1
    o.start = 0 if start is None else int(start)
    keep = None
    if order is not None:
        keep = np.ascontiguousarray(order, dtype=np.uint32)
        if keep.shape != (points.shape[0] - 1,):
            raise ValueError("order must hold n-1 ids")
        o.order = keep.ctypes.data
    o.visited_cap = visited_cap
    o.spill_cap = spill_cap
    o.hash_bits = hash_bits
    o.max_rounds = max_rounds
    o.collect_stats = 1 if collect_stats else 0
    h = C.c_void_p()
    _check(lib().ann_build(points.data_ptr(), points.shape[0], points.shape[1], _dtype_code(points),
                           int(metric), R, L, float(alpha), seed, C.byref(o), _stream_ptr(), C.byref(h)))
    return Graph(h.value, al)


def ann_insert_batch(graph: Graph, points, ids, L, alpha) -> None:
    points = _dev2d(points, "points")
    ids = np.ascontiguousarray(ids, dtype=np.uint32)
    _check(lib().ann_insert_batch(graph.handle, points.data_ptr(), ids.ctypes.data_as(C.c_void_p),
                                  ids.shape[0], L, float(alpha), _stream_ptr()))


def ann_insert_points(graph: Graph, points, L, alpha, seed=1, batch_cap=0, order=None, max_rounds=0) -> None:
    """Streams the rows of `points` beyond the graph's current size into the graph (BatchInsert of
    Alg. 3 on the continued schedule); `points` holds the old points first, then the new ones."""
    points = _dev2d(points, "points")
    o = BuildOpts()
    o.batch_cap = batch_cap
    o.max_rounds = max_rounds
    keep = None
    if order is not None:
        keep = np.ascontiguousarray(order, dtype=np.uint32)
        o.order = keep.ctypes.data
        if keep.shape != (points.shape[0] - graph.info().n,):
            raise ValueError("order must hold one id per new point")
    _check(lib().ann_insert_points(graph.handle, points.data_ptr(), points.shape[0], L, float(alpha), seed,
                                   C.byref(o), _stream_ptr()))


def ann_graph_reserve(graph: Graph, n_cap) -> None:
    _check(lib().ann_graph_reserve(graph.handle, int(n_cap), _stream_ptr()))


def ann_search_eps(graph: Graph, points, queries, k, L, eps, ids_out=None, dists_out=None):
    """greedySearch with the (1 + eps) pruning of Sec. 4.5; returns (ids, dists) device tensors."""
    return ann_search(graph, points, queries, k, L, ids_out, dists_out, eps=eps)


def ann_search(graph: Graph, points, queries, k, L, ids_out=None, dists_out=None, eps=None):
    """greedySearch of Alg. 1 for each row of `queries`; returns (ids, dists) device tensors.
    With `eps` the call goes to ann_search_eps."""
    torch = _torch()
    points = _dev2d(points, "points")
    queries = _dev2d(queries, "queries")
    if queries.dtype != points.dtype or queries.shape[1] != points.shape[1]:
        raise ValueError("queries must match points in dtype and dimension")
    nq = queries.shape[0]
    if ids_out is None:
        ids_out = torch.empty((nq, k), dtype=torch.int32, device=points.device)
    if dists_out is None:
        dists_out = torch.empty((nq, k), dtype=torch.float32 if points.dtype == torch.float32 else torch.int32,
                                device=points.device)
    if eps is None:
        _check(lib().ann_search(graph.handle, points.data_ptr(), queries.data_ptr(), nq, k, L,
                                ids_out.data_ptr(), dists_out.data_ptr(), _stream_ptr()))
    else:
        _check(lib().ann_search_eps(graph.handle, points.data_ptr(), queries.data_ptr(), nq, k, L, float(eps),
                                    ids_out.data_ptr(), dists_out.data_ptr(), _stream_ptr()))
    return ids_out, dists_out


def ann_search_noalloc(graph: Graph, points, queries, k, L, ids_out, dists_out, eps=-1.0) -> None:
    """ann_search / ann_search_eps without any allocation: the caller brings the outputs (nq x k
    int32 ids; int32 or float32 distances) and nothing is allocated here or in the library."""
    nq = queries.shape[0]
    _check(lib().ann_search_noalloc(graph.handle, points.data_ptr(), queries.data_ptr(), nq, k, L, float(eps),
                                    ids_out.data_ptr(), dists_out.data_ptr(), _stream_ptr()))


def ann_start_vertex(points) -> int:
    points = _dev2d(points, "points")
    s = C.c_uint32(0)
    _check(lib().ann_start_vertex(points.data_ptr(), points.shape[0], points.shape[1], _dtype_code(points),
                                  _stream_ptr(), C.byref(s)))
    return int(s.value)


def ann_graph_from_host(rows: np.ndarray, d: int, dtype: int, metric: int, start: int) -> Graph:
    rows = np.ascontiguousarray(rows, dtype=np.uint32)
    h = C.c_void_p()
    _check(lib().ann_graph_from_host(rows.ctypes.data_as(C.c_void_p), rows.shape[0], d, dtype, metric,
                                     rows.shape[1], start, C.byref(h)))
    return Graph(h.value)


def ann_sort_edges(keys, key_bits: int) -> None:
    """In-place stable sort of a device int64 tensor of edge keys by bits [32, 32+key_bits)."""
    if not keys.is_cuda or keys.dim() != 1 or not keys.is_contiguous() or keys.element_size() != 8:
        raise ValueError("keys must be a contiguous 1-D device tensor of 64-bit integers")
    _check(lib().ann_sort_edges(keys.data_ptr(), keys.shape[0], key_bits, _stream_ptr()))


class Hnsw:
    """Owner of an ann_hnsw handle."""

    def __init__(self, handle, allocator=None):
        self._h = C.c_void_p(handle)
        self._allocator = allocator  # its callbacks are called when the index is freed

    def close(self):
        if self._h:
            lib().ann_hnsw_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def info(self) -> HnswInfo:
        hi = HnswInfo()
        _check(lib().ann_hnsw_info(self._h, C.byref(hi)))
        return hi

    def levels(self) -> np.ndarray:
        out = np.empty(self.info().n, np.uint32)
        _check(lib().ann_hnsw_copy_levels(self._h, out.ctypes.data_as(C.c_void_p)))
        return out

    def layer(self, l):
        """(ids, rows) of layer l: the layer's point ids ascending and their adjacency rows."""
        hi = self.info()
        cnt = C.c_uint64(0)
        _check(lib().ann_hnsw_layer_size(self._h, l, C.byref(cnt)))
        ids = np.empty(cnt.value, np.uint32)
        rows = np.empty((cnt.value, 2 * hi.m if l == 0 else hi.m), np.uint32)
        _check(lib().ann_hnsw_copy_layer(self._h, l, ids.ctypes.data_as(C.c_void_p),
                                         rows.ctypes.data_as(C.c_void_p)))
        return ids, rows

    def stats(self, l=0) -> dict:
        st = Stats()
        _check(lib().ann_hnsw_get_stats(self._h, l, C.byref(st)))
        return st.as_dict()


def ann_hnsw_build(points, m, efc, alpha, seed=1, metric=L2SQ, batch_cap=0, order=None, level=None,
                   max_rounds=0, collect_stats=False, allocator="torch") -> Hnsw:
    """The layered index of Sec. 4.2 over a device tensor of points."""
    points = _dev2d(points, "points")
    o = HnswOpts()
    al = _use_allocator(o, allocator)
    o.batch_cap = batch_cap
    o.max_rounds = max_rounds
    o.collect_stats = 1 if collect_stats else 0
    keep = []
    if order is not None:
        a = np.ascontiguousarray(order, dtype=np.uint32)
        if a.shape != (points.shape[0] - 1,):
            raise ValueError("order must hold n-1 ids")
        keep.append(a)
        o.order = a.ctypes.data
    if level is not None:
        a = np.ascontiguousarray(level, dtype=np.uint32)
        if a.shape != (points.shape[0],):
            raise ValueError("level must hold n entries")
        keep.append(a)
        o.level = a.ctypes.data
    h = C.c_void_p()
    _check(lib().ann_hnsw_build(points.data_ptr(), points.shape[0], points.shape[1], _dtype_code(points),
                                int(metric), m, efc, float(alpha), seed, C.byref(o), _stream_ptr(), C.byref(h)))
    return Hnsw(h.value, al)


def ann_hnsw_insert_points(index: Hnsw, points, efc, alpha, seed=1, batch_cap=0, order=None, level=None,
                           max_rounds=0) -> None:
    """Streams the rows of `points` beyond the index's current size into the layered index."""
    points = _dev2d(points, "points")
    n_new = points.shape[0] - index.info().n
    o = HnswOpts()
    o.batch_cap = batch_cap
    o.max_rounds = max_rounds
    keep = []
    for name, arr in (("order", order), ("level", level)):
        if arr is not None:
            a = np.ascontiguousarray(arr, dtype=np.uint32)
            if a.shape != (n_new,):
                raise ValueError(f"{name} must hold one entry per new point")
            keep.append(a)
            setattr(o, name, a.ctypes.data)
    _check(lib().ann_hnsw_insert_points(index.handle, points.data_ptr(), points.shape[0], efc, float(alpha), seed,
                                        C.byref(o), _stream_ptr()))


def ann_hnsw_from_host(points, m, level, entry, layers, metric=L2SQ) -> Hnsw:
    """An index from host arrays: level (n), entry point, layers[l] = n x (2m if l == 0 else m)."""
    points = _dev2d(points, "points")
    n = points.shape[0]
    level = np.ascontiguousarray(level, dtype=np.uint32)
    layers = [np.ascontiguousarray(a, dtype=np.uint32) for a in layers]
    if level.shape != (n,):
        raise ValueError("level must hold n entries")
    for l, a in enumerate(layers):
        if a.shape != (n, 2 * m if l == 0 else m):
            raise ValueError(f"layer {l} has the wrong shape")
    ptrs = (C.c_void_p * len(layers))(*[a.ctypes.data for a in layers])
    h = C.c_void_p()
    if len(layers) != int(level.max()) + 1:
        raise ValueError("one array per layer, up to the highest level")
    _check(lib().ann_hnsw_from_host(points.data_ptr(), n, points.shape[1], _dtype_code(points), int(metric), m,
                                    level.ctypes.data_as(C.c_void_p), int(entry), ptrs, _stream_ptr(), C.byref(h)))
    return Hnsw(h.value)


def ann_hnsw_search(index: Hnsw, points, queries, k, L, eps=-1.0, ids_out=None, dists_out=None):
    torch = _torch()
    points = _dev2d(points, "points")
    queries = _dev2d(queries, "queries")
    if queries.dtype != points.dtype or queries.shape[1] != points.shape[1]:
        raise ValueError("queries must match points in dtype and dimension")
    nq = queries.shape[0]
    if ids_out is None:
        ids_out = torch.empty((nq, k), dtype=torch.int32, device=points.device)
    if dists_out is None:
        dists_out = torch.empty((nq, k), dtype=torch.float32 if points.dtype == torch.float32 else torch.int32,
                                device=points.device)
    _check(lib().ann_hnsw_search(index.handle, points.data_ptr(), queries.data_ptr(), nq, k, L, float(eps),
                                 ids_out.data_ptr(), dists_out.data_ptr(), _stream_ptr()))
    return ids_out, dists_out


def ann_hcnng_build(points, T, Ls, s, l, R, alpha, seed=1, metric=L2SQ) -> Graph:
    """The clustering-based builder of Sec. 4.3 over a device tensor of uint8 or int8 points."""
    points = _dev2d(points, "points")
    h = C.c_void_p()
    _check(lib().ann_hcnng_build(points.data_ptr(), points.shape[0], points.shape[1], _dtype_code(points),
                                 int(metric), T, Ls, s, l, R, float(alpha), seed, _stream_ptr(), C.byref(h)))
    return Graph(h.value)


def ann_hcnng_tree_edges(points, Ls, s, l, seed, tree, metric=L2SQ):
    """One cluster tree: (perm, leaf_off, pairs) as numpy arrays."""
    points = _dev2d(points, "points")
    n = points.shape[0]
    perm = np.empty(n, np.uint32)
    off = np.empty(n + 1, np.uint64)
    pairs = np.empty((n, 2), np.uint32)
    nl, npairs = C.c_uint64(0), C.c_uint64(0)
    _check(lib().ann_hcnng_tree_edges(points.data_ptr(), n, points.shape[1], _dtype_code(points), int(metric), Ls, s, l,
                                      seed,
                                      tree, _stream_ptr(), perm.ctypes.data_as(C.c_void_p),
                                      off.ctypes.data_as(C.c_void_p), C.byref(nl),
                                      pairs.ctypes.data_as(C.c_void_p), C.byref(npairs)))
    return perm, off[:nl.value + 1].astype(np.int64), pairs[:npairs.value].copy()


def ann_hcnng_leaf_knn(points, Ls, l, seed, tree, metric=L2SQ):
    """One cluster tree's leaves and every point's l nearest neighbours inside its leaf:
    (perm, leaf_off, knn_ids[n, l], knn_dists[n, l]); row i belongs to the point perm[i]."""
    points = _dev2d(points, "points")
    n = points.shape[0]
    perm = np.empty(n, np.uint32)
    off = np.empty(n + 1, np.uint64)
    ids = np.empty((n, l), np.uint32)
    dists = np.empty((n, l), np.float32 if _dtype_code(points) == F32 else np.int32)
    nl = C.c_uint64(0)
    _check(lib().ann_hcnng_leaf_knn(points.data_ptr(), n, points.shape[1], _dtype_code(points), int(metric), Ls, l, seed,
                                    tree, _stream_ptr(), perm.ctypes.data_as(C.c_void_p),
                                    off.ctypes.data_as(C.c_void_p), C.byref(nl), ids.ctypes.data_as(C.c_void_p),
                                    dists.ctypes.data_as(C.c_void_p)))
    return perm, off[:nl.value + 1].astype(np.int64), ids, dists
