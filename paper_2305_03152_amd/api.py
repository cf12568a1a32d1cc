"""Python binding of libspp.so: argument marshalling only.

Every step of the path runs in the HIP kernels behind the C interface (include/spp.h);
torch is used here for device memory and streams.  There is no CPU fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import atexit
import ctypes as C
import os
import sys
import threading
import weakref
from typing import List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspp.so")

SPP_MAX_L = 8
SPP_MAX_FANOUT = 64
SPP_SYNC = 0x1
SPP_VIP_INCLUDE_HOP0 = 0x2
SPP_GRAPH_IN_LISTS = 0x4
SPP_NO_JOIN = 0x8
SPP_HIT_BESIDE_MISS = 0x80
SPP_STORE_ORDER = 0x10
SPP_GRAPH_CHUNKED = 0x20
SPP_SAMPLE_GLOBAL_TABLE = 0x40
SPP_STATIC_GATHER_MAX_ROWS = 131072
SPP_T_VIP_TOTAL, SPP_T_VIP_HOP_FIRST, SPP_T_SAMPLE = 0, 1, 9
SPP_T_GATHER_HIT, SPP_T_GATHER_MISS, SPP_T_GATHER_CLASSIFY, SPP_T_COUNT = 10, 11, 12, 16

EXPORTS = [
    "spp_last_error", "spp_ctx_create", "spp_ctx_destroy", "spp_ctx_sync", "spp_graph_create",
    "spp_graph_destroy", "spp_vip_propagate", "spp_vip_last_hops", "spp_build_vip_cache", "spp_cache_destroy",
    "spp_cache_set_limit", "spp_cache_lookup", "spp_mfg_bound", "spp_sample_mfg", "spp_sample_mfg_multi",
    "spp_gather_features", "spp_gather_features_multi", "spp_gather_last_stats", "spp_gather_join", "spp_ctx_timing", "spp_ctx_times", "spp_ctx_time_stats", "spp_ctx_totals",
    "spp_build_local_store", "spp_local_store_destroy", "spp_local_store_set_limit", "spp_local_store_rank",
    "spp_gather_features_split", "spp_access_count", "spp_vip_propagate_general", "spp_sample_mfg_general",
    "spp_stream_rates", "spp_gather_features_static",
]


class SppError(RuntimeError):
    pass


class _MfgStruct(C.Structure):
    _fields_ = [
        ("n_nodes_cap", C.c_int64),
        ("n_edges_cap", C.c_int64 * SPP_MAX_L),
        ("d_node_ids", C.c_void_p),
        ("d_indptr", C.c_void_p * SPP_MAX_L),
        ("d_src", C.c_void_p * SPP_MAX_L),
        ("d_counts", C.c_void_p),
        ("n", C.c_int64 * (SPP_MAX_L + 1)),
        ("e", C.c_int64 * (SPP_MAX_L + 1)),
    ]


class _SampleItem(C.Structure):
    _fields_ = [("d_seeds", C.c_void_p), ("nseeds", C.c_int32), ("batch_index", C.c_uint64),
                ("io", C.POINTER(_MfgStruct))]


class _GatherList(C.Structure):
    _fields_ = [("d_node_ids", C.c_void_p), ("n", C.c_int64), ("d_n", C.c_void_p), ("d_out", C.c_void_p)]


class _IdList(C.Structure):
    _fields_ = [("d_ids", C.c_void_p), ("n", C.c_int64), ("d_n", C.c_void_p)]


class _GatherStats(C.Structure):
    _fields_ = [("n_local", C.c_int64), ("n_cache_hit", C.c_int64), ("n_miss", C.c_int64),
                ("miss_bytes", C.c_int64), ("n_local_host", C.c_int64), ("n_miss_shared", C.c_int64)]


_lib = None


def load_library():
    """Loads libspp.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise SppError(f"{LIB_PATH} is missing: build it with `python -m paper_2305_03152_amd.build` "
                       "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    lib.spp_last_error.restype = C.c_char_p
    for name in EXPORTS:
        getattr(lib, name)          # AttributeError if a declared symbol is not exported
    lib.spp_ctx_destroy.restype = None
    lib.spp_graph_destroy.restype = None
    lib.spp_cache_destroy.restype = None
    lib.spp_ctx_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_void_p]
    lib.spp_ctx_destroy.argtypes = [C.c_void_p]
    lib.spp_ctx_sync.argtypes = [C.c_void_p]
    lib.spp_graph_create.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_void_p, C.c_uint32,
                                     C.POINTER(C.c_void_p)]
    lib.spp_graph_destroy.argtypes = [C.c_void_p]
    lib.spp_vip_propagate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                      C.POINTER(C.c_int32), C.c_int32, C.c_void_p, C.c_void_p, C.c_uint32]
    lib.spp_vip_last_hops.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.c_int32]
    lib.spp_build_vip_cache.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32,
                                        C.c_double, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                        C.POINTER(C.c_int64), C.POINTER(C.c_void_p)]
    lib.spp_cache_destroy.argtypes = [C.c_void_p]
    lib.spp_cache_set_limit.argtypes = [C.c_void_p, C.c_int64]
    lib.spp_cache_lookup.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.spp_mfg_bound.argtypes = [C.c_int32, C.POINTER(C.c_int32), C.c_int32, C.c_int64,
                                  C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    lib.spp_sample_mfg.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32),
                                   C.c_int32, C.c_uint64, C.c_uint64, C.POINTER(_MfgStruct), C.c_uint32]
    lib.spp_sample_mfg_multi.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(_SampleItem), C.c_int32,
                                         C.POINTER(C.c_int32), C.c_int32, C.c_uint64, C.c_uint32]
    lib.spp_gather_features.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                        C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p,
                                        C.c_void_p, C.POINTER(_GatherStats), C.c_uint32]
    lib.spp_gather_features_static.argtypes = lib.spp_gather_features.argtypes
    lib.spp_gather_features_multi.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                              C.c_void_p, C.c_int32, C.c_int32, C.POINTER(_GatherList), C.c_int32,
                                              C.POINTER(_GatherStats), C.c_uint32]
    lib.spp_gather_last_stats.argtypes = [C.c_void_p, C.POINTER(_GatherStats)]
    lib.spp_local_store_destroy.restype = None
    lib.spp_build_local_store.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                          C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_int64),
                                          C.POINTER(C.c_void_p)]
    lib.spp_local_store_destroy.argtypes = [C.c_void_p]
    lib.spp_local_store_set_limit.argtypes = [C.c_void_p, C.c_int64]
    lib.spp_local_store_rank.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_void_p]
    lib.spp_gather_features_split.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64,
                                              C.c_void_p, C.c_int32, C.c_int32, C.POINTER(_GatherList), C.c_int32,
                                              C.POINTER(_GatherStats), C.c_uint32]
    lib.spp_access_count.argtypes = [C.c_void_p, C.POINTER(_IdList), C.c_int32, C.c_int64, C.c_void_p, C.c_uint32]
    lib.spp_vip_propagate_general.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.c_int32,
                                              C.c_void_p, C.c_void_p, C.c_uint32]
    lib.spp_sample_mfg_general.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_void_p), C.POINTER(_SampleItem),
                                           C.c_int32, C.c_int32, C.c_uint64, C.c_uint32]
    lib.spp_gather_join.argtypes = [C.c_void_p]
    lib.spp_ctx_timing.argtypes = [C.c_void_p, C.c_int]
    lib.spp_ctx_times.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int64)]
    lib.spp_ctx_time_stats.argtypes = [C.c_void_p, C.POINTER(C.c_float), C.POINTER(C.c_int64), C.POINTER(C.c_float),
                                       C.POINTER(C.c_float)]
    lib.spp_ctx_totals.argtypes = [C.c_void_p, C.POINTER(C.c_int64), C.c_int]
    lib.spp_stream_rates.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.POINTER(C.c_float)]
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise SppError(f"libspp error {rc}: {load_library().spp_last_error().decode()}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dev(t: torch.Tensor, dtype, name: str):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise SppError(f"{name} must be a contiguous {dtype} tensor on the GPU")
    return t


def _fan(fanouts: Sequence[int]):
    L = len(fanouts)
    return (C.c_int32 * L)(*[int(f) for f in fanouts]), L


# Lifetime rules of the handles (Context, Graph, Cache, LocalStore):
#  * every destroy call of the library is safe on its own: a graph, cache or local store keeps the
#    device it lives on, not the context it was built with, so it may be closed before or after the
#    context; closing twice, or closing a handle that was never created, does nothing;
#  * Context.close() closes the handles built with it first (they would otherwise outlive their
#    workspaces' owner and keep device memory until the collector finds them), then the context;
#  * at interpreter exit every handle still alive is closed by one atexit hook, children before
#    contexts, while the HIP runtime is still up; a __del__ that runs later, while the interpreter
#    is finalizing, makes no library call at all (the runtime's own teardown may already have run);
#  * a Context keeps a reference to the torch stream it was given, so the stream outlives it.
_live_lock = threading.Lock()
_live = weakref.WeakSet()           # every open handle object


class _Handle:
    """Shared close / __del__ behaviour of the four handle classes; `_destroy` names the C call."""
    _destroy = ""
    _h = None

    def _opened(self):
        with _live_lock:
            _live.add(self)

    def close(self):
        h, self._h = self._h, C.c_void_p()
        if h:
            with _live_lock:
                _live.discard(self)
            getattr(load_library(), self._destroy)(h)

    def __del__(self):
        if sys.is_finalizing():         # the atexit hook has closed what was open; make no call into a runtime
            return                      # that may be tearing down
        try:
            self.close()
        except Exception:
            pass


@atexit.register
def _close_all_handles():
    with _live_lock:
        objs = list(_live)
    for o in sorted(objs, key=lambda o: isinstance(o, Context)):     # children first, contexts last
        try:
            o.close()
        except Exception:
            pass


class Context(_Handle):
    """Owns the library context bound to a torch stream (default: the current stream)."""
    _destroy = "spp_ctx_destroy"

    def __init__(self, device: int = 0, stream: Optional[torch.cuda.Stream] = None):
        lib = load_library()
        if not torch.cuda.is_available():
            raise SppError("no GPU visible: the path has no CPU fallback")
        torch.cuda.set_device(device)
        self.device = device
        self.stream = stream if stream is not None else torch.cuda.current_stream(device)
        self._children = weakref.WeakSet()
        self._h = C.c_void_p()
        _check(lib.spp_ctx_create(C.byref(self._h), device, C.c_void_p(self.stream.cuda_stream)))
        self._opened()

    def _adopt(self, child):
        self._children.add(child)
        child._opened()

    def sync(self):
        _check(load_library().spp_ctx_sync(self._h))

    def timing(self, enable: bool = True):
        _check(load_library().spp_ctx_timing(self._h, int(enable)))

    def times(self):
        """(sum_ms, count) per SPP_T_* index since timing was enabled or last read; waits for the streams."""
        ms = (C.c_float * SPP_T_COUNT)()
        cnt = (C.c_int64 * SPP_T_COUNT)()
        _check(load_library().spp_ctx_times(self._h, ms, cnt))
        return list(ms), list(cnt)

    def time_stats(self):
        """(sum_ms, count, min_ms, median_ms) per SPP_T_* index, like times()."""
        ms, mn, med = (C.c_float * SPP_T_COUNT)(), (C.c_float * SPP_T_COUNT)(), (C.c_float * SPP_T_COUNT)()
        cnt = (C.c_int64 * SPP_T_COUNT)()
        _check(load_library().spp_ctx_time_stats(self._h, ms, cnt, mn, med))
        return list(ms), list(cnt), list(mn), list(med)

    def totals(self, reset: bool = False):
        """Running sums since the last reset: batches, |S_L|, edges, gather calls, local / cache / missed rows,
        local rows read from host memory (split local store)."""
        buf = (C.c_int64 * 16)()
        _check(load_library().spp_ctx_totals(self._h, buf, int(reset)))
        keys = ("batches", "n_nodes", "n_edges", "gather_calls", "n_local", "n_cache_hit", "n_miss", "n_local_host",
                "n_miss_shared")
        return dict(zip(keys, list(buf)))

    def close(self):
        for child in list(getattr(self, "_children", ())):
            child.close()
        super().close()


class Graph(_Handle):
    """G in CSR on the device: rowptr int64[N+1], col int32[M]; keeps the tensors alive."""
    _destroy = "spp_graph_destroy"

    def __init__(self, ctx: Context, rowptr: torch.Tensor, col: torch.Tensor, in_lists: bool = False,
                 chunked: bool = False):
        """in_lists: also build the transposed structure that vip_propagate needs; chunked: in the layout for
        graphs whose per-vertex vectors exceed the caches, whatever N is (default: above 2^23 vertices)."""
        self.ctx = ctx
        self.rowptr = _dev(rowptr, torch.int64, "rowptr")
        self.col = _dev(col, torch.int32, "col")
        self.N = rowptr.numel() - 1
        self.M = col.numel()
        self._h = C.c_void_p()
        flags = (SPP_GRAPH_IN_LISTS if in_lists else 0) | (SPP_GRAPH_CHUNKED if in_lists and chunked else 0)
        _check(load_library().spp_graph_create(ctx._h, self.N, self.M, _ptr(rowptr), _ptr(col), flags,
                                               C.byref(self._h)))
        ctx._adopt(self)


def vip_propagate(ctx: Context, graph: Graph, T: torch.Tensor, B: int, fanouts: Sequence[int],
                  per_hop: bool = False, include_hop0: bool = False, sync: bool = True):
    """Proposition 1.  Returns p_total fp32[N] (and p_hop fp32[L, N] when per_hop)."""
    T = _dev(T, torch.int32, "T")
    f, L = _fan(fanouts)
    p_total = torch.empty(graph.N, dtype=torch.float32, device=T.device)
    p_hop = torch.empty((L, graph.N), dtype=torch.float32, device=T.device) if per_hop else None
    flags = (SPP_SYNC if sync else 0) | (SPP_VIP_INCLUDE_HOP0 if include_hop0 else 0)
    _check(load_library().spp_vip_propagate(ctx._h, graph._h, _ptr(T), T.numel(), int(B), f, L, _ptr(p_total),
                                            _ptr(p_hop), flags))
    return (p_total, p_hop) if per_hop else p_total


def _tptrs(t, L: int, M: int):
    """Host array of L device pointers to fp32[M] transition probabilities (one tensor serves every hop)."""
    if isinstance(t, torch.Tensor):
        t = [t] * L
    if len(t) != L:
        raise SppError("one transition-probability tensor per hop is needed")
    for a in t:
        _dev(a, torch.float32, "t")
        if a.numel() != M:
            raise SppError("a transition-probability tensor must have one entry per edge")
    return (C.c_void_p * L)(*[a.data_ptr() for a in t]), list(t)


def vip_propagate_general(ctx: Context, graph: Graph, p0: torch.Tensor, t, L: int, per_hop: bool = False,
                          include_hop0: bool = False, sync: bool = True):
    """Proposition 1 with initial probabilities p0[N] and transition probabilities t[h][M] (aligned with col)."""
    p0 = _dev(p0, torch.float32, "p0")
    if p0.numel() != graph.N:
        raise SppError("p0 must hold N entries")
    tp, keep = _tptrs(t, L, graph.M)
    p_total = torch.empty(graph.N, dtype=torch.float32, device=p0.device)
    p_hop = torch.empty((L, graph.N), dtype=torch.float32, device=p0.device) if per_hop else None
    flags = (SPP_SYNC if sync else 0) | (SPP_VIP_INCLUDE_HOP0 if include_hop0 else 0)
    _check(load_library().spp_vip_propagate_general(ctx._h, graph._h, _ptr(p0), tp, L, _ptr(p_total), _ptr(p_hop), flags))
    del keep
    return (p_total, p_hop) if per_hop else p_total


def vip_last_hops(ctx: Context, L: int):
    """Per hop of the last vip_propagate: (pushed over a sparse frontier?, out-edges of the frontier)."""
    pushed = (C.c_int32 * L)()
    edges = (C.c_int64 * L)()
    _check(load_library().spp_vip_last_hops(ctx._h, pushed, edges, L))
    return [bool(x) for x in pushed], [int(x) for x in edges]


class Cache(_Handle):
    """Replica cache handle: ids in rank order (slot = rank) plus the library-owned table and rows."""
    _destroy = "spp_cache_destroy"

    def __init__(self, ctx, handle, ids, N, lo, hi, remote_keepalive):
        self.ctx, self._h, self.ids, self.N, self.lo, self.hi = ctx, handle, ids, N, lo, hi
        self._keep = remote_keepalive
        ctx._adopt(self)

    @property
    def n_cached(self) -> int:
        return int(self.ids.numel())

    def set_limit(self, n_slots: int):
        _check(load_library().spp_cache_set_limit(self._h, int(n_slots)))

    def lookup(self, ids: torch.Tensor) -> torch.Tensor:
        ids = _dev(ids, torch.int32, "ids")
        out = torch.empty_like(ids)
        _check(load_library().spp_cache_lookup(self.ctx._h, self._h, _ptr(ids), ids.numel(), _ptr(out)))
        return out


def _row_store(t: Optional[torch.Tensor], name: str):
    if t is None:
        return None
    if not t.is_contiguous() or t.dim() != 2:
        raise SppError(f"{name} must be a contiguous 2-D tensor")
    if not (t.is_cuda or t.is_pinned()):
        raise SppError(f"{name} must live in pinned host memory or on the GPU")
    return t


def build_vip_cache(ctx: Context, score: torch.Tensor, lo: int, hi: int, K: int, alpha: float,
                    remote: Optional[torch.Tensor], D: int, elem_bytes: int) -> Cache:
    """Top floor(alpha*N/K) remote vertices by (score desc, id asc); table built, rows copied once."""
    score = _dev(score, torch.float32, "score")
    N = score.numel()
    remote = _row_store(remote, "remote")
    cap = int(alpha * float(N) / K)          # floor for non-negative values; the library recomputes it
    ids = torch.empty(cap + 1, dtype=torch.int32, device=score.device)
    n_cached = C.c_int64(0)
    h = C.c_void_p()
    _check(load_library().spp_build_vip_cache(ctx._h, _ptr(score), N, int(lo), int(hi), int(K), float(alpha),
                                              _ptr(remote), int(D), int(elem_bytes), _ptr(ids),
                                              C.byref(n_cached), C.byref(h)))
    return Cache(ctx, h, ids[:n_cached.value], N, lo, hi, remote)


class LocalStore(_Handle):
    """The partition's own rows split by a score order: a device-resident prefix plus the caller's host array."""
    _destroy = "spp_local_store_destroy"

    def __init__(self, ctx, handle, n_device_rows, N, lo, hi, local_rows):
        self.ctx, self._h, self.n_device_rows, self.N, self.lo, self.hi = ctx, handle, n_device_rows, N, lo, hi
        self.local_rows = local_rows            # kept alive: the library reads it on the miss path
        ctx._adopt(self)

    def set_limit(self, n_rows: int):
        _check(load_library().spp_local_store_set_limit(self._h, int(n_rows)))

    def rank(self, ids: torch.Tensor) -> torch.Tensor:
        ids = _dev(ids, torch.int32, "ids")
        out = torch.empty_like(ids)
        _check(load_library().spp_local_store_rank(self.ctx._h, self._h, _ptr(ids), ids.numel(), _ptr(out)))
        return out


def build_local_store(ctx: Context, score: torch.Tensor, lo: int, hi: int, beta: float,
                      local_rows: torch.Tensor) -> LocalStore:
    """Rank the vertices of [lo, hi) by (score desc, id asc); rows of the first floor(beta*(hi-lo)) go to the GPU."""
    score = _dev(score, torch.float32, "score")
    local_rows = _row_store(local_rows, "local_rows")
    if local_rows.shape[0] != hi - lo:
        raise SppError("local_rows must hold hi - lo rows")
    n_rows = C.c_int64(0)
    h = C.c_void_p()
    _check(load_library().spp_build_local_store(ctx._h, _ptr(score), score.numel(), int(lo), int(hi), float(beta),
                                                _ptr(local_rows), int(local_rows.shape[1]),
                                                int(local_rows.element_size()), C.byref(n_rows), C.byref(h)))
    return LocalStore(ctx, h, n_rows.value, score.numel(), lo, hi, local_rows)


def access_count(ctx: Context, lists, N: int, count: Optional[torch.Tensor] = None, sync: bool = True) -> torch.Tensor:
    """count[v] += 1 for every id of every list; `lists` is a sequence of (ids, n, n_device or None).

    The counts (float32, one per vertex) are a score for build_vip_cache / build_local_store.
    """
    if count is None:
        count = torch.zeros(int(N), dtype=torch.float32, device=torch.device("cuda", ctx.device))
    count = _dev(count, torch.float32, "count")
    if count.numel() != int(N):
        raise SppError("count must hold N entries")
    arr = (_IdList * max(len(lists), 1))()
    for j, (ids, n, n_dev) in enumerate(lists):
        ids = _dev(ids, torch.int32, "ids")
        if int(n) > ids.numel():
            raise SppError(f"list {j}: n exceeds the id buffer")
        arr[j].d_ids = ids.data_ptr()
        arr[j].n = int(n)
        arr[j].d_n = n_dev.data_ptr() if n_dev is not None else None
    _check(load_library().spp_access_count(ctx._h, arr, len(lists), int(N), _ptr(count), SPP_SYNC if sync else 0))
    return count


def _stats_dict(st):
    return dict(n_local=st.n_local, n_cache_hit=st.n_cache_hit, n_miss=st.n_miss, miss_bytes=st.miss_bytes,
                n_local_host=st.n_local_host, n_miss_shared=st.n_miss_shared)


def mfg_bound(nseeds: int, fanouts: Sequence[int], N: int):
    f, L = _fan(fanouts)
    nb = (C.c_int64 * (L + 1))()
    eb = (C.c_int64 * (L + 1))()
    _check(load_library().spp_mfg_bound(int(nseeds), f, L, int(N), nb, eb))
    return list(nb), list(eb)


class MFGBuffers:
    """Caller-owned output buffers of sample_mfg, sized once from the bounds and reused."""

    def __init__(self, device, max_seeds: int, fanouts: Sequence[int], N: int, capacities=None):
        """Sized from the fanout bounds, or (capacities = (n_nodes_cap, [edge cap per hop])) as given: the
        sampler with transition probabilities has no bound of its own and checks these capacities."""
        if capacities is not None:
            ncap, ecaps = int(capacities[0]), [int(e) for e in capacities[1]]
            self.fanouts = ()
            self.L = len(ecaps)
            self.nb, self.eb = [ncap] * (self.L + 1), [0] + ecaps
        else:
            self.fanouts = tuple(int(f) for f in fanouts)
            self.L = len(self.fanouts)
            self.nb, self.eb = mfg_bound(max_seeds, self.fanouts, N)
        self.node_ids = torch.empty(max(self.nb[self.L], 1), dtype=torch.int32, device=device)
        self.indptr = [torch.empty(self.nb[h] + 1, dtype=torch.int32, device=device) for h in range(self.L)]
        self.src = [torch.empty(max(self.eb[h + 1], 1), dtype=torch.int32, device=device) for h in range(self.L)]
        self.counts = torch.zeros(2 * (SPP_MAX_L + 1), dtype=torch.int64, device=device)
        self.n: List[int] = [0] * (self.L + 1)
        self.e: List[int] = [0] * (self.L + 1)
        s = _MfgStruct()
        s.n_nodes_cap = self.node_ids.numel()
        s.d_node_ids = self.node_ids.data_ptr()
        s.d_counts = self.counts.data_ptr()
        for h in range(self.L):
            s.n_edges_cap[h] = self.src[h].numel()
            s.d_indptr[h] = self.indptr[h].data_ptr()
            s.d_src[h] = self.src[h].data_ptr()
        self._s = s

    @property
    def n_final_device(self) -> torch.Tensor:
        """Device view of |S_L| (for a gather that must not wait for the host)."""
        return self.counts[self.L:self.L + 1]


def sample_mfg(ctx: Context, graph: Graph, seeds: torch.Tensor, fanouts: Sequence[int], seed: int,
               batch_index: int, out: Optional[MFGBuffers] = None, sync: bool = True,
               global_table: bool = False) -> MFGBuffers:
    """Multi-hop fanout sampling into per-layer MFGs.  With sync the host counts out.n / out.e are filled."""
    seeds = _dev(seeds, torch.int32, "seeds")
    if out is None:
        out = MFGBuffers(seeds.device, seeds.numel(), fanouts, graph.N)
    f, L = _fan(fanouts)
    _check(load_library().spp_sample_mfg(ctx._h, graph._h, _ptr(seeds), seeds.numel(), f, L,
                                         C.c_uint64(int(seed) & (2**64 - 1)), C.c_uint64(int(batch_index) & (2**64 - 1)),
                                         C.byref(out._s),
                                         (SPP_SYNC if sync else 0) | (SPP_SAMPLE_GLOBAL_TABLE if global_table else 0)))
    if sync:
        out.n = [int(out._s.n[h]) for h in range(L + 1)]
        out.e = [int(out._s.e[h]) for h in range(L + 1)]
    return out


def sample_mfg_multi(ctx: Context, graph: Graph, items, fanouts: Sequence[int], seed: int, sync: bool = True,
                     global_table: bool = False):
    """Several minibatches sampled by one set of launches.

    `items` is a sequence of (seeds, batch_index, MFGBuffers); each MFGBuffers receives the result of
    its minibatch exactly as a single sample_mfg call would produce it.
    """
    f, L = _fan(fanouts)
    arr = (_SampleItem * max(len(items), 1))()
    for j, (seeds, batch_index, out) in enumerate(items):
        seeds = _dev(seeds, torch.int32, "seeds")
        arr[j].d_seeds = seeds.data_ptr()
        arr[j].nseeds = seeds.numel()
        arr[j].batch_index = int(batch_index) & (2**64 - 1)
        arr[j].io = C.pointer(out._s)
    _check(load_library().spp_sample_mfg_multi(ctx._h, graph._h, arr, len(items), f, L,
                                               C.c_uint64(int(seed) & (2**64 - 1)),
                                               (SPP_SYNC if sync else 0) | (SPP_SAMPLE_GLOBAL_TABLE if global_table else 0)))
    if sync:
        for _, _, out in items:
            out.n = [int(out._s.n[h]) for h in range(L + 1)]
            out.e = [int(out._s.e[h]) for h in range(L + 1)]
    return [out for _, _, out in items]


def sample_mfg_general(ctx: Context, graph: Graph, t, items, L: int, seed: int, sync: bool = True):
    """The sampler with given transition probabilities t[h][M]: a target takes every entry of its row
    independently with the entry's probability.  `items` as for sample_mfg_multi, with MFGBuffers built
    from capacities; raises when a minibatch exceeds them (sync only)."""
    tp, keep = _tptrs(t, L, graph.M)
    arr = (_SampleItem * max(len(items), 1))()
    for j, (seeds, batch_index, out) in enumerate(items):
        seeds = _dev(seeds, torch.int32, "seeds")
        if out.L != L:
            raise SppError("the buffers were built for another number of hops")
        arr[j].d_seeds = seeds.data_ptr()
        arr[j].nseeds = seeds.numel()
        arr[j].batch_index = int(batch_index) & (2**64 - 1)
        arr[j].io = C.pointer(out._s)
    _check(load_library().spp_sample_mfg_general(ctx._h, graph._h, tp, arr, len(items), L,
                                                 C.c_uint64(int(seed) & (2**64 - 1)), SPP_SYNC if sync else 0))
    del keep
    if sync:
        for _, _, out in items:
            out.n = [int(out._s.n[h]) for h in range(L + 1)]
            out.e = [int(out._s.e[h]) for h in range(L + 1)]
    return [out for _, _, out in items]


def gather_features(ctx: Context, cache: Optional[Cache], local: torch.Tensor, N: int, lo: int, hi: int,
                    remote: Optional[torch.Tensor], node_ids: torch.Tensor, n: Optional[int] = None,
                    n_device: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                    sync: bool = True, store_order: bool = False):
    """out[i,:] = row of node_ids[i] from the local shard, the cache, or the remote store on a miss.

    `local` is the partition's rows on the GPU, or a LocalStore (rows split between GPU and host).
    Returns (out, stats) where stats = dict(n_local, n_cache_hit, n_miss, miss_bytes, n_local_host) when sync,
    else None.
    """
    if isinstance(local, LocalStore):
        node_ids = _dev(node_ids, torch.int32, "node_ids")
        n = int(node_ids.numel() if n is None else n)
        rows = local.local_rows
        if out is None:
            out = torch.empty((n, rows.shape[1]), dtype=rows.dtype, device=node_ids.device)
        stats = gather_features_multi(ctx, cache, local, N, lo, hi, remote, [(node_ids, n, n_device, out)], sync=sync,
                                      store_order=store_order)
        return out, stats
    local = _row_store(local, "local")
    if not local.is_cuda:
        raise SppError("local must be on the GPU")
    remote = _row_store(remote, "remote")
    node_ids = _dev(node_ids, torch.int32, "node_ids")
    n = int(node_ids.numel() if n is None else n)
    D, eb = local.shape[1], local.element_size()
    if out is None:
        out = torch.empty((n, D), dtype=local.dtype, device=local.device)
    if out.shape[0] < n or out.shape[1] != D or not out.is_contiguous():
        raise SppError("out is too small or not contiguous")
    st = _GatherStats()
    _check(load_library().spp_gather_features(ctx._h, cache._h if cache is not None else None, _ptr(local),
                                              int(N), int(lo), int(hi), _ptr(remote), D, eb, _ptr(node_ids), n,
                                              _ptr(n_device), _ptr(out), C.byref(st),
                                              (SPP_SYNC if sync else 0) | (SPP_STORE_ORDER if store_order else 0)))
    return out, (_stats_dict(st) if sync else None)


def gather_features_static(ctx: Context, cache: Optional[Cache], local: torch.Tensor, N: int, lo: int, hi: int,
                           remote: Optional[torch.Tensor], node_ids: torch.Tensor, out: torch.Tensor,
                           n: Optional[int] = None, n_device: Optional[torch.Tensor] = None, sync: bool = True):
    """gather_features through the entry point that allocates nothing (the output is the caller's)."""
    local = _row_store(local, "local")
    remote = _row_store(remote, "remote")
    node_ids = _dev(node_ids, torch.int32, "node_ids")
    n = int(node_ids.numel() if n is None else n)
    D, eb = local.shape[1], local.element_size()
    if out.shape[0] < n or out.shape[1] != D or not out.is_contiguous() or out.dtype != local.dtype:
        raise SppError("out is too small, not contiguous or of another type")
    st = _GatherStats()
    _check(load_library().spp_gather_features_static(ctx._h, cache._h if cache is not None else None, _ptr(local),
                                                     int(N), int(lo), int(hi), _ptr(remote), D, eb, _ptr(node_ids), n,
                                                     _ptr(n_device), _ptr(out), C.byref(st), SPP_SYNC if sync else 0))
    return _stats_dict(st) if sync else None


def gather_features_multi(ctx: Context, cache: Optional[Cache], local: torch.Tensor, N: int, lo: int, hi: int,
                          remote: Optional[torch.Tensor], lists, sync: bool = True, join: bool = True,
                          store_order: bool = False, hit_beside_miss: bool = False):
    """One classification / hit copy / miss copy over several id lists.

    store_order: fetch the missed remote rows in the order of the remote store (same result; faster when the
    call misses an eighth or more of the store's rows).
    hit_beside_miss: in a loop of unjoined calls, start this call's miss copy before its hit copy (same result;
    the host link never idles, the hit copy shares the chip with the miss copy).

    `lists` is a sequence of (node_ids, n, n_device or None, out); returns the summed stats when sync.
    `local` is the partition's rows on the GPU, or a LocalStore (rows split between GPU and host).
    """
    store = local if isinstance(local, LocalStore) else None
    local = _row_store(store.local_rows if store is not None else local, "local")
    if store is None and not local.is_cuda:
        raise SppError("local must be on the GPU (or pass a LocalStore)")
    remote = _row_store(remote, "remote")
    D, eb = local.shape[1], local.element_size()
    arr = (_GatherList * max(len(lists), 1))()
    for j, (ids, n, n_dev, out) in enumerate(lists):
        ids = _dev(ids, torch.int32, "node_ids")
        if out.shape[0] < n or out.shape[1] != D or not out.is_contiguous() or out.dtype != local.dtype:
            raise SppError(f"out of list {j} is too small, not contiguous or of another type")
        arr[j].d_node_ids = ids.data_ptr()
        arr[j].n = int(n)
        arr[j].d_n = n_dev.data_ptr() if n_dev is not None else None
        arr[j].d_out = out.data_ptr()
    st = _GatherStats()
    flags = ((SPP_SYNC if sync else 0) | (0 if join else SPP_NO_JOIN) | (SPP_STORE_ORDER if store_order else 0) |
             (SPP_HIT_BESIDE_MISS if hit_beside_miss else 0))
    lib = load_library()
    if store is not None:
        _check(lib.spp_gather_features_split(ctx._h, cache._h if cache is not None else None, store._h,
                                             int(N), int(lo), int(hi), _ptr(remote), D, eb, arr, len(lists),
                                             C.byref(st), flags))
    else:
        _check(lib.spp_gather_features_multi(ctx._h, cache._h if cache is not None else None, _ptr(local),
                                             int(N), int(lo), int(hi), _ptr(remote), D, eb, arr, len(lists),
                                             C.byref(st), flags))
    return _stats_dict(st) if sync else None


def stream_rates(ctx: Context, nbytes: int = 1 << 30, reps: int = 10):
    """GB/s of the library's plain streaming kernels over two fresh buffers of `nbytes` bytes: read-only,
    copy (bytes read + bytes written), write-only."""
    dev = torch.device("cuda", ctx.device)
    a = torch.zeros(nbytes // 4, dtype=torch.int32, device=dev)
    b = torch.empty_like(a)
    out = (C.c_float * 3)()
    _check(load_library().spp_stream_rates(ctx._h, _ptr(a), _ptr(b), a.numel() * 4, int(reps), out))
    return {"read_only": round(out[0], 1), "copy_read_plus_write": round(out[1], 1), "write_only": round(out[2], 1)}


def gather_join(ctx: Context):
    """Make the context's stream wait for a miss copy left running by a gather called with join=False."""
    _check(load_library().spp_gather_join(ctx._h))


def gather_last_stats(ctx: Context):
    st = _GatherStats()
    _check(load_library().spp_gather_last_stats(ctx._h, C.byref(st)))
    return _stats_dict(st)
