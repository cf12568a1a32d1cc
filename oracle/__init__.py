"""CPU oracle of the per-partition data path: TEST INFRASTRUCTURE ONLY.

Thin ctypes marshalling around `oracle.c` (plain C, fp64, single thread).  Only the tests,
the smoke check and the benchmark's CPU-baseline leg may import this package; the HIP library
and its Python binding never do, and this package imports nothing of theirs.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile oracle.c with gcc (strict IEEE arithmetic: no fast-math, no contraction)."""
    src = os.path.join(_HERE, "oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _SO, src, "-lm"])
    return _SO


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = C.CDLL(_SO)
        _lib.orc_cache_select.restype = C.c_int64
        _lib.orc_cache_capacity.restype = C.c_int64
        _lib.orc_rand32.restype = C.c_uint32
        _lib.orc_local_capacity.restype = C.c_int64
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def vip(rowptr, col, T, B, fanouts, include_hop0=False, literal_product=False, verbose=False):
    """Proposition 1 in fp64.  Returns (p_total[N], p_hop[L, N]) as float64 arrays."""
    lib = _load()
    rowptr, col, T = _i64(rowptr), _i32(col), _i32(T)
    N = rowptr.size - 1
    f = _i32(fanouts)
    L = f.size
    p_hop = np.empty((L, N), dtype=np.float64)
    p_tot = np.empty(N, dtype=np.float64)
    rc = lib.orc_vip(C.c_int64(N), _p(rowptr), _p(col), _p(T), C.c_int64(T.size), C.c_int32(int(B)),
                     _p(f), C.c_int32(L), C.c_int(int(include_hop0)), C.c_int(int(literal_product)),
                     _p(p_hop), _p(p_tot), C.c_int(int(verbose)))
    if rc != 0:
        raise ValueError(f"orc_vip failed ({rc})")
    return p_tot, p_hop


def cache_capacity(N, K, alpha) -> int:
    return int(_load().orc_cache_capacity(C.c_int64(int(N)), C.c_int32(int(K)), C.c_double(float(alpha))))


def cache_select(score, lo, hi, K, alpha):
    """Ids of the cached remote vertices in rank order (slot = rank)."""
    lib = _load()
    score = np.ascontiguousarray(score, dtype=np.float32)
    N = score.size
    cap = cache_capacity(N, K, alpha)
    ids = np.empty(max(cap, 1), dtype=np.int32)
    n = lib.orc_cache_select(_p(score), C.c_int64(N), C.c_int64(int(lo)), C.c_int64(int(hi)),
                             C.c_int32(int(K)), C.c_double(float(alpha)), _p(ids))
    if n < 0:
        raise ValueError("orc_cache_select failed")
    return ids[:n].copy()


def philox4x32_10(ctr, key):
    lib = _load()
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib.orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def rand32(seed, batch, hop, vertex, slot) -> int:
    return int(_load().orc_rand32(C.c_uint64(int(seed)), C.c_uint64(int(batch)), C.c_uint32(int(hop)),
                                  C.c_uint32(int(vertex)), C.c_uint32(int(slot))))


def sample_positions(seed, batch, hop, vertex, d, f):
    lib = _load()
    pos = np.empty(max(int(f), int(min(d, f)), 1), dtype=np.int64)
    lib.orc_sample_positions.restype = C.c_int32
    c = lib.orc_sample_positions(C.c_uint64(int(seed)), C.c_uint64(int(batch)), C.c_uint32(int(hop)),
                                 C.c_uint32(int(vertex)), C.c_int64(int(d)), C.c_int32(int(f)), _p(pos))
    return pos[:c].copy()


def mfg_bound(nseeds, fanouts):
    """Upper bounds on |S_L| and on the edges of the largest hop: n_h <= n_{h-1} (1 + f_h)."""
    n, emax = int(nseeds), 0
    for f in fanouts:
        e = n * int(f)
        emax = max(emax, e)
        n = n + e
    return n, emax


class MFG:
    """node_ids = S_L; n[h] = |S_h|; indptr[h-1], src[h-1] describe hop h (targets S_{h-1}, sources S_h)."""
    __slots__ = ("node_ids", "n", "e", "indptr", "src")


def sample_mfg(rowptr, col, seeds, fanouts, seed, batch):
    lib = _load()
    rowptr, col, seeds, f = _i64(rowptr), _i32(col), _i32(seeds), _i32(fanouts)
    N, L = rowptr.size - 1, f.size
    node_cap, edge_cap = mfg_bound(seeds.size, f)
    node_cap = max(min(node_cap, N), seeds.size, 1)
    # per-hop capacities
    caps_n, caps_e, n = [], [], seeds.size
    for fh in f:
        caps_n.append(min(n, N))
        caps_e.append(max(min(n, N) * int(fh), 1))
        n = min(n * (1 + int(fh)), N)
    node_ids = np.empty(node_cap, dtype=np.int32)
    indptr = [np.empty(cn + 1, dtype=np.int32) for cn in caps_n]
    src = [np.empty(ce, dtype=np.int32) for ce in caps_e]
    ip_arr = (C.c_void_p * L)(*[a.ctypes.data for a in indptr])
    sp_arr = (C.c_void_p * L)(*[a.ctypes.data for a in src])
    n_out = np.zeros(L + 1, dtype=np.int64)
    e_out = np.zeros(L + 1, dtype=np.int64)
    rc = lib.orc_sample_mfg(C.c_int64(N), _p(rowptr), _p(col), _p(seeds), C.c_int32(seeds.size), _p(f),
                            C.c_int32(L), C.c_uint64(int(seed)), C.c_uint64(int(batch)),
                            C.c_int64(node_cap), C.c_int64(max(caps_e)), _p(node_ids), ip_arr, sp_arr,
                            _p(n_out), _p(e_out))
    if rc != 0:
        raise ValueError(f"orc_sample_mfg failed ({rc})")
    m = MFG()
    m.n = [int(x) for x in n_out]
    m.e = [int(x) for x in e_out]
    m.node_ids = node_ids[:m.n[L]].copy()
    m.indptr = [indptr[h][:m.n[h] + 1].copy() for h in range(L)]
    m.src = [src[h][:m.e[h + 1]].copy() for h in range(L)]
    return m


def gather(N, lo, hi, local, cache_rows, cache_ids, remote, node_ids):
    """out[i,:] = X[node_ids[i],:] from the three stores.  Arrays are 2-D, any fixed-size dtype.

    Returns (out, src_tag[int8: 0 local / 1 cache / 2 miss], (n_local, n_cache_hit, n_miss)).
    """
    lib = _load()
    local = np.ascontiguousarray(local)
    remote = np.ascontiguousarray(remote)
    row_bytes = local.shape[1] * local.dtype.itemsize
    cache_ids = _i32(cache_ids if cache_ids is not None else [])
    if cache_rows is None or cache_ids.size == 0:
        cache_rows = np.empty((1, local.shape[1]), dtype=local.dtype)
    cache_rows = np.ascontiguousarray(cache_rows)
    node_ids = _i32(node_ids)
    out = np.empty((node_ids.size, local.shape[1]), dtype=local.dtype)
    tag = np.empty(max(node_ids.size, 1), dtype=np.int8)
    counts = np.zeros(3, dtype=np.int64)
    rc = lib.orc_gather(C.c_int64(int(N)), C.c_int64(int(lo)), C.c_int64(int(hi)), _p(local), _p(cache_rows),
                        _p(cache_ids), C.c_int64(cache_ids.size), _p(remote), C.c_int64(row_bytes),
                        _p(node_ids), C.c_int64(node_ids.size), _p(out), _p(tag), _p(counts))
    if rc != 0:
        raise ValueError(f"orc_gather failed ({rc})")
    return out, tag[:node_ids.size], tuple(int(c) for c in counts)


def local_capacity(beta, n_local) -> int:
    """floor(beta * n_local): local rows kept in device memory."""
    return int(_load().orc_local_capacity(C.c_double(float(beta)), C.c_int64(int(n_local))))


def local_rank(score, lo, hi):
    """Order of the partition's own vertices [lo, hi) by (score descending, id ascending).

    Returns (rank[int32, hi-lo], order[int32, hi-lo]): rank[i] is the position of vertex lo+i,
    order[r] the local index at position r.
    """
    lib = _load()
    score = np.ascontiguousarray(score, dtype=np.float32)
    n = int(hi) - int(lo)
    rank = np.empty(max(n, 1), dtype=np.int32)
    order = np.empty(max(n, 1), dtype=np.int32)
    rc = lib.orc_local_rank(_p(score), C.c_int64(int(lo)), C.c_int64(int(hi)), _p(rank), _p(order))
    if rc != 0:
        raise MemoryError("orc_local_rank")
    return rank[:n], order[:n]


def gather_split(N, lo, hi, local_dev, local_host, rank, n_dev, cache_rows, cache_ids, remote, node_ids):
    """The gather with the local store split into a device prefix (rows in rank order) and the
    host array (all local rows in id order).

    Returns (out, src_tag[int8: 0 local device / 1 cache / 2 miss / 3 local host],
             (n_local_dev, n_cache_hit, n_miss, n_local_host)).
    """
    lib = _load()
    local_host = np.ascontiguousarray(local_host)
    remote = np.ascontiguousarray(remote)
    D = local_host.shape[1]
    row_bytes = D * local_host.dtype.itemsize
    if local_dev is None or int(n_dev) == 0:
        local_dev = np.empty((1, D), dtype=local_host.dtype)
    local_dev = np.ascontiguousarray(local_dev)
    cache_ids = _i32(cache_ids if cache_ids is not None else [])
    if cache_rows is None or cache_ids.size == 0:
        cache_rows = np.empty((1, D), dtype=local_host.dtype)
    cache_rows = np.ascontiguousarray(cache_rows)
    rank = _i32(rank)
    node_ids = _i32(node_ids)
    out = np.empty((node_ids.size, D), dtype=local_host.dtype)
    tag = np.empty(max(node_ids.size, 1), dtype=np.int8)
    counts = np.zeros(4, dtype=np.int64)
    rc = lib.orc_gather_split(C.c_int64(int(N)), C.c_int64(int(lo)), C.c_int64(int(hi)), _p(local_dev),
                              _p(local_host), _p(rank), C.c_int64(int(n_dev)), _p(cache_rows), _p(cache_ids),
                              C.c_int64(cache_ids.size), _p(remote), C.c_int64(row_bytes), _p(node_ids),
                              C.c_int64(node_ids.size), _p(out), _p(tag), _p(counts))
    if rc != 0:
        raise ValueError(f"orc_gather_split failed ({rc})")
    return out, tag[:node_ids.size], tuple(int(c) for c in counts)


def access_count(N, node_ids, count=None):
    """count[v] += 1 for every id of the list (float32 counts, exact below 2^24); returns count."""
    lib = _load()
    if count is None:
        count = np.zeros(int(N), dtype=np.float32)
    assert count.dtype == np.float32 and count.flags.c_contiguous and count.size == int(N)
    node_ids = _i32(node_ids)
    rc = lib.orc_access_count(C.c_int64(int(N)), _p(node_ids), C.c_int64(node_ids.size), _p(count))
    if rc != 0:
        raise ValueError("orc_access_count: id outside [0, N)")
    return count


def _tlist(t, L, M):
    """One float32[M] array per hop (a single array serves every hop)."""
    if isinstance(t, np.ndarray) and t.ndim == 1:
        t = [t] * L
    t = [np.ascontiguousarray(a, dtype=np.float32) for a in t]
    assert len(t) == L and all(a.size == M for a in t)
    return t


def vip_general(rowptr, col, p0, t, L, include_hop0=False):
    """Proposition 1 with given initial probabilities p0[N] and transition probabilities t[h][M]
    (aligned with col).  Returns (p_total[N], p_hop[L, N]) in float64."""
    lib = _load()
    rowptr, col = _i64(rowptr), _i32(col)
    N, M = rowptr.size - 1, col.size
    p0 = np.ascontiguousarray(p0, dtype=np.float32)
    t = _tlist(t, L, M)
    tp = (C.c_void_p * L)(*[a.ctypes.data for a in t])
    p_total = np.empty(N, dtype=np.float64)
    p_hop = np.empty((L, N), dtype=np.float64)
    rc = lib.orc_vip_general(C.c_int64(N), _p(rowptr), _p(col), _p(p0), tp, C.c_int32(L),
                             C.c_int(int(include_hop0)), _p(p_hop), _p(p_total))
    if rc != 0:
        raise ValueError(f"orc_vip_general failed ({rc})")
    return p_total, p_hop


def sample_mfg_general(rowptr, col, t, seeds, L, seed, batch):
    """Independent-inclusion sampler: target v takes col[e] with probability t[h][e].  Returns an MFG."""
    lib = _load()
    rowptr, col, seeds = _i64(rowptr), _i32(col), _i32(seeds)
    N, M = rowptr.size - 1, col.size
    t = _tlist(t, L, M)
    tp = (C.c_void_p * L)(*[a.ctypes.data for a in t])
    n_out = np.zeros(L + 1, dtype=np.int64)
    e_out = np.zeros(L + 1, dtype=np.int64)

    def call(node_cap, edge_cap, node_ids, ip_arr, sp_arr):
        rc = lib.orc_sample_mfg_general(C.c_int64(N), _p(rowptr), _p(col), tp, _p(seeds), C.c_int32(seeds.size),
                                        C.c_int32(L), C.c_uint64(int(seed)), C.c_uint64(int(batch)),
                                        C.c_int64(node_cap), C.c_int64(edge_cap), node_ids, ip_arr, sp_arr,
                                        _p(n_out), _p(e_out))
        if rc != 0:
            raise ValueError(f"orc_sample_mfg_general failed ({rc})")

    call(0, 0, None, None, None)                                   # sizes only
    n = [int(x) for x in n_out]
    e = [int(x) for x in e_out]
    node_ids = np.empty(max(n[L], 1), dtype=np.int32)
    indptr = [np.empty(n[h] + 1, dtype=np.int32) for h in range(L)]
    src = [np.empty(max(e[h + 1], 1), dtype=np.int32) for h in range(L)]
    ip_arr = (C.c_void_p * L)(*[a.ctypes.data for a in indptr])
    sp_arr = (C.c_void_p * L)(*[a.ctypes.data for a in src])
    call(n[L], max(max(e), 1), _p(node_ids), ip_arr, sp_arr)
    m = MFG()
    m.n, m.e = n, e
    m.node_ids = node_ids[:n[L]].copy()
    m.indptr = indptr
    m.src = [src[h][:e[h + 1]].copy() for h in range(L)]
    return m
