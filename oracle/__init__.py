"""ctypes front end of the CPU oracle -- TEST INFRASTRUCTURE, not product code.

Only tests, ``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline`` leg
import this package.  It loads ``libivf_oracle.so`` (built from ``ivf_oracle.c``
by ``python -m oracle.build``) and marshals numpy arrays; every number it
returns is computed by the C code in double precision.  Nothing here imports or
calls the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

IP = 0
L2 = 1

_lib = None


def lib():
    global _lib
    if _lib is None:
        from . import build as _build
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build()
        L = C.CDLL(path)
        vp, i32, i64 = C.c_void_p, C.c_int, C.c_int64
        L.orc_index_new.restype = vp
        L.orc_index_new.argtypes = [vp, i32, i32, i32]
        L.orc_index_free.restype = None
        L.orc_index_free.argtypes = [vp]
        L.orc_assign.argtypes = [vp, vp, i64, vp]
        L.orc_build.argtypes = [vp, vp, vp, i64]
        L.orc_insert.argtypes = [vp, vp, vp, i64, vp, vp]
        L.orc_ntotal.restype = i64
        L.orc_ntotal.argtypes = [vp]
        L.orc_split.argtypes = [vp, i64, i32]
        L.orc_nlist.argtypes = [vp]
        L.orc_centroids.argtypes = [vp, vp]
        L.orc_delete.restype = i64
        L.orc_delete.argtypes = [vp, vp, i64]
        L.orc_list_lengths.argtypes = [vp, vp]
        L.orc_list_ids.restype = i64
        L.orc_list_ids.argtypes = [vp, i32, vp, i64]
        L.orc_coarse.argtypes = [vp, vp, i64, i32, vp, vp]
        L.orc_scan_probes.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        L.orc_search.argtypes = [vp, vp, i64, i32, i32, vp, vp]
        L.orc_search_multi.argtypes = [vp, i32, vp, vp, i32, i32, vp, vp]
        L.orc_bruteforce.argtypes = [vp, vp, i64, i32, i32, vp, i64, i32, vp, vp]
        L.orc_union_probes.argtypes = [vp, i32, vp, i64, i32, i32, vp, vp, vp, vp]
        L.orc_search_union.argtypes = [vp, i32, vp, i64, i32, i32, vp, vp, vp]
        L.orc_pair_values.argtypes = [vp, vp, i64, i32, i32, vp]
        L.orc_kmeans.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp]
        L.orc_num_threads.restype = i32
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().orc_num_threads())


class Index:
    """One agent's IVF index held by the oracle (lists of (id, vector))."""

    def __init__(self, centroids, metric: int):
        c = _f32(centroids)
        assert c.ndim == 2
        self.nlist, self.d = int(c.shape[0]), int(c.shape[1])
        self.metric = int(metric)
        self._h = lib().orc_index_new(_ptr(c), self.nlist, self.d, self.metric)
        if not self._h:
            raise ValueError("orc_index_new failed")
        self._keep = []  # base arrays the C side points into

    def __del__(self):
        h, self._h = getattr(self, "_h", None), None
        if h and _lib is not None:
            _lib.orc_index_free(h)

    def assign(self, x):
        x = _f32(x).reshape(-1, self.d)
        out = np.empty(x.shape[0], dtype=np.int32)
        assert lib().orc_assign(self._h, _ptr(x), x.shape[0], _ptr(out)) == 0
        return out

    def build(self, x, ids=None):
        x = _f32(x).reshape(-1, self.d)
        self._keep.append(x)
        if ids is not None:
            ids = np.ascontiguousarray(ids, dtype=np.int64)
            assert ids.shape[0] == x.shape[0]
        assert lib().orc_build(self._h, _ptr(x), _ptr(ids), x.shape[0]) == 0

    def insert(self, x, ids=None, forced_lists=None):
        x = _f32(x).reshape(-1, self.d)
        m = x.shape[0]
        if ids is not None:
            ids = np.ascontiguousarray(ids, dtype=np.int64)
        if forced_lists is not None:
            forced_lists = np.ascontiguousarray(forced_lists, dtype=np.int32)
        out = np.empty(m, dtype=np.int32)
        rc = lib().orc_insert(self._h, _ptr(x), _ptr(ids), m, _ptr(forced_lists), _ptr(out))
        assert rc == 0
        return out

    def split(self, threshold: int, iters: int) -> int:
        """IVF-Split: lists longer than threshold are split by a 2-means; returns the number of splits."""
        n = int(lib().orc_split(self._h, int(threshold), int(iters)))
        assert n >= 0
        self.nlist = int(lib().orc_nlist(self._h))
        return n

    def centroids(self):
        out = np.empty((self.nlist, self.d), dtype=np.float32)
        assert lib().orc_centroids(self._h, _ptr(out)) == 0
        return out

    def delete(self, ids) -> int:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
        n = int(lib().orc_delete(self._h, _ptr(ids), ids.shape[0]))
        assert n >= 0
        return n

    @property
    def ntotal(self) -> int:
        return int(lib().orc_ntotal(self._h))

    def list_lengths(self):
        out = np.empty(self.nlist, dtype=np.int64)
        assert lib().orc_list_lengths(self._h, _ptr(out)) == 0
        return out

    def list_ids(self, j: int):
        n = int(self.list_lengths()[j])
        out = np.empty(max(n, 1), dtype=np.int64)
        got = lib().orc_list_ids(self._h, int(j), _ptr(out), n)
        assert got == n
        return out[:n]

    def coarse(self, q, nprobe: int, with_scores: bool = False):
        q = _f32(q).reshape(-1, self.d)
        nq = q.shape[0]
        probes = np.empty((nq, nprobe), dtype=np.int32)
        scores = np.empty((nq, self.nlist), dtype=np.float64) if with_scores else None
        assert lib().orc_coarse(self._h, _ptr(q), nq, nprobe, _ptr(probes), _ptr(scores)) == 0
        return (probes, scores) if with_scores else probes

    def scan_probes(self, q, k: int, probes):
        q = _f32(q).reshape(-1, self.d)
        probes = np.ascontiguousarray(probes, dtype=np.int32)
        nq, nprobe = probes.shape
        assert nq == q.shape[0]
        ids = np.empty((nq, k), dtype=np.int64)
        val = np.empty((nq, k), dtype=np.float64)
        rc = lib().orc_scan_probes(self._h, _ptr(q), nq, k, nprobe, _ptr(probes), _ptr(ids), _ptr(val))
        assert rc == 0
        return ids, val

    def search(self, q, k: int, nprobe: int):
        q = _f32(q).reshape(-1, self.d)
        nq = q.shape[0]
        ids = np.empty((nq, k), dtype=np.int64)
        val = np.empty((nq, k), dtype=np.float64)
        assert lib().orc_search(self._h, _ptr(q), nq, k, nprobe, _ptr(ids), _ptr(val)) == 0
        return ids, val


def search_multi(indexes, q_offsets, q, k: int, nprobe: int):
    d = indexes[0].d
    q = _f32(q).reshape(-1, d)
    offs = np.ascontiguousarray(q_offsets, dtype=np.int64)
    assert offs.shape[0] == len(indexes) + 1 and offs[-1] == q.shape[0]
    hs = (C.c_void_p * len(indexes))(*[ix._h for ix in indexes])
    ids = np.empty((q.shape[0], k), dtype=np.int64)
    val = np.empty((q.shape[0], k), dtype=np.float64)
    rc = lib().orc_search_multi(hs, len(indexes), _ptr(offs), _ptr(q), k, nprobe, _ptr(ids), _ptr(val))
    assert rc == 0
    return ids, val


def search_union(indexes, q, k: int, nprobe: int, probes=None):
    """Every query searched in every index of the scope, results merged (Section 3.2); probes, if given,
    are [n_indexes, nq, nprobe].  Returns (source position, ids, values)."""
    d = indexes[0].d
    q = _f32(q).reshape(-1, d)
    hs = (C.c_void_p * len(indexes))(*[ix._h for ix in indexes])
    src = np.empty((q.shape[0], k), dtype=np.int32)
    ids = np.empty((q.shape[0], k), dtype=np.int64)
    val = np.empty((q.shape[0], k), dtype=np.float64)
    if probes is None:
        rc = lib().orc_search_union(hs, len(indexes), _ptr(q), q.shape[0], k, nprobe, _ptr(src), _ptr(ids), _ptr(val))
    else:
        probes = np.ascontiguousarray(probes, dtype=np.int32)
        assert probes.shape == (len(indexes), q.shape[0], nprobe)
        rc = lib().orc_union_probes(hs, len(indexes), _ptr(q), q.shape[0], k, nprobe, _ptr(probes), _ptr(src),
                                    _ptr(ids), _ptr(val))
    assert rc == 0
    return src, ids, val


def search_levels(levels, q, k: int, nprobes, stop, kx: int = 0, probes=None):
    """Search down a stack of indexes, top level first, with the early-termination rule of Section 4.2:
    a query stops at a level as soon as that level gives it k candidates all of which are closer than
    stop[q] (= alpha_et * d_agent of its agent; inner product: all scores above stop[q]); otherwise it
    is searched again in the next level, whose result replaces the upper one (every level holds a subset
    of the one below).  The last level always ends the search.  The decision looks at the first k
    results; kx more are returned for the comparator.  probes, if given, is one [nq, nprobes[l]] array
    per level (the lists to scan instead of the coarse step's).  Returns (level, ids, values)."""
    d = levels[0].d
    q = _f32(q).reshape(-1, d)
    nq = q.shape[0]
    stop = np.asarray(stop, dtype=np.float64).reshape(nq)
    ip = levels[0].metric == 0
    ids = np.full((nq, k + kx), -1, dtype=np.int64)
    val = np.full((nq, k + kx), -np.inf if ip else np.inf, dtype=np.float64)
    level = np.full(nq, len(levels) - 1, dtype=np.int32)
    active = np.arange(nq)
    for l, ix in enumerate(levels):
        if active.size == 0:
            break
        if probes is None:
            li, lv = ix.search(q[active], k + kx, int(nprobes[l]))
        else:
            li, lv = ix.scan_probes(q[active], k + kx, np.ascontiguousarray(probes[l][active], dtype=np.int32))
        ids[active] = li
        val[active] = lv
        full = li[:, k - 1] >= 0
        kth = lv[:, k - 1]  # rows are sorted best first: the k-th is the farthest of the top k
        done = full & ((kth > stop[active]) if ip else (kth < stop[active]))
        if l == len(levels) - 1:
            done[:] = True
        level[active[done]] = l
        active = active[~done]
    return level, ids, val


def bruteforce(x, q, k: int, metric: int, ids=None):
    x = _f32(x)
    n, d = x.shape
    q = _f32(q).reshape(-1, d)
    if ids is not None:
        ids = np.ascontiguousarray(ids, dtype=np.int64)
    out_ids = np.empty((q.shape[0], k), dtype=np.int64)
    out_val = np.empty((q.shape[0], k), dtype=np.float64)
    rc = lib().orc_bruteforce(_ptr(x), _ptr(ids), n, d, int(metric), _ptr(q), q.shape[0], k,
                              _ptr(out_ids), _ptr(out_val))
    assert rc == 0
    return out_ids, out_val


def pair_values(q, x, metric: int):
    q = _f32(q)
    x = _f32(x)
    assert q.shape == x.shape and q.ndim == 2
    out = np.empty(q.shape[0], dtype=np.float64)
    assert lib().orc_pair_values(_ptr(q), _ptr(x), q.shape[0], q.shape[1], int(metric), _ptr(out)) == 0
    return out


def kmeans(x, nlist: int, iters: int, init_rows):
    x = _f32(x)
    n, d = x.shape
    init_rows = np.ascontiguousarray(init_rows, dtype=np.int64)
    assert init_rows.shape[0] == nlist
    cent = np.empty((nlist, d), dtype=np.float32)
    inertia = np.empty(max(iters, 1), dtype=np.float64)
    assign = np.empty(n, dtype=np.int32)
    rc = lib().orc_kmeans(_ptr(x), n, d, nlist, iters, _ptr(init_rows), _ptr(cent), _ptr(inertia), _ptr(assign))
    assert rc == 0
    return cent, inertia[:iters], assign
