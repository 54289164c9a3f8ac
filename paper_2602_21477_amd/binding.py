"""ctypes binding of libpancake.so: the C-ABI entry points under their own names.

Argument marshalling only.  Every step of search / insert / build runs in the HIP
kernels behind the C ABI; PyTorch is used for device memory (tensors own the
buffers, including arenas) and for the current HIP stream.  There is no CPU
fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpancake.so")

PK_METRIC_IP, PK_METRIC_L2 = 0, 1
PK_F32, PK_F16 = 0, 1
PK_OK = 0
PK_ERR_INVALID_ARG, PK_ERR_BAD_HANDLE, PK_ERR_DIM_MISMATCH, PK_ERR_NOMEM, PK_ERR_HIP, PK_ERR_UNSUPPORTED = (
    -1, -2, -3, -4, -5, -6)
PK_ERR_WORKSPACE = -7
PK_NOALLOC_WORKSPACE_BYTES = 64 << 20

EXPORTS = ["pk_workspace_reserve", "pk_index_set_emit_cap", "pk_search_noalloc", "pk_search_noalloc_bytes", "pk_search_levels", "pk_search_union", "pk_insert_multi", "pk_delete", "pk_index_split", "pk_index_centroids", "pk_list_ids", "pk_arena_bytes", "pk_index_build", "pk_index_add_arena", "pk_index_compact", "pk_kmeans", "pk_insert", "pk_insert_assigned", "pk_search",
           "pk_search_multi", "pk_coarse", "pk_scan_probes", "pk_index_stats", "pk_list_lengths", "pk_profile_begin",
           "pk_profile_end", "pk_index_free", "pk_strerror"]


class pk_config(C.Structure):
    _fields_ = [("d", C.c_int32), ("nlist", C.c_int32), ("metric", C.c_int32), ("storage", C.c_int32),
                ("page_vecs", C.c_int32), ("max_delta_pages", C.c_int32)]


class pk_stats(C.Structure):
    _fields_ = [("n_total", C.c_int64), ("n_inserted", C.c_int64), ("pages_total", C.c_int64),
                ("pages_used", C.c_int64), ("arena_bytes", C.c_int64), ("workspace_bytes", C.c_int64),
                ("workspace_grows", C.c_int64),
                ("max_list_len", C.c_int64), ("device_error", C.c_int32), ("n_arenas", C.c_int32)]


class pk_profile(C.Structure):
    _fields_ = [("launches", C.c_int32), ("coarse_ms", C.c_float), ("worklist_ms", C.c_float),
                ("scan_ms", C.c_float), ("select_ms", C.c_float), ("scanned_rows", C.c_int64),
                ("candidates", C.c_int64), ("tiles", C.c_int64), ("emitted", C.c_int64),
                ("overflowed", C.c_int64), ("max_emitted", C.c_int64), ("scan_hot_ms", C.c_float)]


class PancakeError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


_lib = None


def lib():
    """The loaded library; raises if it has not been built (python -m paper_2602_21477_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_21477_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.pk_arena_bytes.restype = C.c_size_t
        L.pk_arena_bytes.argtypes = [C.POINTER(pk_config), i64, i64]
        L.pk_index_build.argtypes = [C.POINTER(pk_config), vp, vp, vp, i64, vp, C.c_size_t, vp, C.POINTER(vp)]
        L.pk_index_add_arena.argtypes = [vp, vp, C.c_size_t, vp]
        L.pk_index_compact.argtypes = [vp, vp, C.c_size_t, vp]
        L.pk_index_split.argtypes = [vp, vp, C.c_size_t, i64, i32, C.POINTER(i32), vp]
        L.pk_index_centroids.argtypes = [vp, vp, vp]
        L.pk_list_ids.argtypes = [vp, i32, vp, i64, vp]
        L.pk_kmeans.argtypes = [vp, i64, i32, i32, i32, vp, vp, C.POINTER(C.c_double), vp]
        L.pk_insert.argtypes = [vp, vp, vp, i64, vp, vp]
        L.pk_insert_assigned.argtypes = [vp, vp, vp, i64, vp, vp]
        L.pk_insert_multi.argtypes = [C.POINTER(vp), i32, C.POINTER(i64), vp, vp, vp, vp]
        L.pk_delete.argtypes = [vp, vp, i64, C.POINTER(i64), vp]
        L.pk_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        L.pk_workspace_reserve.argtypes = [C.POINTER(vp), i32, i64, i32, i32, i64, vp]
        L.pk_index_set_emit_cap.argtypes = [vp, i32]
        L.pk_search_noalloc.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
        L.pk_search_noalloc_bytes.restype = C.c_size_t
        L.pk_search_noalloc_bytes.argtypes = [vp, i64, i32, i32]
        L.pk_search_multi.argtypes = [C.POINTER(vp), i32, C.POINTER(i64), vp, i32, i32, vp, vp, vp]
        L.pk_search_union.argtypes = [C.POINTER(vp), i32, vp, i64, i32, i32, vp, vp, vp, vp]
        L.pk_search_levels.argtypes = [C.POINTER(vp), i32, C.POINTER(i32), vp, i64, i32, vp, vp, vp, vp, vp]
        L.pk_coarse.argtypes = [vp, vp, i64, i32, vp, vp]
        L.pk_scan_probes.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp, vp]
        L.pk_index_stats.argtypes = [vp, C.POINTER(pk_stats), vp]
        L.pk_list_lengths.argtypes = [vp, vp, vp]
        L.pk_profile_begin.argtypes = [vp, vp]
        L.pk_profile_end.argtypes = [vp, C.POINTER(pk_profile), vp]
        L.pk_index_free.argtypes = [vp]
        L.pk_strerror.restype = C.c_char_p
        L.pk_strerror.argtypes = [C.c_int]
        for name in EXPORTS:
            if name not in ("pk_arena_bytes", "pk_strerror", "pk_search_noalloc_bytes"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def strerror(status: int) -> str:
    return lib().pk_strerror(int(status)).decode()


def _check(status: int, what: str):
    if status != PK_OK:
        raise PancakeError(status, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t, dtype, what):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise ValueError(f"{what}: need a contiguous {dtype} CUDA tensor")
    return t.data_ptr()


def pk_arena_bytes(cfg: pk_config, n: int, n_insert_reserve: int) -> int:
    return int(lib().pk_arena_bytes(C.byref(cfg), int(n), int(n_insert_reserve)))


def pk_index_build(cfg: pk_config, centroids, vectors, ids, arena) -> int:
    """Returns the handle (an integer).  `arena` is a uint8 CUDA tensor the caller keeps alive."""
    n = 0 if vectors is None else vectors.shape[0]
    h = C.c_void_p()
    rc = lib().pk_index_build(C.byref(cfg), _dev(centroids, torch.float32, "centroids"),
                              _dev(vectors, torch.float32, "vectors"), _dev(ids, torch.int64, "ids"), n,
                              _dev(arena, torch.uint8, "arena"), arena.numel(), _stream(), C.byref(h))
    _check(rc, "pk_index_build")
    return h.value


def pk_index_add_arena(handle: int, arena):
    _check(lib().pk_index_add_arena(handle, _dev(arena, torch.uint8, "arena"), arena.numel(), _stream()),
           "pk_index_add_arena")


def pk_kmeans(vectors, centroids, iters: int, assign_out=None):
    """Lloyd iterations in place on `centroids`; returns the per-iteration objective (host floats)."""
    n, d = vectors.shape
    inertia = (C.c_double * iters)()
    _check(lib().pk_kmeans(_dev(vectors, torch.float32, "vectors"), n, d, centroids.shape[0], iters,
                           _dev(centroids, torch.float32, "centroids"), _dev(assign_out, torch.int32, "assign_out"),
                           inertia, _stream()), "pk_kmeans")
    return [float(v) for v in inertia]


def pk_insert_multi(handles, v_offsets, vectors, ids=None, assigned_lists=None):
    hs = (C.c_void_p * len(handles))(*handles)
    offs = (C.c_int64 * len(v_offsets))(*[int(v) for v in v_offsets])
    _check(lib().pk_insert_multi(hs, len(handles), offs, _dev(vectors, torch.float32, "vectors"),
                                 _dev(ids, torch.int64, "ids"), _dev(assigned_lists, torch.int32, "assigned_lists"),
                                 _stream()), "pk_insert_multi")


def pk_index_split(handle: int, arena, threshold: int, iters: int) -> int:
    n = C.c_int32(0)
    _check(lib().pk_index_split(handle, _dev(arena, torch.uint8, "arena"), arena.numel(), threshold, iters,
                                C.byref(n), _stream()), "pk_index_split")
    return int(n.value)


def pk_index_centroids(handle: int, out):
    _check(lib().pk_index_centroids(handle, _dev(out, torch.float32, "out"), _stream()), "pk_index_centroids")


def pk_list_ids(handle: int, lst: int, out):
    _check(lib().pk_list_ids(handle, lst, _dev(out, torch.int64, "out"), out.numel(), _stream()), "pk_list_ids")


def pk_delete(handle: int, ids) -> int:
    n = C.c_int64(0)
    _check(lib().pk_delete(handle, _dev(ids, torch.int64, "ids"), ids.shape[0], C.byref(n), _stream()), "pk_delete")
    return int(n.value)


def pk_index_compact(handle: int, arena):
    _check(lib().pk_index_compact(handle, _dev(arena, torch.uint8, "arena"), arena.numel(), _stream()),
           "pk_index_compact")


def pk_insert(handle: int, vectors, ids=None, assigned_lists=None):
    _check(lib().pk_insert(handle, _dev(vectors, torch.float32, "vectors"), _dev(ids, torch.int64, "ids"),
                           vectors.shape[0], _dev(assigned_lists, torch.int32, "assigned_lists"), _stream()),
           "pk_insert")


def pk_insert_assigned(handle: int, vectors, ids, lists):
    _check(lib().pk_insert_assigned(handle, _dev(vectors, torch.float32, "vectors"), _dev(ids, torch.int64, "ids"),
                                    vectors.shape[0], _dev(lists, torch.int32, "lists"), _stream()),
           "pk_insert_assigned")


def pk_search(handle: int, queries, k: int, nprobe: int, out_ids, out_dist):
    _check(lib().pk_search(handle, _dev(queries, torch.float32, "queries"), queries.shape[0], k, nprobe,
                           _dev(out_ids, torch.int64, "out_ids"), _dev(out_dist, torch.float32, "out_dist"),
                           _stream()), "pk_search")


def pk_workspace_reserve(handles, nq_max: int, k_max: int, nprobe_max: int, inserts_ahead: int = 0):
    hs = (C.c_void_p * len(handles))(*handles)
    _check(lib().pk_workspace_reserve(hs, len(handles), int(nq_max), int(k_max), int(nprobe_max), int(inserts_ahead),
                                      _stream()), "pk_workspace_reserve")


def pk_index_set_emit_cap(handle: int, entries: int):
    _check(lib().pk_index_set_emit_cap(handle, int(entries)), "pk_index_set_emit_cap")


def pk_search_noalloc(handle: int, queries, k: int, nprobe: int, out_ids, out_dist):
    _check(lib().pk_search_noalloc(handle, _dev(queries, torch.float32, "queries"), queries.shape[0], k, nprobe,
                                   _dev(out_ids, torch.int64, "out_ids"), _dev(out_dist, torch.float32, "out_dist"),
                                   _stream()), "pk_search_noalloc")


def pk_search_noalloc_bytes(handle: int, nq: int, k: int, nprobe: int) -> int:
    return int(lib().pk_search_noalloc_bytes(handle, int(nq), int(k), int(nprobe)))


def pk_search_multi(handles, q_offsets, queries, k: int, nprobe: int, out_ids, out_dist):
    n = len(handles)
    hs = (C.c_void_p * n)(*handles)
    offs = (C.c_int64 * (n + 1))(*[int(o) for o in q_offsets])
    _check(lib().pk_search_multi(hs, n, offs, _dev(queries, torch.float32, "queries"), k, nprobe,
                                 _dev(out_ids, torch.int64, "out_ids"), _dev(out_dist, torch.float32, "out_dist"),
                                 _stream()), "pk_search_multi")


def pk_coarse(handle: int, queries, nprobe: int, out_probes):
    _check(lib().pk_coarse(handle, _dev(queries, torch.float32, "queries"), queries.shape[0], nprobe,
                           _dev(out_probes, torch.int32, "out_probes"), _stream()), "pk_coarse")


def pk_scan_probes(handle: int, queries, k: int, probes, out_ids, out_dist):
    _check(lib().pk_scan_probes(handle, _dev(queries, torch.float32, "queries"), queries.shape[0], k,
                                probes.shape[1], _dev(probes, torch.int32, "probes"),
                                _dev(out_ids, torch.int64, "out_ids"), _dev(out_dist, torch.float32, "out_dist"),
                                _stream()), "pk_scan_probes")


def pk_index_stats(handle: int) -> pk_stats:
    st = pk_stats()
    _check(lib().pk_index_stats(handle, C.byref(st), _stream()), "pk_index_stats")
    return st


def pk_list_lengths(handle: int, nlist: int):
    import numpy as np
    out = np.empty(nlist, dtype=np.int64)
    _check(lib().pk_list_lengths(handle, out.ctypes.data_as(C.c_void_p), _stream()), "pk_list_lengths")
    return out


def pk_profile_begin(handle: int):
    _check(lib().pk_profile_begin(handle, _stream()), "pk_profile_begin")


def pk_profile_end(handle: int) -> pk_profile:
    pr = pk_profile()
    _check(lib().pk_profile_end(handle, C.byref(pr), _stream()), "pk_profile_end")
    return pr


def pk_index_free(handle: int):
    _check(lib().pk_index_free(handle), "pk_index_free")


class Index:
    """Convenience owner of one handle and its arena tensors (no arithmetic here)."""

    def __init__(self, centroids, vectors, metric=PK_METRIC_IP, storage=PK_F32, ids=None, page_vecs=0,
                 max_delta_pages=0, insert_reserve=0, arena_bytes=None):
        nlist, d = centroids.shape
        self.cfg = pk_config(d, nlist, metric, storage, page_vecs, max_delta_pages)
        n = 0 if vectors is None else vectors.shape[0]
        if arena_bytes is None:
            arena_bytes = pk_arena_bytes(self.cfg, n, insert_reserve)
            if arena_bytes == 0:
                raise PancakeError(PK_ERR_INVALID_ARG, "pk_arena_bytes")
        self.device = centroids.device
        self.arenas = [torch.empty(arena_bytes, dtype=torch.uint8, device=self.device)]
        self.nlist, self.d = nlist, d
        self.handle = pk_index_build(self.cfg, centroids, vectors, ids, self.arenas[0])

    def add_arena(self, nbytes: int):
        t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        pk_index_add_arena(self.handle, t)
        self.arenas.append(t)

    def compact(self, nbytes: int):
        """Moves the index into one new arena of nbytes; the old arena tensors are released."""
        t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        pk_index_compact(self.handle, t)
        self.arenas = [t]

    def insert(self, vectors, ids=None, want_lists=False):
        out = torch.empty(vectors.shape[0], dtype=torch.int32, device=self.device) if want_lists else None
        pk_insert(self.handle, vectors, ids, out)
        return out

    def split(self, threshold: int, iters: int, nbytes: int) -> int:
        """IVF-Split into one new arena of nbytes; returns the number of lists split (nlist grows by it)."""
        t = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        n = pk_index_split(self.handle, t, threshold, iters)
        self.arenas = [t]
        self.nlist += n
        self.cfg.nlist = self.nlist
        return n

    def centroids(self):
        out = torch.empty((self.nlist, self.d), dtype=torch.float32, device=self.device)
        pk_index_centroids(self.handle, out)
        return out

    def list_ids(self, lst: int):
        n = int(self.list_lengths()[lst])
        out = torch.empty(max(n, 1), dtype=torch.int64, device=self.device)
        pk_list_ids(self.handle, lst, out[:n])
        return out[:n]

    def delete(self, ids) -> int:
        return pk_delete(self.handle, ids)

    def insert_assigned(self, vectors, lists, ids=None):
        pk_insert_assigned(self.handle, vectors, ids, lists)

    def search(self, queries, k, nprobe):
        ids = torch.empty((queries.shape[0], k), dtype=torch.int64, device=self.device)
        dist = torch.empty((queries.shape[0], k), dtype=torch.float32, device=self.device)
        pk_search(self.handle, queries, k, nprobe, ids, dist)
        return ids, dist

    def coarse(self, queries, nprobe):
        out = torch.empty((queries.shape[0], nprobe), dtype=torch.int32, device=self.device)
        pk_coarse(self.handle, queries, nprobe, out)
        return out

    def scan_probes(self, queries, k, probes):
        ids = torch.empty((queries.shape[0], k), dtype=torch.int64, device=self.device)
        dist = torch.empty((queries.shape[0], k), dtype=torch.float32, device=self.device)
        pk_scan_probes(self.handle, queries, k, probes, ids, dist)
        return ids, dist

    def stats(self):
        return pk_index_stats(self.handle)

    def reserve(self, nq_max, k_max, nprobe_max, inserts_ahead=0):
        pk_workspace_reserve([self.handle], nq_max, k_max, nprobe_max, inserts_ahead)

    def list_lengths(self):
        return pk_list_lengths(self.handle, self.nlist)

    def close(self):
        if self.handle:
            torch.cuda.synchronize(self.device)
            pk_index_free(self.handle)
            self.handle = None
            self.arenas = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def pk_search_union(handles, queries, k: int, nprobe: int, out_src, out_ids, out_dist):
    hs = (C.c_void_p * len(handles))(*handles)
    _check(lib().pk_search_union(hs, len(handles), _dev(queries, torch.float32, "queries"), queries.shape[0], k, nprobe,
                                 _dev(out_src, torch.int32, "out_src"), _dev(out_ids, torch.int64, "out_ids"),
                                 _dev(out_dist, torch.float32, "out_dist"), _stream()), "pk_search_union")


def pk_search_levels(handles, nprobes, queries, k: int, stop, out_level, out_ids, out_dist):
    hs = (C.c_void_p * len(handles))(*handles)
    nps = (C.c_int32 * len(handles))(*[int(x) for x in nprobes])
    _check(lib().pk_search_levels(hs, len(handles), nps, _dev(queries, torch.float32, "queries"), queries.shape[0], k,
                                  _dev(stop, torch.float32, "stop"), _dev(out_level, torch.int32, "out_level"),
                                  _dev(out_ids, torch.int64, "out_ids"), _dev(out_dist, torch.float32, "out_dist"),
                                  _stream()), "pk_search_levels")


def search_levels(indexes, nprobes, queries, k, stop):
    """Top level first; returns (level each query ended at, ids, values)."""
    dev = queries.device
    level = torch.empty(queries.shape[0], dtype=torch.int32, device=dev)
    ids = torch.empty((queries.shape[0], k), dtype=torch.int64, device=dev)
    dist = torch.empty((queries.shape[0], k), dtype=torch.float32, device=dev)
    pk_search_levels([ix.handle for ix in indexes], nprobes, queries, k, stop, level, ids, dist)
    return level, ids, dist


def search_union(indexes, queries, k, nprobe):
    dev = queries.device
    src = torch.empty((queries.shape[0], k), dtype=torch.int32, device=dev)
    ids = torch.empty((queries.shape[0], k), dtype=torch.int64, device=dev)
    dist = torch.empty((queries.shape[0], k), dtype=torch.float32, device=dev)
    pk_search_union([ix.handle for ix in indexes], queries, k, nprobe, src, ids, dist)
    return src, ids, dist


def search_multi(indexes, q_offsets, queries, k, nprobe):
    dev = queries.device
    ids = torch.empty((queries.shape[0], k), dtype=torch.int64, device=dev)
    dist = torch.empty((queries.shape[0], k), dtype=torch.float32, device=dev)
    pk_search_multi([ix.handle for ix in indexes], q_offsets, queries, k, nprobe, ids, dist)
    return ids, dist
