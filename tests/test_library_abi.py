"""The C-ABI library loads without a GPU and exports what include/pancake.h declares.
Only host-side paths are exercised here (no kernel is launched)."""
import ctypes as C
import os
import re

import pytest

from paper_2602_21477_amd import binding as B

HEADER = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "pancake.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2602_21477_amd import build
        build.build()
    return B.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pk_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_and_arena_bytes(lib):
    assert B.strerror(0) == "ok"
    assert "handle" in B.strerror(B.PK_ERR_BAD_HANDLE)
    cfg = B.pk_config(768, 1024, B.PK_METRIC_IP, B.PK_F32, 0, 0)
    a = B.pk_arena_bytes(cfg, 1_000_000, 0)
    # at least the raw vectors; at most one partly filled page per list plus the tables more
    assert 1_000_000 * 768 * 4 < a < 1_000_000 * 768 * 4 + 1025 * 128 * (768 * 4 + 12) + 64 * 2 ** 20
    assert B.pk_arena_bytes(cfg, 1_000_000, 100_000) > a
    h = B.pk_config(768, 1024, B.PK_METRIC_L2, B.PK_F16, 0, 0)
    assert B.pk_arena_bytes(h, 1_000_000, 0) < 0.6 * a
    for bad in (B.pk_config(0, 4, 0, 0, 0, 0), B.pk_config(8, 0, 0, 0, 0, 0), B.pk_config(8, 4, 2, 0, 0, 0),
                B.pk_config(8, 4, 0, 3, 0, 0), B.pk_config(8, 4, 0, 0, 48, 0), B.pk_config(4096, 4, 0, 0, 0, 0)):
        assert B.pk_arena_bytes(bad, 10, 0) == 0


def test_host_side_argument_checks_without_gpu(lib):
    null = C.c_void_p(None)
    out = C.c_void_p()
    cfg = B.pk_config(16, 4, 0, 0, 0, 0)
    assert lib.pk_index_build(C.byref(cfg), null, null, null, 0, null, 0, null, C.byref(out)) == B.PK_ERR_INVALID_ARG
    assert lib.pk_search(null, null, 1, 1, 1, null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_search_noalloc(null, null, 1, 1, 1, null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_index_set_emit_cap(null, 0) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_search_noalloc_bytes(null, 1, 1, 1) == 0
    assert lib.pk_insert(null, null, null, 1, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_coarse(null, null, 1, 1, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_index_free(null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_index_compact(null, null, 0, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_delete(null, null, 1, None, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_index_split(null, null, 0, 10, 2, None, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_index_centroids(null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_list_ids(null, 0, null, 0, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_kmeans(null, 10, 8, 4, 1, null, null, None, null) == B.PK_ERR_INVALID_ARG
    # a buffer that is not a handle is rejected by the magic check
    fake = (C.c_uint64 * 64)()
    assert lib.pk_search(C.cast(fake, C.c_void_p), null, 1, 1, 1, null, null, null) == B.PK_ERR_BAD_HANDLE
    hs = (C.c_void_p * 1)(None)
    offs = (C.c_int64 * 2)(0, 1)
    assert lib.pk_search_multi(hs, 1, offs, null, 1, 1, null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_search_multi(hs, 0, offs, null, 1, 1, null, null, null) == B.PK_ERR_INVALID_ARG
    assert lib.pk_workspace_reserve(hs, 1, 1, 1, 1, 0, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_workspace_reserve(hs, 0, 1, 1, 1, 0, null) == B.PK_ERR_INVALID_ARG
    assert lib.pk_search_union(hs, 1, null, 1, 1, 1, null, null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_insert_multi(hs, 1, offs, null, null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_search_union(hs, 0, null, 1, 1, 1, null, null, null, null) == B.PK_ERR_INVALID_ARG
    nps = (C.c_int32 * 1)(1)
    assert lib.pk_search_levels(hs, 1, nps, null, 1, 1, null, null, null, null, null) == B.PK_ERR_BAD_HANDLE
    assert lib.pk_search_levels(hs, 0, nps, null, 1, 1, null, null, null, null, null) == B.PK_ERR_INVALID_ARG
    assert lib.pk_search_levels(hs, 1, None, null, 1, 1, null, null, null, null, null) == B.PK_ERR_INVALID_ARG


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(FileNotFoundError):
        B.lib()
