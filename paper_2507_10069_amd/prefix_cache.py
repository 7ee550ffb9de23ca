"""ctypes binding of the host-side prefix cache declared in ``include/emm_prefix_cache.h``.

Argument marshalling only: the functions have the names and meanings of the C entry points, take and
return numpy arrays / Python ints, and raise :class:`binding.EmmError` on a non-zero status.  The tree,
the eviction order and the hash are all in ``libemm.so`` (``csrc/prefix_cache.cpp``).
"""
from __future__ import annotations

import ctypes
from typing import Tuple

import numpy as np

from . import binding as B

EMM_ERR_NO_SPACE, EMM_ERR_NOT_FOUND = 6, 7

EXPORTS = ["emm_mm_content_hash", "emm_mm_token_ids", "emm_prefix_cache_create", "emm_prefix_cache_destroy",
           "emm_prefix_cache_begin", "emm_prefix_cache_append", "emm_prefix_cache_commit", "emm_prefix_cache_release",
           "emm_prefix_cache_get_stats"]


class emm_prefix_cache_stats(ctypes.Structure):
    _fields_ = [("lookups", ctypes.c_int64), ("lookup_tokens", ctypes.c_int64), ("hit_tokens", ctypes.c_int64),
                ("evictions", ctypes.c_int64), ("num_pages", ctypes.c_int32), ("free_pages", ctypes.c_int32),
                ("cached_pages", ctypes.c_int32), ("evictable_pages", ctypes.c_int32),
                ("private_pages", ctypes.c_int32), ("live_requests", ctypes.c_int32)]


_declared = False


def _lib() -> ctypes.CDLL:
    global _declared
    lib = B.load()
    if not _declared:
        vp, ci, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int32, ctypes.c_int64
        i32p, i64p, u8p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_uint8)
        lib.emm_mm_content_hash.restype = ci
        lib.emm_mm_content_hash.argtypes = [vp, ctypes.c_size_t, u8p]
        lib.emm_mm_token_ids.restype = ci
        lib.emm_mm_token_ids.argtypes = [u8p, i32, i64p]
        lib.emm_prefix_cache_create.restype = ci
        lib.emm_prefix_cache_create.argtypes = [i32, i32, ctypes.POINTER(vp)]
        lib.emm_prefix_cache_destroy.restype = None
        lib.emm_prefix_cache_destroy.argtypes = [vp]
        lib.emm_prefix_cache_begin.restype = ci
        lib.emm_prefix_cache_begin.argtypes = [vp, i64p, i32, i32, i32p, i32p, i64p]
        lib.emm_prefix_cache_append.restype = ci
        lib.emm_prefix_cache_append.argtypes = [vp, i64, i64p, i32, i32, i32p]
        lib.emm_prefix_cache_commit.restype = ci
        lib.emm_prefix_cache_commit.argtypes = [vp, i64, i32]
        lib.emm_prefix_cache_release.restype = ci
        lib.emm_prefix_cache_release.argtypes = [vp, i64]
        lib.emm_prefix_cache_get_stats.restype = ci
        lib.emm_prefix_cache_get_stats.argtypes = [vp, ctypes.POINTER(emm_prefix_cache_stats)]
        _declared = True
    return lib


def _i64(tokens) -> np.ndarray:
    return np.ascontiguousarray(tokens, dtype=np.int64)


def emm_mm_content_hash(data: bytes) -> bytes:
    digest = (ctypes.c_uint8 * 32)()
    buf = ctypes.create_string_buffer(bytes(data), len(data)) if len(data) else None
    B._check(_lib().emm_mm_content_hash(ctypes.cast(buf, ctypes.c_void_p) if buf is not None else None,
                                        len(data), digest), "emm_mm_content_hash")
    return bytes(digest)


def emm_mm_token_ids(digest: bytes, n_tokens: int) -> np.ndarray:
    ids = np.empty(max(n_tokens, 0), dtype=np.int64)
    d = (ctypes.c_uint8 * 32).from_buffer_copy(digest)
    B._check(_lib().emm_mm_token_ids(d, n_tokens, ids.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))),
             "emm_mm_token_ids")
    return ids


def emm_prefix_cache_create(num_pages: int, page_size: int) -> int:
    handle = ctypes.c_void_p()
    B._check(_lib().emm_prefix_cache_create(num_pages, page_size, ctypes.byref(handle)), "emm_prefix_cache_create")
    return handle.value


def emm_prefix_cache_destroy(cache: int) -> None:
    _lib().emm_prefix_cache_destroy(cache)


def emm_prefix_cache_begin(cache: int, tokens, max_pages: int) -> Tuple[np.ndarray, int, int]:
    """Returns (page_table_row [max_pages] int32, prefix_len, request id)."""
    tok = _i64(tokens)
    row = np.empty(max(max_pages, 0), dtype=np.int32)
    prefix_len, request = ctypes.c_int32(), ctypes.c_int64()
    B._check(_lib().emm_prefix_cache_begin(cache, tok.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)), tok.size,
                                           max_pages, row.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                           ctypes.byref(prefix_len), ctypes.byref(request)),
             "emm_prefix_cache_begin")
    return row, prefix_len.value, request.value


def emm_prefix_cache_append(cache: int, request: int, tokens, max_pages: int) -> np.ndarray:
    tok = _i64(tokens)
    row = np.empty(max(max_pages, 0), dtype=np.int32)
    B._check(_lib().emm_prefix_cache_append(cache, request, tok.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                            tok.size, max_pages, row.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))),
             "emm_prefix_cache_append")
    return row


def emm_prefix_cache_commit(cache: int, request: int, n_computed: int) -> None:
    B._check(_lib().emm_prefix_cache_commit(cache, request, n_computed), "emm_prefix_cache_commit")


def emm_prefix_cache_release(cache: int, request: int) -> None:
    B._check(_lib().emm_prefix_cache_release(cache, request), "emm_prefix_cache_release")


def emm_prefix_cache_get_stats(cache: int) -> dict:
    s = emm_prefix_cache_stats()
    B._check(_lib().emm_prefix_cache_get_stats(cache, ctypes.byref(s)), "emm_prefix_cache_get_stats")
    return {name: int(getattr(s, name)) for name, _ in emm_prefix_cache_stats._fields_}
