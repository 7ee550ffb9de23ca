"""fp64 CPU oracle for prefix-cached paged prefill attention.  TEST INFRASTRUCTURE ONLY.

(``prefix_cache_model.py`` beside this file is the reference model of the host-side prefix cache; it is
plain Python and is imported on its own.)

Importable from ``tests/``, the smoke check and the benchmark's ``cpu_baseline`` leg; nothing in
the product package imports it, and it imports nothing from the product package.

``oracle.c`` holds the plain definition (paged KV pool, byte-exact scatter, one softmax row at
a time in fp64); ``bruteforce.py`` is a dense numpy recomputation that knows neither pages nor
a cache and serves as one of the oracle's pins.  The functions here only marshal numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

from . import build as _build

_F32, _BF16 = 0, 1
_CAUSAL, _CROSS = 0, 1
_lib = None


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Load (building first if the library is missing or stale) and declare signatures."""
    global _lib
    if path is None and _lib is not None:
        return _lib
    # EMM_ORACLE_LIB names another build of the same source (the sanitized one of tests/test_sanitized_host.py)
    lib = ctypes.CDLL(path or os.environ.get("EMM_ORACLE_LIB") or _build.build())
    i32p, vp, i64p, f64p = (ctypes.POINTER(ctypes.c_int32), ctypes.c_void_p,
                            ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double))
    ci, cd, c64 = ctypes.c_int, ctypes.c_double, ctypes.c_int64
    lib.oracle_kv_scatter.restype = ci
    lib.oracle_kv_scatter.argtypes = [ci] * 7 + [i32p] * 4 + [vp] * 4
    lib.oracle_attention.restype = ci
    lib.oracle_attention.argtypes = [ci] * 9 + [cd] + [i32p] * 4 + [vp] * 3 + [c64, i64p, f64p, f64p]
    lib.oracle_row_weights.restype = ci
    lib.oracle_row_weights.argtypes = [ci] * 9 + [cd] + [i32p] * 4 + [vp] * 3 + [c64, ci, f64p, ci]
    lib.oracle_num_threads.restype = ci
    lib.oracle_num_threads.argtypes = []
    if path is None:
        _lib = lib
    return lib


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(ty)


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return _F32
    if a.dtype == np.uint16:
        return _BF16
    raise TypeError("oracle tensors are float32 or uint16 (bf16 bit patterns), got %s" % a.dtype)


def kv_scatter(page_table, prefix_lens, new_lens, cu_new_lens, k_new, v_new, k_cache, v_cache, lib=None):
    """Return copies of ``k_cache``/``v_cache`` ([num_pages][Hkv][page_size][d]) with the new tokens'
    K/V rows ([T][Hkv][d]) written to the slots after each request's cached prefix."""
    lib = lib or load()
    page_table, prefix_lens, new_lens, cu = map(_i32, (page_table, prefix_lens, new_lens, cu_new_lens))
    k_out = np.array(k_cache, copy=True, order="C")
    v_out = np.array(v_cache, copy=True, order="C")
    num_pages, n_kv, ps, d = k_out.shape
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    assert k_new.dtype == k_out.dtype and v_new.dtype == v_out.dtype
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = lib.oracle_kv_scatter(len(prefix_lens), n_kv, d, ps, num_pages, page_table.shape[1],
                               k_out.dtype.itemsize, _p(page_table, i32p), _p(prefix_lens, i32p),
                               _p(new_lens, i32p), _p(cu, i32p), k_new.ctypes.data, v_new.ctypes.data,
                               k_out.ctypes.data, v_out.ctypes.data)
    if rc != 0:
        raise ValueError("oracle_kv_scatter: page id out of range")
    return k_out, v_out


def attention(kind: str, page_table, prefix_lens, new_lens, cu_new_lens, q, k_cache, v_cache,
              scale: float, tokens: Optional[Sequence[int]] = None, lib=None):
    """Attention rows in fp64.  ``kind`` is "causal" (keys 0..P_r+j) or "cross" (keys 0..P_r-1).
    ``tokens`` selects packed query tokens (default all).  Returns (out [n][H][d], lse [n][H])."""
    lib = lib or load()
    page_table, prefix_lens, new_lens, cu = map(_i32, (page_table, prefix_lens, new_lens, cu_new_lens))
    q = np.ascontiguousarray(q)
    k_cache = np.ascontiguousarray(k_cache)
    v_cache = np.ascontiguousarray(v_cache)
    code = _dtype_code(q)
    assert _dtype_code(k_cache) == code and _dtype_code(v_cache) == code
    T, n_q, d = q.shape
    num_pages, n_kv, ps, d2 = k_cache.shape
    assert d2 == d and n_q % n_kv == 0 and T == int(cu[-1])
    if tokens is None:
        n, tok_p = T, None
    else:
        tok = np.ascontiguousarray(tokens, dtype=np.int64)
        n, tok_p = len(tok), _p(tok, ctypes.POINTER(ctypes.c_int64))
    out = np.zeros((n, n_q, d), dtype=np.float64)
    lse = np.zeros((n, n_q), dtype=np.float64)
    i32p, f64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
    rc = lib.oracle_attention({"causal": _CAUSAL, "cross": _CROSS}[kind], code, len(prefix_lens), n_q, n_kv,
                              d, ps, num_pages, page_table.shape[1], float(scale), _p(page_table, i32p),
                              _p(prefix_lens, i32p), _p(new_lens, i32p), _p(cu, i32p), q.ctypes.data,
                              k_cache.ctypes.data, v_cache.ctypes.data, n, tok_p, _p(out, f64p), _p(lse, f64p))
    if rc != 0:
        raise ValueError("oracle_attention failed with code %d" % rc)
    return out, lse


def row_weights(kind: str, page_table, prefix_lens, new_lens, cu_new_lens, q, k_cache, v_cache,
                scale: float, token: int, head: int, lib=None) -> np.ndarray:
    """Normalised softmax weights of one (packed token, query head) row."""
    lib = lib or load()
    page_table, prefix_lens, new_lens, cu = map(_i32, (page_table, prefix_lens, new_lens, cu_new_lens))
    q = np.ascontiguousarray(q)
    k_cache = np.ascontiguousarray(k_cache)
    v_cache = np.ascontiguousarray(v_cache)
    code = _dtype_code(q)
    T, n_q, d = q.shape
    num_pages, n_kv, ps, _ = k_cache.shape
    cap = int(prefix_lens.max()) + int(new_lens.max()) + 1
    w = np.zeros(cap, dtype=np.float64)
    i32p, f64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
    n = lib.oracle_row_weights({"causal": _CAUSAL, "cross": _CROSS}[kind], code, len(prefix_lens), n_q, n_kv,
                               d, ps, num_pages, page_table.shape[1], float(scale), _p(page_table, i32p),
                               _p(prefix_lens, i32p), _p(new_lens, i32p), _p(cu, i32p), q.ctypes.data,
                               k_cache.ctypes.data, v_cache.ctypes.data, int(token), int(head), _p(w, f64p), cap)
    if n < 0:
        raise ValueError("oracle_row_weights failed")
    return w[:n]


def num_threads() -> int:
    return int(load().oracle_num_threads())


def run_workload(wl, tokens: Optional[Sequence[int]] = None):
    """Scatter (causal only) then attention for an object with the ``Workload`` fields.
    Returns (k_cache_after, v_cache_after, out, lse)."""
    if wl.kind == "causal":
        kc, vc = kv_scatter(wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens,
                            wl.k_new, wl.v_new, wl.k_cache, wl.v_cache)
    else:
        kc, vc = wl.k_cache, wl.v_cache
    out, lse = attention(wl.kind, wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens,
                         wl.q, kc, vc, wl.softmax_scale, tokens)
    return kc, vc, out, lse
