"""Reference for the KV page migration primitive.  TEST INFRASTRUCTURE ONLY.

Appendix B.5 of the paper: when an instance is scaled, a request's KV cache is copied to another GPU
exactly (the error of every tensor is zero) and the copy is verified with checksums.  The part of that
which one GPU can show is written out here with numpy and zlib: a request's pages are gathered from the
pools into a contiguous staging buffer (what would travel over the link), a checksum is taken per page,
and on the other side the staging buffer is scattered into whatever free pages the destination pool has,
checksums taken again.

Readings where the paper is silent: the unit of transfer is one page of both pools, laid out in the
staging buffer as the page's K bytes (all KV heads) followed by its V bytes; the checksum is Adler-32
(RFC 1950) over those bytes, one 32-bit value per page.
Nothing in the product package imports this file and it imports nothing from the product package.
"""
from __future__ import annotations

import zlib
from typing import Tuple

import numpy as np


def pack(k_cache: np.ndarray, v_cache: np.ndarray, page_ids) -> Tuple[np.ndarray, np.ndarray]:
    """Pools [num_pages][...] (any dtype) -> (staging uint8 [n][2 * page_bytes], checksums uint32 [n])."""
    rows, sums = [], []
    for p in np.asarray(page_ids, dtype=np.int64).tolist():
        data = k_cache[p].tobytes() + v_cache[p].tobytes()
        rows.append(np.frombuffer(data, dtype=np.uint8))
        sums.append(zlib.adler32(data))
    n_bytes = k_cache[0].nbytes + v_cache[0].nbytes
    staging = np.stack(rows) if rows else np.zeros((0, n_bytes), dtype=np.uint8)
    return staging, np.asarray(sums, dtype=np.uint32)


def unpack(staging: np.ndarray, page_ids, k_cache: np.ndarray, v_cache: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Staging rows into the given pages of copies of the pools; returns (k_cache, v_cache, checksums of the
    rows as received)."""
    k_out, v_out = k_cache.copy(), v_cache.copy()
    page_bytes = k_cache[0].nbytes
    sums = []
    for row, p in zip(staging, np.asarray(page_ids, dtype=np.int64).tolist()):
        data = row.tobytes()
        k_out[p] = np.frombuffer(data[:page_bytes], dtype=k_cache.dtype).reshape(k_cache.shape[1:])
        v_out[p] = np.frombuffer(data[page_bytes:], dtype=v_cache.dtype).reshape(v_cache.shape[1:])
        sums.append(zlib.adler32(data))
    return k_out, v_out, np.asarray(sums, dtype=np.uint32)
