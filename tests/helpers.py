"""Test-side helpers: page a dense sequence into a pool, widen tensors, error metrics."""
from __future__ import annotations

import numpy as np

from paper_2507_10069_amd import workloads as W


def as_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return W.bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


def store(x_f32: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> storage form of ``dtype`` (float32, or bf16 bit patterns)."""
    return x_f32.astype(np.float32) if dtype == "f32" else W.to_bf16_bits(x_f32)


def sentinel(dtype: str):
    return W.SENTINEL_F32 if dtype == "f32" else W.SENTINEL_BF16_BITS


def page_dense(rng, seqs_k, seqs_v, prefix_lens, page_size, dtype, spare=3, causal=True):
    """Put the first ``prefix_lens[r]`` tokens of each dense sequence ([L_r][Hkv][d], storage form)
    into a sentinel-filled pool through a random page table; return
    (page_table, k_cache, v_cache, k_new, v_new, cu_new_lens, new_lens)."""
    B = len(seqs_k)
    Hkv, d = seqs_k[0].shape[1], seqs_k[0].shape[2]
    total = [len(s) for s in seqs_k]
    pages = [-(-t // page_size) for t in total]
    num_pages = sum(pages) + spare
    perm = rng.permutation(num_pages)
    max_pages = max(1, max(pages))
    pt = np.full((B, max_pages), -1, np.int32)
    np_dtype = np.float32 if dtype == "f32" else np.uint16
    kc = np.full((num_pages, Hkv, page_size, d), sentinel(dtype), np_dtype)
    vc = kc.copy()
    at = 0
    for r in range(B):
        pt[r, :pages[r]] = perm[at:at + pages[r]]
        at += pages[r]
        for i in range(prefix_lens[r]):
            kc[pt[r, i // page_size], :, i % page_size, :] = seqs_k[r][i]
            vc[pt[r, i // page_size], :, i % page_size, :] = seqs_v[r][i]
    new_lens = np.array([total[r] - prefix_lens[r] for r in range(B)], np.int32) if causal \
        else np.zeros(B, np.int32)
    cu = np.zeros(B + 1, np.int32)
    cu[1:] = np.cumsum(new_lens)
    if causal and cu[-1] > 0:
        k_new = np.concatenate([seqs_k[r][prefix_lens[r]:] for r in range(B)], axis=0)
        v_new = np.concatenate([seqs_v[r][prefix_lens[r]:] for r in range(B)], axis=0)
    else:
        k_new = np.zeros((0, Hkv, d), np_dtype)
        v_new = np.zeros((0, Hkv, d), np_dtype)
    return pt, kc, vc, k_new, v_new, cu, new_lens


def err_stats(got_f64: np.ndarray, want_f64: np.ndarray):
    diff = np.abs(got_f64 - want_f64)
    return float(diff.max()) if diff.size else 0.0, float(diff.mean()) if diff.size else 0.0
