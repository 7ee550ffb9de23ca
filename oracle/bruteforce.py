"""Dense recomputation with no cache and no pages (numpy, fp64).  TEST INFRASTRUCTURE ONLY.

Appendix B.7 states that prefilling the un-cached suffix against cached K/V equals prefilling the
whole sequence.  This file is the right-hand side of that equality: it takes one request's *whole*
sequence as contiguous arrays, forms the full causal score matrix, applies a row-wise softmax and
multiplies by V.  It never sees a page table, a prefix length or a pool, so an indexing mistake in
``oracle.c`` (page lookup, prefix offset, causal boundary, head grouping) cannot be repeated here.
"""
from __future__ import annotations

import numpy as np


def dense_causal(q_full: np.ndarray, k_full: np.ndarray, v_full: np.ndarray, scale: float):
    """q_full [L][H][d], k_full/v_full [L][Hkv][d] (float64).  Returns (out [L][H][d], lse [L][H])
    of ordinary causal softmax attention over the L tokens; query head h uses KV head h // (H // Hkv)."""
    L, H, d = q_full.shape
    Hkv = k_full.shape[1]
    G = H // Hkv
    k_rep = np.repeat(k_full, G, axis=1)            # [L][H][d]: KV head of every query head
    v_rep = np.repeat(v_full, G, axis=1)
    s = scale * np.einsum("ihc,jhc->hij", q_full, k_rep)     # [H][L][L]
    visible = np.tril(np.ones((L, L), dtype=bool))
    s = np.where(visible[None], s, -np.inf)
    m = s.max(axis=2, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=2, keepdims=True)
    out = np.einsum("hij,jhc->ihc", e / z, v_rep)
    lse = (m + np.log(z))[:, :, 0].T
    return out, lse


def dense_full(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float):
    """Unmasked attention: q [Nq][H][d] over k/v [L][Hkv][d] (float64).  Returns (out, lse)."""
    Nq, H, d = q.shape
    G = H // k.shape[1]
    k_rep = np.repeat(k, G, axis=1)
    v_rep = np.repeat(v, G, axis=1)
    s = scale * np.einsum("ihc,jhc->hij", q, k_rep)
    m = s.max(axis=2, keepdims=True)
    e = np.exp(s - m)
    z = e.sum(axis=2, keepdims=True)
    out = np.einsum("hij,jhc->ihc", e / z, v_rep)
    lse = (m + np.log(z))[:, :, 0].T
    return out, lse
