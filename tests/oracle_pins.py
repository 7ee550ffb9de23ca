"""Pins for the CPU oracle, written as plain functions of an oracle library handle so that the
same checks can be run against deliberately broken copies of ``oracle.c`` (tests/test_oracle_mutants.py).

Each pin compares the oracle with something that is not the oracle: a dense recomputation that
knows no pages or cache, a closed form, a hand-derived fixture, or a scipy routine."""
from __future__ import annotations

import json
import math
import os

import numpy as np
import scipy.special

import oracle
from oracle import bruteforce
from helpers import as_f64, page_dense, store, sentinel

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
LN2 = math.log(2.0)


def _dense_case(rng, P, N, ps, H, Hkv, d, dtype, lib, scale=None):
    """Prefix-cached oracle (pages, scatter) vs dense causal recomputation of the whole sequence."""
    L = P + N
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    q_full = store(rng.standard_normal((L, H, d), dtype=np.float32), dtype)
    k_full = store(rng.standard_normal((L, Hkv, d), dtype=np.float32), dtype)
    v_full = store(rng.standard_normal((L, Hkv, d), dtype=np.float32), dtype)
    pt, kc, vc, k_new, v_new, cu, new_lens = page_dense(rng, [k_full], [v_full], [P], ps, dtype)
    prefix = np.array([P], np.int32)
    kc2, vc2 = oracle.kv_scatter(pt, prefix, new_lens, cu, k_new, v_new, kc, vc, lib=lib)
    out, lse = oracle.attention("causal", pt, prefix, new_lens, cu, q_full[P:], kc2, vc2, scale, lib=lib)
    ref_out, ref_lse = bruteforce.dense_causal(as_f64(q_full), as_f64(k_full), as_f64(v_full), scale)
    np.testing.assert_allclose(out, ref_out[P:], rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_lse[P:], rtol=0, atol=1e-12)


def pin_dense_recompute_sweep(lib):
    """I1: cached prefix + remaining prefill == full dense prefill (Appendix B.7), tiny sweep."""
    rng = np.random.default_rng(11)
    for P in (0, 1, 15, 16, 17, 33):
        for N in (1, 2, 16, 17):
            for ps in (1, 4, 16):
                H, Hkv = ((1, 1), (4, 1), (7, 1), (4, 2), (6, 3))[(P + N + ps) % 5]
                d = (8, 64)[(P + N) % 2]
                dtype = ("f32", "bf16")[(P + ps) % 2]
                _dense_case(rng, P, N, ps, H, Hkv, d, dtype, lib)


def pin_dense_recompute_large_pages(lib):
    """The same identity with pages of 32 and 64 tokens (the device kernels take pages up to 256): prefixes and
    suffixes that end inside, at and just past a page."""
    rng = np.random.default_rng(14)
    for P in (0, 31, 32, 65, 130):
        for N in (1, 33, 70):
            for ps in (32, 64):
                H, Hkv = ((4, 1), (4, 2), (6, 3))[(P + N + ps) % 3]
                _dense_case(rng, P, N, ps, H, Hkv, 8, ("f32", "bf16")[(P + N) % 2], lib)


def pin_dense_recompute_gqa(lib):
    """Head grouping with several KV heads and a group size that is not a power of two."""
    rng = np.random.default_rng(12)
    _dense_case(rng, 19, 9, 4, 6, 2, 8, "f32", lib)
    _dense_case(rng, 5, 21, 16, 14, 2, 16, "bf16", lib)
    _dense_case(rng, 32, 8, 16, 8, 8, 8, "f32", lib)


def pin_dense_recompute_batch(lib):
    """Several requests in one batch (packed rows, one page table row each), incl. an empty one."""
    rng = np.random.default_rng(13)
    H, Hkv, d, ps, dtype = 4, 2, 8, 4, "f32"
    P = [5, 0, 16, 9]
    N = [3, 7, 0, 6]
    qs, ks, vs = [], [], []
    for p, n in zip(P, N):
        qs.append(store(rng.standard_normal((p + n, H, d), dtype=np.float32), dtype))
        ks.append(store(rng.standard_normal((p + n, Hkv, d), dtype=np.float32), dtype))
        vs.append(store(rng.standard_normal((p + n, Hkv, d), dtype=np.float32), dtype))
    pt, kc, vc, k_new, v_new, cu, new_lens = page_dense(rng, ks, vs, P, ps, dtype)
    prefix = np.array(P, np.int32)
    kc2, vc2 = oracle.kv_scatter(pt, prefix, new_lens, cu, k_new, v_new, kc, vc, lib=lib)
    q = np.concatenate([qs[r][P[r]:] for r in range(4)], axis=0)
    out, lse = oracle.attention("causal", pt, prefix, new_lens, cu, q, kc2, vc2, 0.3, lib=lib)
    for r in range(4):
        ref_out, ref_lse = bruteforce.dense_causal(as_f64(qs[r]), as_f64(ks[r]), as_f64(vs[r]), 0.3)
        np.testing.assert_allclose(out[cu[r]:cu[r + 1]], ref_out[P[r]:], rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[cu[r]:cu[r + 1]], ref_lse[P[r]:], rtol=0, atol=1e-12)


def pin_cross_dense(lib):
    """Cross-attention (Section 2.1): unmasked attention over the cached keys, ragged last page."""
    rng = np.random.default_rng(14)
    H, Hkv, d, ps, dtype = 6, 2, 8, 4, "bf16"
    L = [13, 4, 0, 7]
    Nq = [5, 2, 3, 1]
    ks = [store(rng.standard_normal((l, Hkv, d), dtype=np.float32), dtype) for l in L]
    vs = [store(rng.standard_normal((l, Hkv, d), dtype=np.float32), dtype) for l in L]
    pt, kc, vc, _, _, _, _ = page_dense(rng, ks, vs, L, ps, dtype, causal=False)
    cu = np.zeros(5, np.int32)
    cu[1:] = np.cumsum(Nq)
    q = store(rng.standard_normal((int(cu[-1]), H, d), dtype=np.float32), dtype)
    out, lse = oracle.attention("cross", pt, np.array(L, np.int32), np.array(Nq, np.int32), cu, q, kc, vc,
                                0.41, lib=lib)
    for r in range(4):
        rows = slice(int(cu[r]), int(cu[r + 1]))
        if L[r] == 0:
            assert np.all(out[rows] == 0.0) and np.all(np.isneginf(lse[rows]))
            continue
        ref_out, ref_lse = bruteforce.dense_full(as_f64(q[rows]), as_f64(ks[r]), as_f64(vs[r]), 0.41)
        np.testing.assert_allclose(out[rows], ref_out, rtol=0, atol=1e-12)
        np.testing.assert_allclose(lse[rows], ref_lse, rtol=0, atol=1e-12)


def _single(rng, P, N, ps, H, Hkv, d, q, k, v, scale, lib, kind="causal"):
    """q [N][H][d], k/v [P+N][Hkv][d] float32 -> oracle rows (fp32 storage)."""
    pt, kc, vc, k_new, v_new, cu, new_lens = page_dense(rng, [k.astype(np.float32)], [v.astype(np.float32)],
                                                        [P], ps, "f32")
    prefix = np.array([P], np.int32)
    kc2, vc2 = oracle.kv_scatter(pt, prefix, new_lens, cu, k_new, v_new, kc, vc, lib=lib)
    return oracle.attention(kind, pt, prefix, new_lens, cu, q.astype(np.float32), kc2, vc2, scale, lib=lib)


def pin_closed_forms(lib):
    rng = np.random.default_rng(15)
    P, N, ps, H, Hkv, d = 7, 6, 4, 4, 2, 8
    L = P + N
    q = rng.standard_normal((N, H, d)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    # zero keys: uniform weights -> running mean of V over the attended range, lse = ln(len)
    out, lse = _single(rng, P, N, ps, H, Hkv, d, q, np.zeros((L, Hkv, d), np.float32), v, 0.7, lib)
    for j in range(N):
        for h in range(H):
            want = v[:P + j + 1, h // 2].astype(np.float64).mean(axis=0)
            np.testing.assert_allclose(out[j, h], want, rtol=0, atol=1e-13)
            assert abs(lse[j, h] - math.log(P + j + 1)) < 1e-13
    # constant V: the weights sum to one, so the output is that constant
    k = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    out, _ = _single(rng, P, N, ps, H, Hkv, d, q, k, np.full((L, Hkv, d), 1.0, np.float32), 0.7, lib)
    np.testing.assert_allclose(out, 1.0, rtol=0, atol=1e-14)
    # no prefix, first token: it attends to itself only
    out, lse = _single(rng, 0, 3, ps, H, Hkv, d, q[:3], k[:3], v[:3], 0.7, lib)
    for h in range(H):
        np.testing.assert_array_equal(out[0, h], v[0, h // 2].astype(np.float64))
        want = 0.7 * float(np.dot(q[0, h].astype(np.float64), k[0, h // 2].astype(np.float64)))
        assert abs(lse[0, h] - want) < 1e-13
    # a dominant key (score ~ +2000 above the rest, far beyond exp's fp64 range without the max
    # subtraction): the output is that key's value
    k_dom = 0.01 * k.copy()
    q_one = np.ones((N, H, d), np.float32)
    k_dom[3] = 250.0                                     # key 3 lies in the prefix: visible to all rows
    out, _ = _single(rng, P, N, ps, H, Hkv, d, q_one, k_dom, v, 1.0, lib)
    for h in range(H):
        np.testing.assert_allclose(out[:, h], np.broadcast_to(v[3, h // 2].astype(np.float64), (N, d)),
                                   rtol=0, atol=1e-12)
    # adding one vector to every key shifts all scores of a row equally: output unchanged
    shift = rng.standard_normal((1, 1, d)).astype(np.float32)
    k_exact = np.round(k * 8) / 8                       # keep k + shift exactly representable
    shift = np.round(shift * 8) / 8
    out_a, lse_a = _single(rng, P, N, ps, H, Hkv, d, q, k_exact, v, 0.7, lib)
    out_b, lse_b = _single(rng, P, N, ps, H, Hkv, d, q, k_exact + shift, v, 0.7, lib)
    np.testing.assert_allclose(out_a, out_b, rtol=0, atol=1e-12)
    for j in range(N):
        for h in range(H):
            delta = 0.7 * float(np.dot(q[j, h].astype(np.float64), shift[0, 0].astype(np.float64)))
            assert abs((lse_b[j, h] - lse_a[j, h]) - delta) < 1e-12


def pin_golden_causal(lib):
    with open(os.path.join(GOLDEN, "causal_powers_of_two.json")) as f:
        g = json.load(f)
    rng = np.random.default_rng(16)
    P, N, ps = g["prefix_len"], g["new_len"], g["page_size"]
    q = np.array(g["q"], np.float32).reshape(N, 1, 1)
    k = np.array(g["k"], np.float32).reshape(P + N, 1, 1)
    v = np.array(g["v"], np.float32).reshape(P + N, 1, 1)
    out, lse = _single(rng, P, N, ps, 1, 1, 1, q, k, v, LN2, lib)
    for j in range(N):
        assert abs(out[j, 0, 0] - g["expected_out_num"][j] / g["expected_out_den"][j]) < 1e-14
        assert abs(math.exp(lse[j, 0]) - g["expected_expm_lse"][j]) < 1e-12


def pin_golden_gqa(lib):
    with open(os.path.join(GOLDEN, "gqa_two_kv_heads.json")) as f:
        g = json.load(f)
    rng = np.random.default_rng(17)
    k = np.array(g["k"], np.float32)                    # [token][kv head][d]
    v = np.array(g["v"], np.float32)
    q = np.broadcast_to(np.array(g["q_all"], np.float32), (2, 4, 2)).copy()
    out, lse = _single(rng, 0, 2, g["page_size"], 4, 2, 2, q, k, v, LN2, lib)
    np.testing.assert_allclose(out[0], np.array(g["expected_token0"]), rtol=0, atol=1e-14)
    np.testing.assert_allclose(out[1], np.array(g["expected_token1"]), rtol=0, atol=1e-14)
    np.testing.assert_allclose(np.exp(lse[1]), np.array(g["expected_expm_lse_token1"]), rtol=0, atol=1e-13)


def pin_golden_cross(lib):
    with open(os.path.join(GOLDEN, "cross_partial_page.json")) as f:
        g = json.load(f)
    rng = np.random.default_rng(18)
    L, ps = g["kv_len"], g["page_size"]
    k = np.array(g["k"], np.float32).reshape(L, 1, 1)
    v = np.array(g["v"], np.float32).reshape(L, 1, 1)
    pt, kc, vc, _, _, _, _ = page_dense(rng, [k], [v], [L], ps, "f32", causal=False)
    q = np.array(g["q"], np.float32).reshape(3, 1, 1)
    cu = np.array([0, 3], np.int32)
    out, lse = oracle.attention("cross", pt, np.array([L], np.int32), np.array([3], np.int32), cu, q, kc, vc,
                                LN2, lib=lib)
    for j in range(3):
        assert abs(out[j, 0, 0] - g["expected_out_num"][j] / g["expected_out_den"][j]) < 1e-13
        assert abs(math.exp(lse[j, 0]) - g["expected_expm_lse_num"][j] / g["expected_expm_lse_den"][j]) < 1e-13


def pin_scipy_page_size_one(lib):
    """With page size 1 and an identity page table the oracle is textbook dense attention; scipy's
    softmax / logsumexp give a third opinion on one head."""
    rng = np.random.default_rng(19)
    L, d = 23, 16
    q = rng.standard_normal((L, 1, d)).astype(np.float32)
    k = rng.standard_normal((L, 1, d)).astype(np.float32)
    v = rng.standard_normal((L, 1, d)).astype(np.float32)
    pt = np.arange(L, dtype=np.int32).reshape(1, L)
    kc = np.full((L, 1, 1, d), sentinel("f32"), np.float32)
    vc = kc.copy()
    cu = np.array([0, L], np.int32)
    zero, full = np.array([0], np.int32), np.array([L], np.int32)
    kc2, vc2 = oracle.kv_scatter(pt, zero, full, cu, k, v, kc, vc, lib=lib)
    np.testing.assert_array_equal(kc2[:, 0, 0, :], k[:, 0, :])
    out, lse = oracle.attention("causal", pt, zero, full, cu, q, kc2, vc2, 0.25, lib=lib)
    s = 0.25 * (q[:, 0].astype(np.float64) @ k[:, 0].astype(np.float64).T)
    s = np.where(np.tril(np.ones((L, L), bool)), s, -np.inf)
    np.testing.assert_allclose(out[:, 0], scipy.special.softmax(s, axis=1) @ v[:, 0].astype(np.float64),
                               rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse[:, 0], scipy.special.logsumexp(s, axis=1), rtol=0, atol=1e-13)


def pin_scatter_bytes(lib):
    """I4: the scatter writes exactly the new tokens' slots, byte for byte, and nothing else.
    Expected pool built here by direct numpy indexing from the dense sequences."""
    rng = np.random.default_rng(20)
    for dtype in ("f32", "bf16"):
        Hkv, d, ps = 3, 8, 4
        P, N = [6, 0, 8], [5, 9, 0]
        ks = [store(rng.standard_normal((p + n, Hkv, d), dtype=np.float32), dtype) for p, n in zip(P, N)]
        vs = [store(rng.standard_normal((p + n, Hkv, d), dtype=np.float32), dtype) for p, n in zip(P, N)]
        pt, kc, vc, k_new, v_new, cu, new_lens = page_dense(rng, ks, vs, P, ps, dtype)
        kc2, vc2 = oracle.kv_scatter(pt, np.array(P, np.int32), new_lens, cu, k_new, v_new, kc, vc, lib=lib)
        want_k, want_v = kc.copy(), vc.copy()
        for r in range(3):
            for i in range(P[r], P[r] + N[r]):
                want_k[pt[r, i // ps], :, i % ps, :] = ks[r][i]
                want_v[pt[r, i // ps], :, i % ps, :] = vs[r][i]
        assert kc2.tobytes() == want_k.tobytes() and vc2.tobytes() == want_v.tobytes()
        assert (kc2 == sentinel(dtype)).sum() == (want_k == sentinel(dtype)).sum() > 0


def pin_weights_sum_to_one(lib):
    """I2: the normalised softmax weights of a row sum to 1 and reproduce the output row."""
    rng = np.random.default_rng(21)
    P, N, ps, H, Hkv, d = 21, 5, 16, 4, 2, 8
    k = rng.standard_normal((P + N, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((P + N, Hkv, d)).astype(np.float32)
    q = rng.standard_normal((N, H, d)).astype(np.float32)
    pt, kc, vc, k_new, v_new, cu, new_lens = page_dense(rng, [k], [v], [P], ps, "f32")
    prefix = np.array([P], np.int32)
    kc2, vc2 = oracle.kv_scatter(pt, prefix, new_lens, cu, k_new, v_new, kc, vc, lib=lib)
    out, _ = oracle.attention("causal", pt, prefix, new_lens, cu, q, kc2, vc2, 0.5, lib=lib)
    for j in range(N):
        for h in range(H):
            w = oracle.row_weights("causal", pt, prefix, new_lens, cu, q, kc2, vc2, 0.5, j, h, lib=lib)
            assert len(w) == P + j + 1 and abs(w.sum() - 1.0) < 1e-14 and (w >= 0).all()
            s = 0.5 * (k[:P + j + 1, h // 2].astype(np.float64) @ q[j, h].astype(np.float64))
            np.testing.assert_allclose(w, scipy.special.softmax(s), rtol=0, atol=1e-14)
            np.testing.assert_allclose(out[j, h], w @ v[:P + j + 1, h // 2].astype(np.float64), rtol=0, atol=1e-13)


ALL_PINS = [pin_dense_recompute_sweep, pin_dense_recompute_large_pages, pin_dense_recompute_gqa, pin_dense_recompute_batch, pin_cross_dense,
            pin_closed_forms, pin_golden_causal, pin_golden_gqa, pin_golden_cross, pin_scipy_page_size_one,
            pin_scatter_bytes, pin_weights_sum_to_one]
