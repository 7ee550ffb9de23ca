"""Invariants of the method checked on the CPU oracle with the named workloads at reduced size."""
import numpy as np
import pytest

import oracle
from paper_2507_10069_amd import workloads as W


def _run(wl, tokens=None):
    return oracle.run_workload(wl, tokens)


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 16), (3, 64), (4, 32), (5, 32)])
def test_configs_run_and_are_convex_combinations(cfg, shrink):
    wl = W.config(cfg, shrink)
    kc, vc, out, lse = _run(wl)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    # every output coordinate lies between the extremes of the values that exist in the pool
    vals = W.bf16_bits_to_f32(vc) if wl.dtype == "bf16" else vc
    valid = vals[vals < 1e29]
    assert out.min() >= valid.min() - 1e-9 and out.max() <= valid.max() + 1e-9


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 16), (4, 32), (5, 32)])
def test_page_permutation_invariance_is_bitwise(cfg, shrink):
    """I3: relabelling physical pages consistently in pool and table changes nothing."""
    wl = W.config(cfg, shrink)
    _, _, out, lse = _run(wl)
    rng = np.random.default_rng(5)
    perm = rng.permutation(wl.num_pages)          # old id -> new id
    wl2 = W.config(cfg, shrink)
    wl2.k_cache = np.empty_like(wl.k_cache)
    wl2.v_cache = np.empty_like(wl.v_cache)
    wl2.k_cache[perm] = wl.k_cache
    wl2.v_cache[perm] = wl.v_cache
    wl2.page_table = np.where(wl.page_table >= 0, perm[np.maximum(wl.page_table, 0)], -1).astype(np.int32)
    _, _, out2, lse2 = _run(wl2)
    assert out.tobytes() == out2.tobytes() and lse.tobytes() == lse2.tobytes()


def test_chunked_prefill_equals_single_prefill():
    """Prefilling N tokens in two calls (the first chunk becomes cached prefix) gives the same rows
    (Section 2.2, chunked prefill; Appendix B.7)."""
    wl = W.build_workload("t", "causal", "bf16", 77, num_q_heads=4, num_kv_heads=2, head_dim=16, page_size=16,
                          prefix_lens=[21, 0], new_lens=[30, 19])
    kc, vc, out, lse = _run(wl)
    n1 = np.array([11, 7], np.int32)
    n2 = wl.new_lens - n1
    cu = wl.cu_new_lens
    first = np.concatenate([np.arange(cu[r], cu[r] + n1[r]) for r in range(2)])
    second = np.concatenate([np.arange(cu[r] + n1[r], cu[r + 1]) for r in range(2)])
    cu1 = np.array([0, n1[0], n1.sum()], np.int32)
    cu2 = np.array([0, n2[0], n2.sum()], np.int32)
    kc1, vc1 = oracle.kv_scatter(wl.page_table, wl.prefix_lens, n1, cu1, wl.k_new[first], wl.v_new[first],
                                 wl.k_cache, wl.v_cache)
    out1, _ = oracle.attention("causal", wl.page_table, wl.prefix_lens, n1, cu1, wl.q[first], kc1, vc1,
                               wl.softmax_scale)
    p2 = wl.prefix_lens + n1
    kc2, vc2 = oracle.kv_scatter(wl.page_table, p2, n2, cu2, wl.k_new[second], wl.v_new[second], kc1, vc1)
    out2, _ = oracle.attention("causal", wl.page_table, p2, n2, cu2, wl.q[second], kc2, vc2, wl.softmax_scale)
    assert kc2.tobytes() == kc.tobytes() and vc2.tobytes() == vc.tobytes()
    assert out1.tobytes() == out[first].tobytes() and out2.tobytes() == out[second].tobytes()


def test_batch_order_is_irrelevant():
    wl = W.config(4, 64)
    _, _, out, _ = _run(wl)
    order = np.random.default_rng(9).permutation(wl.num_reqs)
    cu = wl.cu_new_lens
    rows = np.concatenate([np.arange(cu[r], cu[r + 1]) for r in order])
    new = wl.new_lens[order]
    cu2 = np.zeros_like(cu)
    cu2[1:] = np.cumsum(new)
    kc, vc = oracle.kv_scatter(wl.page_table[order], wl.prefix_lens[order], new, cu2, wl.k_new[rows],
                               wl.v_new[rows], wl.k_cache, wl.v_cache)
    out2, _ = oracle.attention("causal", wl.page_table[order], wl.prefix_lens[order], new, cu2, wl.q[rows],
                               kc, vc, wl.softmax_scale)
    assert out2.tobytes() == out[rows].tobytes()


def test_shared_pages_equal_private_copies():
    """Requests whose prefix lives in common physical pages get what they would get from private copies."""
    wl = W.config(2, 16)
    _, _, out, _ = _run(wl)
    # give request 1..3 and 5..7 private copies of the shared prefix pages
    n_shared = int(wl.prefix_lens[0]) // wl.page_size
    extra = 6 * n_shared
    kc = np.concatenate([wl.k_cache, np.zeros((extra,) + wl.k_cache.shape[1:], wl.k_cache.dtype)])
    vc = np.concatenate([wl.v_cache, np.zeros((extra,) + wl.v_cache.shape[1:], wl.v_cache.dtype)])
    pt = wl.page_table.copy()
    nxt = wl.num_pages
    for r in (1, 2, 3, 5, 6, 7):
        for lp in range(n_shared):
            kc[nxt] = wl.k_cache[pt[r, lp]]
            vc[nxt] = wl.v_cache[pt[r, lp]]
            pt[r, lp] = nxt
            nxt += 1
    assert len(set(pt[0, :n_shared]) & set(pt[1, :n_shared])) == 0
    kc2, vc2 = oracle.kv_scatter(pt, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, wl.k_new, wl.v_new, kc, vc)
    out2, _ = oracle.attention("causal", pt, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, wl.q, kc2, vc2,
                               wl.softmax_scale)
    assert out2.tobytes() == out.tobytes()


def test_token_subset_matches_full_run():
    wl = W.config(2, 16)
    _, _, out, lse = _run(wl)
    pick = [0, 5, wl.total_new_tokens - 1, 17]
    _, _, out_s, lse_s = _run(wl, pick)
    assert out_s.tobytes() == out[pick].tobytes() and lse_s.tobytes() == lse[pick].tobytes()
