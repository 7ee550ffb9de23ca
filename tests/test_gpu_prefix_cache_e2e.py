"""End to end on the GPU: the host-side prefix cache decides prefix lengths and pages, the device path
scatters the new tokens' K/V and attends over cached + new tokens, and the result must equal ordinary causal
attention over every request's WHOLE sequence (Appendix B.7: prefilling the un-cached rest against cached
K/V is identical to prefilling everything), computed densely in fp64 by the oracle, which knows nothing of
pages or caches.  The pool is small enough that pages are evicted and reused for other content, requests
overlap in time, share prefixes (a system prompt, an image), duplicate each other, and decode a few tokens.

A token's Q/K/V rows are a fixed function of (token id, position): all the test needs of a model layer is that
equal prefixes give equal rows."""
from __future__ import annotations

import numpy as np
import pytest

from oracle import bruteforce
from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import prefix_cache as PC

pytestmark = pytest.mark.gpu

H, HKV, D, PS = 8, 2, 128, 16
NUM_PAGES, MAX_PAGES = 22, 24
SCALE = 1.0 / np.sqrt(D)
TOL_MAX, TOL_MEAN = 2e-2, 2e-3
UNITS_SEEN = []


def _bf16_round(x: np.ndarray) -> np.ndarray:
    """fp32 -> nearest-even bf16, returned as fp32 values."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    u = ((u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000).astype(np.uint32)
    return u.view(np.float32)


class _Rows:
    """Q/K/V rows of a token as a function of (token id, position)."""

    def __init__(self, seed):
        rng = np.random.default_rng(seed)
        self.tab = {n: (_bf16_round(rng.standard_normal((97, h, D)) * s), _bf16_round(rng.standard_normal((512, h, D)) * s))
                    for n, h, s in (("q", H, 1.0), ("k", HKV, 1.0), ("v", HKV, 1.0))}

    def rows(self, name, tokens, start=0):
        tok = np.asarray(tokens, dtype=np.int64)
        by_id, by_pos = self.tab[name]
        pos = np.arange(start, start + tok.size)
        return _bf16_round(by_id[tok % 97] * 0.7 + by_pos[pos] * 0.7)


def _dev_bf16(x_f32, torch):
    return torch.from_numpy(np.ascontiguousarray(x_f32, dtype=np.float32)).to("cuda:0").to(torch.bfloat16)


def _run_batch(torch, pools, rows, reqs, decode=False):
    """reqs: list of (tokens, page_table_row, prefix_len).  Scatter + attention for the tokens from prefix_len
    on; returns one [n_new][H][D] float64 array per request."""
    k_pool, v_pool = pools
    new_lens = np.array([len(t) - pl for t, _, pl in reqs], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(new_lens)]).astype(np.int32)
    T = int(cu[-1])
    q = np.concatenate([rows.rows("q", t[pl:], pl) for t, _, pl in reqs])
    k_new = np.concatenate([rows.rows("k", t[pl:], pl) for t, _, pl in reqs])
    v_new = np.concatenate([rows.rows("v", t[pl:], pl) for t, _, pl in reqs])
    pt = torch.from_numpy(np.stack([r for _, r, _ in reqs]).astype(np.int32)).to("cuda:0")
    pl_d = torch.tensor([pl for _, _, pl in reqs], dtype=torch.int32, device="cuda:0")
    nl_d = torch.from_numpy(new_lens).to("cuda:0")
    cu_d = torch.from_numpy(cu).to("cuda:0")
    batch = B.make_batch(num_reqs=len(reqs), num_q_heads=H, num_kv_heads=HKV, head_dim=D, page_size=PS,
                         num_pages=NUM_PAGES, max_pages_per_req=MAX_PAGES, total_new_tokens=T,
                         max_new_len=int(new_lens.max()), dtype="bf16", softmax_scale=SCALE, page_table=pt,
                         prefix_lens=pl_d, new_lens=nl_d, cu_new_lens=cu_d)
    assert B.emm_validate_batch_host(batch, pt.cpu().numpy(), pl_d.cpu().numpy(), new_lens, cu, True) == B.EMM_OK
    q_d, k_d, v_d = _dev_bf16(q, torch), _dev_bf16(k_new, torch), _dev_bf16(v_new, torch)
    out = torch.empty_like(q_d)
    ws = torch.empty(max(B.emm_prefill_attn_workspace_size(batch), 16), dtype=torch.uint8, device="cuda:0")
    B.emm_kv_scatter(batch, k_d, v_d, k_pool, v_pool)
    (B.emm_decode_attn if decode else B.emm_prefill_attn)(batch, q_d, k_pool, v_pool, out, None, ws)
    torch.cuda.synchronize()
    o = out.to(torch.float32).cpu().numpy().astype(np.float64)
    if decode:
        # the same step with the pages that the cache made common to several requests read once per unit
        plan = B.emm_shared_prefix_plan_host(batch, pt.cpu().numpy(), pl_d.cpu().numpy(), new_lens)
        UNITS_SEEN.append(plan["num_units"])
        arrays = {k: torch.from_numpy(np.ascontiguousarray(v if len(v) else np.zeros(1, np.int32))).to("cuda:0")
                  for k, v in plan.items() if isinstance(v, np.ndarray)}
        sp = B.make_shared_prefix(plan["num_units"], planned_tiles=plan["planned_tiles"],
                                  max_own_tiles=plan["max_own_tiles"], max_unit_tiles=plan["max_unit_tiles"], **arrays)
        ws2 = torch.empty(max(B.emm_decode_attn_shared_workspace_size(batch, sp), 16), dtype=torch.uint8, device="cuda:0")
        out2 = torch.zeros_like(q_d)
        B.emm_decode_attn_shared(batch, sp, q_d, k_pool, v_pool, out2, None, ws2)
        torch.cuda.synchronize()
        o2 = out2.to(torch.float32).cpu().numpy().astype(np.float64)
        assert np.abs(o2 - o).max() <= TOL_MAX
        o = o2                                           # the caller checks this one against the oracle
    return [o[cu[i]:cu[i + 1]] for i in range(len(reqs))]


def _expect(rows, tokens, first):
    n = len(tokens)
    out, _ = bruteforce.dense_causal(rows.rows("q", tokens).astype(np.float64), rows.rows("k", tokens).astype(np.float64),
                                     rows.rows("v", tokens).astype(np.float64), SCALE)
    return out[first:n]


def _check(got, want, what):
    err = np.abs(got - want)
    assert err.max() <= TOL_MAX and err.mean() <= TOL_MEAN, (what, err.max(), err.mean())


def test_cached_prefixes_give_the_answers_of_full_prefill():
    import torch
    rng = np.random.default_rng(4242)
    rows = _Rows(7)
    # sentinel-filled pools: a stale or wrong page shows up as a large error, not as a small one
    pools = tuple(torch.full((NUM_PAGES, HKV, PS, D), 1e30, dtype=torch.bfloat16, device="cuda:0") for _ in range(2))
    cache = PC.emm_prefix_cache_create(NUM_PAGES, PS)
    system = rng.integers(0, 30000, 23).tolist()
    images = [PC.emm_mm_token_ids(PC.emm_mm_content_hash(b"picture-%d" % i), n).tolist() for i, n in enumerate((70, 45, 100))]

    def question(n):
        return rng.integers(0, 30000, n).tolist()

    hits = 0
    waves = [
        [system + images[0] + question(9)],                                   # cold
        [system + images[0] + question(14), system + images[0] + question(5)],    # share system + image 0
        [system + images[1] + question(30), system + question(40)],           # share the system prompt's full page
        [system + images[2] + question(11)],                                  # 134 tokens: evicts older nodes
        [system + images[0] + question(9), system + images[0] + question(9)],     # duplicates in one batch
        [system + images[2] + question(3), system + images[1] + question(3)],
    ]
    for w, wave in enumerate(waves):
        begun = []
        for tokens in wave:
            row, pl, rid = PC.emm_prefix_cache_begin(cache, tokens, MAX_PAGES)
            assert pl % PS == 0 and pl < len(tokens)
            hits += pl
            begun.append((tokens, row, pl, rid))
        outs = _run_batch(torch, pools, rows, [(t, r, pl) for t, r, pl, _ in begun])
        for (tokens, row, pl, rid), got in zip(begun, outs):
            _check(got, _expect(rows, tokens, pl), ("prefill", w, pl))
            PC.emm_prefix_cache_commit(cache, rid, len(tokens))
        # decode three tokens for every request of the wave, one step at a time, all requests in one batch
        state = [[list(t), rid] for t, _, _, rid in begun]
        for step in range(3):
            reqs = []
            for st in state:
                nxt = int(rng.integers(0, 30000))
                row = PC.emm_prefix_cache_append(cache, st[1], [nxt], MAX_PAGES)
                st[0].append(nxt)
                reqs.append((st[0], row, len(st[0]) - 1))
            outs = _run_batch(torch, pools, rows, reqs, decode=True)
            for (tokens, _, pl), got, st in zip(reqs, outs, state):
                _check(got, _expect(rows, tokens, pl), ("decode", w, step))
                PC.emm_prefix_cache_commit(cache, st[1], len(tokens))
        for st in state:
            PC.emm_prefix_cache_release(cache, st[1])
    st = PC.emm_prefix_cache_get_stats(cache)
    assert max(UNITS_SEEN) >= 1                      # requests of a wave that hit the same cached pages formed units
    assert hits > 0 and st["hit_tokens"] == hits
    assert st["evictions"] > 0                       # pages were reused for other content along the way
    assert st["live_requests"] == 0 and st["free_pages"] + st["cached_pages"] == NUM_PAGES
    PC.emm_prefix_cache_destroy(cache)


def test_chunked_prefill_equals_one_shot():
    """Section 2.2 (chunked prefill): a long prompt prefilled in segments, each segment attending to the K/V that
    the earlier segments left in the pool, gives the rows of one prefill over the whole prompt.  The segment
    boundaries are not page aligned, and two requests of different lengths run in the same batches."""
    import torch
    rng = np.random.default_rng(99)
    rows = _Rows(11)
    pools = tuple(torch.full((NUM_PAGES * 4, HKV, PS, D), 1e30, dtype=torch.bfloat16, device="cuda:0") for _ in range(2))
    prompts = [rng.integers(0, 30000, 500).tolist(), rng.integers(0, 30000, 333).tolist()]
    perm = rng.permutation(NUM_PAGES * 4)
    tables = []
    used = 0
    for p in prompts:
        n_pages = -(-len(p) // PS)
        row = np.full(MAX_PAGES * 2, -1, dtype=np.int32)
        row[:n_pages] = perm[used:used + n_pages]
        used += n_pages
        tables.append(row)
    bounds = [[0, 300, 417, 500], [0, 150, 151, 333]]        # three segments each; the second one's middle segment is one token
    got = [[], []]
    for seg in range(3):
        reqs = [(prompts[i][:bounds[i][seg + 1]], tables[i], bounds[i][seg]) for i in range(2)]
        outs = _run_batch_wide(torch, pools, rows, reqs)
        for i in range(2):
            got[i].append(outs[i])
    for i in range(2):
        _check(np.concatenate(got[i]), _expect(rows, prompts[i], 0), ("chunked", i))


def _run_batch_wide(torch, pools, rows, reqs):
    """As _run_batch, for page-table rows of 2 * MAX_PAGES entries over a pool of 4 * NUM_PAGES pages."""
    k_pool, v_pool = pools
    new_lens = np.array([len(t) - pl for t, _, pl in reqs], dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(new_lens)]).astype(np.int32)
    q = np.concatenate([rows.rows("q", t[pl:], pl) for t, _, pl in reqs])
    k_new = np.concatenate([rows.rows("k", t[pl:], pl) for t, _, pl in reqs])
    v_new = np.concatenate([rows.rows("v", t[pl:], pl) for t, _, pl in reqs])
    pt = torch.from_numpy(np.stack([r for _, r, _ in reqs]).astype(np.int32)).to("cuda:0")
    pl_d = torch.tensor([pl for _, _, pl in reqs], dtype=torch.int32, device="cuda:0")
    nl_d = torch.from_numpy(new_lens).to("cuda:0")          # held until the kernels have run: the batch stores addresses
    cu_d = torch.from_numpy(cu).to("cuda:0")
    batch = B.make_batch(num_reqs=len(reqs), num_q_heads=H, num_kv_heads=HKV, head_dim=D, page_size=PS,
                         num_pages=NUM_PAGES * 4, max_pages_per_req=MAX_PAGES * 2, total_new_tokens=int(cu[-1]),
                         max_new_len=int(new_lens.max()), dtype="bf16", softmax_scale=SCALE, page_table=pt,
                         prefix_lens=pl_d, new_lens=nl_d, cu_new_lens=cu_d)
    assert B.emm_validate_batch_host(batch, pt.cpu().numpy(), pl_d.cpu().numpy(), new_lens, cu, True) == B.EMM_OK
    q_d, k_d, v_d = _dev_bf16(q, torch), _dev_bf16(k_new, torch), _dev_bf16(v_new, torch)
    out = torch.empty_like(q_d)
    ws = torch.empty(max(B.emm_prefill_attn_workspace_size(batch), 16), dtype=torch.uint8, device="cuda:0")
    B.emm_kv_scatter(batch, k_d, v_d, k_pool, v_pool)
    B.emm_prefill_attn(batch, q_d, k_pool, v_pool, out, None, ws)
    torch.cuda.synchronize()
    o = out.to(torch.float32).cpu().numpy().astype(np.float64)
    return [o[cu[i]:cu[i + 1]] for i in range(len(reqs))]
