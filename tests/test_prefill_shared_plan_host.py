"""Host side of prefill with shared prefixes (Section 3.3: requests of one batch hold the same cached pages): the
planner that finds the sharing groups and builds the two descriptors.  No GPU: the planner is host code.

The checks are the properties any valid plan has (what the members of a group share really is the same pages, the
two passes together cover every request's keys exactly once, nothing is saved that is not there) and small cases
whose answer is known by hand."""
import ctypes

import numpy as np
import pytest

from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import workloads as W


def _batch(wl, **over):
    kw = dict(num_reqs=wl.num_reqs, num_q_heads=wl.num_q_heads, num_kv_heads=wl.num_kv_heads, head_dim=wl.head_dim,
              page_size=wl.page_size, num_pages=wl.num_pages, max_pages_per_req=wl.max_pages_per_req,
              total_new_tokens=wl.total_new_tokens, max_new_len=wl.max_new_len, dtype=wl.dtype,
              softmax_scale=wl.softmax_scale)
    kw.update(over)
    return B.make_batch(**kw)


def _plan(wl, min_shared_tokens=64, min_saved_key_tiles=0):
    return B.emm_prefill_shared_plan_host(_batch(wl), wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, min_shared_tokens,
                                          min_saved_key_tiles)


def _small(prefix, new, group, shared, H=28, Hkv=4, ps=16, seed=7):
    return W.build_workload("case", "causal", "bf16", seed, num_q_heads=H, num_kv_heads=Hkv, head_dim=128, page_size=ps,
                            prefix_lens=prefix, new_lens=new, share_group=group, shared_len=shared)


def _row_tiles(n_new, G):
    return -(-n_new * G // 256)


def _check_plan(wl, p):
    """What every valid plan satisfies, whatever groups the planner chose."""
    Bn, ps, G = wl.num_reqs, wl.page_size, wl.num_q_heads // wl.num_kv_heads
    S = p["req_shared_len"]
    NG = p["num_groups"]
    assert p["groups"].num_reqs == NG and p["own"].num_reqs == Bn
    # the tables are packed as narrow as their contents allow
    own_pages = [-(-(int(wl.prefix_lens[r]) - int(S[r]) + int(wl.new_lens[r])) // ps) for r in range(Bn)]
    assert p["own"].max_pages_per_req == max(1, max(own_pages)) == p["own_page_table"].shape[1]
    if NG:
        assert p["groups"].max_pages_per_req == max(p["group_prefix_lens"][:NG]) // ps == p["group_page_table"].shape[1]
    assert p["groups"].total_new_tokens == wl.total_new_tokens == p["own"].total_new_tokens
    # members of a group are consecutive requests with the same shared length
    covered = np.zeros(Bn, bool)
    plain = shared_tiles = 0
    for g in range(NG):
        r0 = [r for r in range(Bn) if wl.cu_new_lens[r] == p["group_cu_new_lens"][g] and wl.new_lens[r] > 0][0]
        s = int(p["group_prefix_lens"][g])
        assert s >= 64 and s % 64 == 0 and s % ps == 0
        n_rows, r = 0, r0
        while n_rows < p["group_new_lens"][g]:
            assert S[r] == s and not covered[r] and wl.new_lens[r] > 0
            assert s <= wl.prefix_lens[r]
            assert (wl.page_table[r, :s // ps] == p["group_page_table"][g, :s // ps]).all()
            covered[r] = True
            n_rows += int(wl.new_lens[r])
            plain += _row_tiles(int(wl.new_lens[r]), G)
            r += 1
        assert n_rows == p["group_new_lens"][g]
        assert r - r0 >= 2
        shared_tiles += _row_tiles(n_rows, G)
    assert (S[~covered] == 0).all()
    assert p["group_cu_new_lens"][NG] == wl.total_new_tokens
    assert p["groups"].max_new_len == (max(p["group_new_lens"][:NG]) if NG else 0)
    plain += sum(_row_tiles(int(n), G) for n in wl.new_lens[~covered])
    assert p["rows_tiles_plain"] == plain and p["rows_tiles_shared"] == shared_tiles
    if NG:
        assert shared_tiles < sum(_row_tiles(int(n), G) for n in wl.new_lens[covered])
    # the own part: the same keys as before minus the shared ones, through a page table moved left
    for r in range(Bn):
        skip = int(S[r]) // ps
        assert p["own_prefix_lens"][r] == wl.prefix_lens[r] - S[r]
        n_pages = -(-(int(wl.prefix_lens[r]) + int(wl.new_lens[r])) // ps)
        assert (p["own_page_table"][r, :n_pages - skip] == wl.page_table[r, skip:n_pages]).all()
        assert (p["own_page_table"][r, wl.max_pages_per_req - skip:] == -1).all()


@pytest.mark.parametrize("name", W.PREFILL_SHARED_CONFIGS)
def test_named_workloads_are_grouped_as_they_were_built(name):
    wl = W.prefill_shared_config(name, 8)
    p = _plan(wl)
    _check_plan(wl, p)
    want = {"prefill_shared_video_b8_n12": 1, "prefill_shared_video_b32_n4": 8, "prefill_shared_video_b64_n4": 8,
            "prefill_shared_image_b32": 4}[name]
    assert p["num_groups"] == want
    shared = 2880 // 8 if "image" in name else 16384 // 8
    assert (p["req_shared_len"] == shared // 64 * 64).all()


def test_a_batch_without_common_pages_has_no_groups():
    wl = _small([1024, 1024, 700], [4, 4, 9], None, None)
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 0 and (p["req_shared_len"] == 0).all()
    assert (p["own_page_table"] == wl.page_table).all() and (p["own_prefix_lens"] == wl.prefix_lens).all()
    assert p["rows_tiles_plain"] == 3 and p["rows_tiles_shared"] == 0


def test_groups_that_save_no_row_tile_are_not_formed():
    # 36 tokens x 7 query heads per KV head = 252 rows: every request fills its own tile of 256 rows
    wl = _small([2048] * 4, [36] * 4, [0] * 4, [2048] * 4)
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 0
    # 12 tokens: 84 rows each, the four together 336 rows = 2 tiles in place of 4
    wl = _small([2048] * 4, [12] * 4, [0] * 4, [2048] * 4)
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 1 and p["rows_tiles_plain"] == 4 and p["rows_tiles_shared"] == 2


def test_shared_length_is_cut_to_whole_key_tiles_and_to_the_shortest_member():
    # 66 common pages of 16 tokens = 1056 tokens -> 1024; the third request has cached only 1000 tokens of them
    wl = _small([1100, 1056, 1000, 1200], [4, 6, 3, 5], [0] * 4, [1056] * 4)
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 1
    assert p["req_shared_len"].tolist() == [960, 960, 960, 960]       # 1000 // 16 * 16 = 992 -> 960
    assert p["own_prefix_lens"].tolist() == [140, 96, 40, 240]


def test_a_short_common_part_does_not_pull_down_a_long_one():
    # requests 0..2 share 4096 tokens; request 3 shares only the first 128 of them with the others: taking it in
    # would cut the group's shared part to 128 tokens
    wl = _small([4096, 4096, 4096, 128], [8, 8, 8, 8], [0] * 4, [4096, 4096, 4096, 128])
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 1 and p["req_shared_len"].tolist() == [4096, 4096, 4096, 0]


def test_minimum_shared_length():
    wl = _small([256, 256, 256], [5, 5, 5], [0] * 3, [256] * 3)
    assert _plan(wl, 64)["num_groups"] == 1
    assert _plan(wl, 256)["num_groups"] == 1
    assert _plan(wl, 257)["num_groups"] == 0
    # below one key tile nothing is shared whatever the caller asks for
    wl = _small([48, 48], [5, 5], [0, 0], [48, 48])
    assert _plan(wl, 1)["num_groups"] == 0


def test_requests_without_new_tokens_end_a_group():
    wl = _small([1024] * 5, [4, 4, 0, 4, 4], [0] * 5, [1024] * 5)
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 2 and p["req_shared_len"].tolist() == [1024, 1024, 0, 1024, 1024]


@pytest.mark.parametrize("ps", [16, 32, 64, 128, 256])
def test_page_sizes(ps):
    wl = _small([1536 + 40, 1536, 1536 + 300], [7, 2, 11], [0] * 3, [1536] * 3, ps=ps)
    p = _plan(wl)
    _check_plan(wl, p)
    assert p["num_groups"] == 1 and (p["req_shared_len"] == 1536).all()


def test_random_batches_keep_the_invariants():
    rng = np.random.default_rng(11)
    for case in range(40):
        n = int(rng.integers(1, 13))
        ps = int(rng.choice([16, 32, 64]))
        group = sorted(int(g) for g in rng.integers(0, max(1, n // 2), size=n))
        shared_of_group = {g: int(rng.integers(0, 40)) * ps for g in set(group)}
        shared = [shared_of_group[g] for g in group]
        prefix = [s + int(rng.integers(0, 200)) for s in shared]
        if rng.random() < 0.3:
            k = int(rng.integers(0, n))
            prefix[k] = int(rng.integers(0, shared[k] + 1))
        new = [int(rng.integers(0, 50)) for _ in range(n)]
        if sum(new) == 0:
            new[0] = 3
        H, Hkv = [(28, 4), (32, 8), (8, 8), (4, 1)][case % 4]
        wl = _small(prefix, new, group, shared, H=H, Hkv=Hkv, ps=ps, seed=100 + case)
        _check_plan(wl, _plan(wl))


def test_key_tile_counts_and_the_threshold():
    # 8 requests of 16384 shared cached tokens and 12 new ones, 28/4 heads: every request alone is one row tile per KV
    # head over ceil(16396 / 64) = 257 key tiles; together 96 tokens x 7 = 672 rows = 3 row tiles over the 256 shared
    # key tiles, and each request's own 12 tokens are one more key tile
    wl = W.prefill_shared_config("prefill_shared_video_b8_n12")
    p = _plan(wl, min_saved_key_tiles=0)
    assert p["num_groups"] == 1
    assert p["key_tiles_plain"] == 8 * 257 * 4 and p["key_tiles_shared"] == (3 * 256 + 8 * 1) * 4
    saved = p["key_tiles_plain"] - p["key_tiles_shared"]
    assert _plan(wl, min_saved_key_tiles=saved)["num_groups"] == 1
    q = _plan(wl, min_saved_key_tiles=saved + 1)
    assert q["num_groups"] == 0 and (q["req_shared_len"] == 0).all() and q["groups"].num_reqs == 0
    assert (q["own_page_table"] == wl.page_table).all() and (q["own_prefix_lens"] == wl.prefix_lens).all()
    assert q["key_tiles_plain"] == p["key_tiles_plain"] and q["key_tiles_shared"] == p["key_tiles_shared"]
    # the library's default threshold: this batch saves too little, four times as many requests with 4 tokens each
    # save enough
    assert saved < B.EMM_PREFILL_SHARED_MIN_SAVED_KEY_TILES
    assert _plan(wl, min_saved_key_tiles=-1)["num_groups"] == 0
    wl = W.prefill_shared_config("prefill_shared_video_b32_n4")
    p = _plan(wl, min_saved_key_tiles=-1)
    assert p["num_groups"] == 8 and p["key_tiles_plain"] == 32 * 257 * 4 and p["key_tiles_shared"] == (8 * 256 + 32) * 4


def test_empty_batch_and_argument_errors():
    lib = B.load()
    wl = _small([256, 256], [5, 5], [0, 0], [256, 256])
    i32p = ctypes.POINTER(ctypes.c_int32)
    arrays = [np.ascontiguousarray(a, dtype=np.int32) for a in (wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens)]
    ptrs = [a.ctypes.data_as(i32p) for a in arrays]
    plan = B.emm_prefill_shared_plan()
    # no requests: nothing is read, an empty plan comes back
    empty = _batch(wl, num_reqs=0, total_new_tokens=0, max_new_len=0)
    assert lib.emm_prefill_shared_plan_host(ctypes.byref(empty), None, None, None, None, 64, 0, ctypes.byref(plan)) == 0
    assert plan.num_groups == 0 and plan.groups.num_reqs == 0 and plan.own.num_reqs == 0
    b = _batch(wl)
    assert lib.emm_prefill_shared_plan_host(ctypes.byref(b), *ptrs, 64, 0, None) == B.EMM_ERR_NULL
    assert lib.emm_prefill_shared_plan_host(ctypes.byref(b), *ptrs, 64, 0, ctypes.byref(plan)) == B.EMM_ERR_NULL   # no arrays in the plan
    assert lib.emm_prefill_shared_plan_host(None, *ptrs, 64, 0, ctypes.byref(plan)) == B.EMM_ERR_NULL
    bad = _batch(wl, page_size=48)
    assert lib.emm_prefill_shared_plan_host(ctypes.byref(bad), *ptrs, 64, 0, ctypes.byref(plan)) == B.EMM_ERR_UNSUPPORTED
    bad = _batch(wl, num_kv_heads=3)
    assert lib.emm_prefill_shared_plan_host(ctypes.byref(bad), *ptrs, 64, 0, ctypes.byref(plan)) == B.EMM_ERR_INVALID_ARG


def test_workspace_size_and_pair_checks():
    wl = W.prefill_shared_config("prefill_shared_video_b8_n12", 8)
    p = _plan(wl)
    rows = wl.total_new_tokens * wl.num_q_heads
    need = B.emm_prefill_attn_shared_workspace_size(p["groups"], p["own"])
    assert need >= rows * (128 * 2 + 8) and need % 256 == 0
    lib = B.load()
    n = ctypes.c_size_t(0)
    other = _batch(wl, num_q_heads=32)
    assert lib.emm_prefill_attn_shared_workspace_size(ctypes.byref(p["groups"]), ctypes.byref(other), ctypes.byref(n)) == B.EMM_ERR_INVALID_ARG
    other = _batch(wl, total_new_tokens=wl.total_new_tokens + 1)
    assert lib.emm_prefill_attn_shared_workspace_size(ctypes.byref(p["groups"]), ctypes.byref(other), ctypes.byref(n)) == B.EMM_ERR_INVALID_ARG
    assert lib.emm_prefill_attn_shared_workspace_size(ctypes.byref(p["groups"]), ctypes.byref(p["own"]), None) == B.EMM_ERR_NULL
    f32 = _batch(wl, dtype="f32")
    assert lib.emm_prefill_attn_shared_workspace_size(ctypes.byref(f32), ctypes.byref(f32), ctypes.byref(n)) == B.EMM_ERR_UNSUPPORTED
