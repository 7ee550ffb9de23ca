"""Host logic of the prefill launch (emm_prefill_plan_host): how a batch is dealt to the XCDs, how many work
units each gets, and how the units left over after full rounds are cut.  What carries weight here are the
invariants the kernels rely on (every unit appears once; the extra workgroups, the workspace records and the
merge workgroups suffice; the workspace size covers any plan the scalar fields admit); the second writing-out of
the rule in plain Python only guards against the C++ and the description drifting apart.  No GPU."""
from __future__ import annotations

import numpy as np
import pytest

from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import workloads as W

XCDS, CUS, ROWS = 8, 32, 256


def _batch(H, Hkv, new, dtype="bf16", d=128):
    return B.make_batch(num_reqs=len(new), num_q_heads=H, num_kv_heads=Hkv, head_dim=d, page_size=16, num_pages=1 << 20,
                        max_pages_per_req=1 << 16, total_new_tokens=int(sum(new)), max_new_len=int(max(new)) if len(new) else 0,
                        dtype=dtype, softmax_scale=0.1)


def _model(H, Hkv, new):
    """Units per XCD and pieces per left-over unit, from the description of the scheme alone."""
    G = H // Hkv
    pairs = len(new) * Hkv
    fan = 1
    while fan < XCDS and pairs * fan * 2 <= XCDS:
        fan *= 2
    if len(set(new)) > 1:                                      # requests of different lengths: every request on every XCD
        while fan < XCDS and (Hkv * fan) % XCDS:
            fan *= 2
    units = [0] * XCDS
    for p in range(pairs):
        tiles = -(-new[p // Hkv] * G // ROWS)
        for j in range(fan):                                   # sub-pair j of pair p takes row tiles j, j + fan, ...
            units[(p * fan + j) % XCDS] += len(range(j, tiles, fan))
    per_xcd = -(-pairs * fan // XCDS)
    uniform = len(set(new)) == 1
    cutting = per_xcd <= 64
    uneven_ok = not (uniform and len(set(units)) == 1)
    pieces, ks, halves = [], [], []
    for u in units:
        rem, full = u % CUS, u // CUS
        k = -(-rem // (CUS - rem)) if (16 < rem <= 30 and uneven_ok) else 0
        half = full > 0 and 12 < rem <= 16
        if rem == 0:
            p = 1
        elif k or half:
            p = 2
        elif full == 0:
            p = 1
            while p < 32 and 2 * p * rem <= CUS:
                p *= 2
        else:
            p = 1 if rem > 12 else 2 if rem > 8 else 4
        pieces.append(p); ks.append(k); halves.append(int(half))
    if uniform and cutting and all(p == 1 for p in pieces):
        cutting = False                                        # the host knows that nothing will be cut
    if not cutting:
        pieces, ks, halves = [1] * XCDS, [0] * XCDS, [0] * XCDS
    return fan, units, pieces, ks, halves, cutting


def test_named_workloads():
    cfg3 = W.config(3)
    p = B.emm_prefill_plan_host(_batch(28, 4, cfg3.new_lens.tolist()), cfg3.new_lens)
    assert p["units"] == [56] * 8 and p["cutting"] == 0 and p["grid"] == 448          # two rounds, the second of 24: not cut
    one = B.emm_prefill_plan_host(_batch(28, 4, [36]), [36])                            # a lone unit on every other XCD
    assert one["fan"] == 2 and one["units"] == [1, 0] * 4 and one["pieces"] == [32, 1] * 4 and one["grid"] == 8 * (1 + 31)
    cfg5 = W.config(5)
    p5 = B.emm_prefill_plan_host(_batch(32, 8, cfg5.new_lens.tolist()), cfg5.new_lens)
    want = sum(-(-int(n) * 4 // ROWS) for n in cfg5.new_lens)                           # every XCD holds one KV head of every request
    assert p5["units"] == [want] * 8 and p5["cutting"] == 1
    cfg2 = W.config(2)                                           # requests of different lengths on 4 KV heads: each pair is
    p2 = B.emm_prefill_plan_host(_batch(28, 4, cfg2.new_lens.tolist()), cfg2.new_lens)   # dealt to 2 XCDs, so that every XCD
    assert p2["fan"] == 2                                        # gets half the row tiles of one KV head of every request
    assert max(p2["units"]) - min(p2["units"]) <= len(cfg2.new_lens), p2["units"]
    no_ws = B.emm_prefill_plan_host(_batch(28, 4, [36]), [36], with_workspace=False)
    assert no_ws["cutting"] == 0 and no_ws["pieces"] == [1] * 8 and no_ws["grid"] == 8


@pytest.mark.parametrize("seed", range(40))
def test_random_batches_match_model_and_keep_invariants(seed):
    rng = np.random.default_rng(300 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8, 16]))
    G = int(rng.choice([1, 2, 4, 7, 8]))
    n_req = int(rng.choice([1, 1, 2, 3, 5, 8, 16, 33, 70]))
    top = int(rng.choice([1, 3, 40, 300, 2100]))
    new = [int(x) for x in rng.integers(0, top + 1, n_req)]
    if rng.random() < 0.25:
        new = [top] * n_req                                    # a uniform batch
    if sum(new) == 0:
        new[0] = top
    H = Hkv * G
    p = B.emm_prefill_plan_host(_batch(H, Hkv, new), new)
    fan, units, pieces, ks, halves, cutting = _model(H, Hkv, new)
    assert (p["fan"], p["units"], p["cutting"]) == (fan, units, int(cutting)), (new, p)
    assert (p["pieces"], p["uneven_k"], p["rows_only"]) == (pieces, ks, halves), (new, p)
    assert sum(p["units"]) == sum(-(-n * G // ROWS) for n in new) * Hkv              # every row tile of every pair, once
    assert p["grid"] == XCDS * (p["slots_per_xcd"] + (31 if p["cutting"] else 0))
    for x in range(XCDS):
        rem = p["units"][x] % CUS
        assert p["units"][x] <= p["slots_per_xcd"]                                     # a slot for every unit
        assert rem * (p["pieces"][x] - 1) <= 31                                        # extra workgroups for pieces 1, 2, ...
        assert rem * p["pieces"][x] <= 64                                              # workspace slots of the XCD
        shares = 1 if p["uneven_k"][x] else p["pieces"][x]
        assert p["pieces"][x] == 1 or rem * shares <= 32                               # merge workgroups of the XCD
        assert (p["uneven_k"][x] > 0) <= (16 < rem <= 30)


PIECE_BYTES = 66 * 512 * 4          # a piece record: 64 accumulator values, reference exponent and row sum per thread


@pytest.mark.parametrize("seed", range(40))
def test_workspace_size_covers_the_plan(seed):
    """emm_prefill_attn_workspace_size, which sees only the scalar fields, against what the plan for the real lengths
    needs: 8 XCDs x (left-over units x planned pieces) records, laid out with one stride for all XCDs.  It must cover
    the plan for any lengths the scalars admit, be exact when the host can know the plan (all requests alike), and
    be zero when nothing can be cut."""
    rng = np.random.default_rng(900 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 4, 7, 8]))
    n_req = int(rng.choice([1, 2, 3, 8, 16, 40]))
    top = int(rng.choice([3, 40, 300, 2100]))
    uniform = rng.random() < 0.4
    new = [top] * n_req if uniform else [int(x) for x in rng.integers(0, top + 1, n_req)]
    if sum(new) == 0:
        new[0] = top
    max_pages = int(rng.choice([16, 64, 600, 4096]))          # contexts of at most 256 .. 65536 tokens
    b = B.make_batch(num_reqs=n_req, num_q_heads=Hkv * G, num_kv_heads=Hkv, head_dim=128, page_size=16, num_pages=1 << 20,
                     max_pages_per_req=max_pages, total_new_tokens=int(sum(new)), max_new_len=int(max(new)), dtype="bf16",
                     softmax_scale=0.1)
    size = B.emm_prefill_attn_workspace_size(b)
    p = B.emm_prefill_plan_host(b, new)
    assert size % (XCDS * PIECE_BYTES) == 0
    stride = size // (XCDS * PIECE_BYTES)                      # records per XCD
    cuttable = max_pages * 16 >= 24 * 64                       # a context of 24 key tiles: the shortest that is ever cut
    need = 0
    for x in range(XCDS):
        rem = p["units"][x] % CUS
        if p["cutting"] and p["pieces"][x] > 1 and not p["rows_only"][x] and cuttable:
            need = max(need, rem * p["pieces"][x])
    assert stride >= need, (new, p, stride)
    if not cuttable or not p["cutting"]:
        assert size == 0
    if len(set(new)) == 1:
        assert stride == need                                   # the host knows every XCD's unit count
    assert stride <= 64


def test_workspace_of_the_headline_workload_is_empty():
    cfg3 = W.config(3)
    b = _batch(28, 4, cfg3.new_lens.tolist())
    assert B.emm_prefill_attn_workspace_size(b) == 0          # 56 units per XCD, none cut: no records, no merge


def test_argument_errors():
    lib = B.load()
    import ctypes
    plan = B.emm_prefill_plan()
    ok = (ctypes.c_int32 * 2)(5, 5)
    assert lib.emm_prefill_plan_host(None, ok, 1, ctypes.byref(plan)) == B.EMM_ERR_NULL
    b = _batch(8, 2, [5, 5])
    assert lib.emm_prefill_plan_host(ctypes.byref(b), None, 1, ctypes.byref(plan)) == B.EMM_ERR_NULL
    assert lib.emm_prefill_plan_host(ctypes.byref(b), ok, 1, None) == B.EMM_ERR_NULL
    f32 = _batch(8, 2, [5, 5], dtype="f32", d=64)
    assert lib.emm_prefill_plan_host(ctypes.byref(f32), ok, 1, ctypes.byref(plan)) == B.EMM_ERR_UNSUPPORTED
    empty = _batch(8, 2, [])
    assert lib.emm_prefill_plan_host(ctypes.byref(empty), None, 1, ctypes.byref(plan)) == B.EMM_OK and plan.grid == 0


@pytest.mark.parametrize("n_req,Hkv,G,max_pages", [(1, 4, 7, 1024), (8, 4, 7, 1152), (64, 4, 7, 512), (32, 8, 4, 290), (3, 1, 16, 40),
                                                   (200, 8, 1, 64), (1, 4, 7, 8192), (5, 2, 3, 1)])
def test_decode_workspace_holds_the_pieces_of_the_longest_context(n_req, Hkv, G, max_pages):
    """A decode batch's workspace is [pair][piece][16 rows][130 floats]; pieces are 4 .. 124 tiles of 32 keys, and
    there must be enough of them for a context that fills the page-table row."""
    b = B.make_batch(num_reqs=n_req, num_q_heads=Hkv * G, num_kv_heads=Hkv, head_dim=128, page_size=16, num_pages=1 << 20,
                     max_pages_per_req=max_pages, total_new_tokens=n_req, max_new_len=1, dtype="bf16", softmax_scale=0.1)
    per_piece = 16 * 130 * 4
    size = B.emm_prefill_attn_workspace_size(b)
    assert size % (n_req * Hkv * per_piece) == 0
    pieces = size // (n_req * Hkv * per_piece)
    tiles = -(-max_pages * 16 // 32)
    assert -(-tiles // 124) <= pieces <= max(-(-tiles // 4), 1)
    # hints can only shrink it; a hint larger than the table changes nothing
    small = B.make_shared_prefix(0, planned_tiles=n_req * 4, max_own_tiles=4)
    assert B.emm_decode_attn_shared_workspace_size(b, small) <= size
    wide = B.make_shared_prefix(0, planned_tiles=0, max_own_tiles=10 * tiles)
    assert B.emm_decode_attn_shared_workspace_size(b, wide) == size


def test_decode_plan_of_a_single_request_uses_fewer_longer_pieces():
    """One request cannot be ragged: its contexts are cut so that about 1.5 workgroups per compute unit (at most 384)
    stream them, where a batch of several requests is planned for rounds of 768."""
    per_piece = 16 * 130 * 4
    def pieces(n_req, max_pages):
        b = B.make_batch(num_reqs=n_req, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16, num_pages=1 << 20,
                         max_pages_per_req=max_pages, total_new_tokens=n_req, max_new_len=1, dtype="bf16", softmax_scale=0.1)
        size = B.emm_prefill_attn_workspace_size(b)
        assert size % (n_req * 4 * per_piece) == 0
        return size // (n_req * 4 * per_piece)
    one = pieces(1, 8192)                                       # 131072 tokens: 4096 tiles of 32 keys per KV head
    assert 256 < 4 * one <= 384
    two = pieces(2, 4096)                                       # the same number of tiles in two requests
    assert 384 < 8 * two <= 768
