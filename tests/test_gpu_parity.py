"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on the same seeded inputs.

Bars: the KV scatter is bit-exact over the whole pool; bf16 attention outputs are within max-abs 2e-2
and mean-abs 2e-3 of the oracle (bf16 inputs, fp32 accumulation); the fp32 configuration is held to
max-abs 1e-4.  Every workload is compared element by element, the three large ones at full size too (the
oracle takes 15 to 30 s for each); a quick variant compares them on sampled query tokens."""
import numpy as np
import pytest
import torch

import oracle
from helpers import as_f64, err_stats
from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import workloads as W

pytestmark = pytest.mark.gpu

BF16_MAX_ABS, BF16_MEAN_ABS = 2e-2, 2e-3
F32_MAX_ABS = 1e-4
LSE_ABS = 4e-3   # l is the sum of the bf16-rounded weights: relative error up to 2^-9 when one key dominates


def _gpu_run(wl, poison_unused=False):
    dw = B.DeviceWorkload(wl)
    dw.out.zero_()
    dw.step()
    torch.cuda.synchronize()
    return dw


def _compare(wl, dw, tokens=None):
    kc, vc, out_ref, lse_ref = oracle.run_workload(wl, tokens)
    if wl.kind == "causal":
        assert B.DeviceWorkload.to_numpy_bits(dw.k_cache).tobytes() == kc.tobytes(), "K pool differs"
        assert B.DeviceWorkload.to_numpy_bits(dw.v_cache).tobytes() == vc.tobytes(), "V pool differs"
    out = as_f64(B.DeviceWorkload.to_numpy_bits(dw.out))
    lse = dw.lse.cpu().numpy().astype(np.float64)
    if tokens is not None:
        out, lse = out[np.asarray(tokens)], lse[np.asarray(tokens)]
    assert np.isfinite(out).all()
    mx, mean = err_stats(out, out_ref)
    finite = np.isfinite(lse_ref)
    lse_err = float(np.abs(lse[finite] - lse_ref[finite]).max()) if finite.any() else 0.0
    assert (np.isneginf(lse[~finite])).all()
    if wl.dtype == "bf16":
        assert mx <= BF16_MAX_ABS and mean <= BF16_MEAN_ABS, (mx, mean)
    else:
        assert mx <= F32_MAX_ABS, mx
    assert lse_err <= LSE_ABS, lse_err
    return mx, mean, lse_err


def _sample_tokens(wl, n, seed=0):
    """Sampled packed tokens: first and last row of every request (diagonal edges) plus random ones."""
    rng = np.random.default_rng(seed)
    cu = wl.cu_new_lens
    picks = set()
    for r in range(wl.num_reqs):
        if wl.new_lens[r] > 0:
            picks.update([int(cu[r]), int(cu[r + 1]) - 1])
    picks.update(int(t) for t in rng.integers(0, wl.total_new_tokens, size=n))
    return sorted(picks)


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 4), (3, 16), (4, 8), (5, 8), (2, 1)])
def test_elementwise_parity(cfg, shrink):
    print("case cfg=%d shrink=%d" % (cfg, shrink), flush=True)
    wl = W.config(cfg, shrink)
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)


@pytest.mark.parametrize("cfg,n", [(3, 24), (4, 96), (5, 48)])
def test_full_size_sampled_parity(cfg, n):
    """The sizes and launch configuration bench.py times."""
    print("case full cfg=%d" % cfg, flush=True)
    wl = W.config(cfg, 1)
    dw = _gpu_run(wl)
    tokens = _sample_tokens(wl, n, seed=cfg)
    print("   errors (max, mean, lse):", _compare(wl, dw, tokens), flush=True)


@pytest.mark.parametrize("cfg", [3, 4, 5])
def test_full_size_exhaustive_parity(cfg):
    """Every output element of the three large workloads, at the sizes and in the launch configuration bench.py
    times, against the oracle (which takes 15 to 30 s per workload on the host cores): the max-abs / mean-abs bars
    are stated over all T x H x d elements of a workload, and the pools are compared byte for byte."""
    print("case full exhaustive cfg=%d" % cfg, flush=True)
    wl = W.config(cfg, 1)
    dw = _gpu_run(wl)
    print("   errors over all %d x %d x %d elements (max, mean, lse):" % (wl.total_new_tokens, wl.num_q_heads, wl.head_dim),
          _compare(wl, dw), flush=True)


@pytest.mark.parametrize("name", W.SUFFIX_CONFIGS)
def test_suffix_after_cache_hit_sampled_parity(name):
    """Short suffixes over long cached contexts at the sizes bench.py --others times: every unit is cut into
    2 .. 16 pieces (or halved) because no XCD has a full round of units."""
    print("case", name, flush=True)
    wl = W.suffix_config(name)
    dw = _gpu_run(wl)
    tokens = None if wl.total_new_tokens <= 40 else _sample_tokens(wl, 24, seed=len(name))
    print("   errors (max, mean, lse):", _compare(wl, dw, tokens), flush=True)


RAGGED = [(0, 1), (0, 2), (0, 33), (1, 1), (15, 31), (16, 32), (17, 33), (63, 127), (64, 128), (65, 129),
          (200, 300), (0, 129), (127, 1), (128, 64), (1000, 7)]


def test_ragged_causal_sweep():
    """Prefix / new-token lengths around every tile boundary (16-token pages, 64-key tiles, 32-row waves,
    128-row workgroups), several requests per batch, including an empty request."""
    for gi, (H, Hkv) in enumerate(((8, 2), (7, 1), (4, 4))):
        prefix = [p for p, _ in RAGGED] + [40]
        new = [n for _, n in RAGGED] + [0]
        print("case ragged heads=%d/%d" % (H, Hkv), flush=True)
        wl = W.build_workload("ragged", "causal", "bf16", 500 + gi, num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                              page_size=16, prefix_lens=prefix, new_lens=new)
        dw = _gpu_run(wl)
        _compare(wl, dw)


def test_ragged_cross_sweep():
    """Cross-attention: cached lengths around page and tile boundaries, and a request with nothing cached
    (zero rows, lse = -inf)."""
    lkv = [0, 1, 4, 15, 16, 17, 63, 64, 65, 100, 127, 128, 129, 1601]
    nq = [5, 1, 33, 32, 31, 128, 129, 7, 64, 2, 200, 1, 130, 45]
    print("case ragged cross", flush=True)
    wl = W.build_workload("ragged_cross", "cross", "bf16", 600, num_q_heads=8, num_kv_heads=2, head_dim=128,
                          page_size=16, prefix_lens=lkv, new_lens=nq)
    dw = _gpu_run(wl)
    _compare(wl, dw)
    out = B.DeviceWorkload.to_numpy_bits(dw.out)
    assert (out[:5] == 0).all()


# Batches whose last work units are cut along the key axis and merged by the second kernel.  A unit is a
# 256-row tile of one (request, KV head) pair; pairs are dealt to the 8 XCDs; the units an XCD has left over
# after its full rounds of 32 are cut into 4 pieces (1..8 left over) or 2 (9..12) when every piece gets at least
# 16 key tiles and starts below the diagonal; an XCD without a full round cuts into as many pieces as fill it,
# up to 32, of at least 2 key tiles, if the unit has 24 key tiles or more (four or more such pieces: two short ones
# are no better than two row halves).
CUT_CASES = [
    # name, kind, H, Hkv, prefix lens, new lens
    ("cut4_causal", "causal", 28, 4, [5000], [64]),                 # 1 unit per XCD, planned for 32 pieces; 80 tiles give 8 of 10
    ("cut2_causal", "causal", 28, 4, [2100], [350]),                # 10 units per XCD, 2 pieces each
    ("cut4_cross", "cross", 32, 8, [6404, 6404], [100, 37]),        # 3 units per XCD, 8 pieces; ragged last tile
    ("cut32_causal", "causal", 28, 4, [17000], [36]),               # 1 unit on every other XCD, 267 tiles: 32 pieces
    ("cut32_cross", "cross", 32, 8, [16500], [30]),                 # 1 unit per XCD of 120 rows, 258 tiles: 32 pieces
    ("cut16_causal", "causal", 28, 4, [9000, 9100], [36, 20]),      # 1 unit per XCD, 142-143 tiles: 16 pieces
    ("cut8_planned", "causal", 32, 8, [8200, 8300, 9000], [50, 64, 3]),   # 3 units per XCD, 8 pieces each
    ("cut_2units", "causal", 16, 8, [16400, 16400], [130, 7]),      # 2 and 1 units per XCD: 16 and 32 pieces
    ("cut_table_edge", "causal", 28, 4, [1990, 700], [10, 3]),      # 125 pages hold 2000 slots: 32 tiles, just enough for 4 pieces
    ("cut_table_edge2", "causal", 28, 4, [1970], [14]),             # 124 pages, 31 tiles: not cut
    ("cut32_short", "causal", 28, 4, [16384 - 40], [40]),           # 256 tiles exactly: 32 pieces of 8, the last one on the diagonal
    ("cut_mixed", "causal", 16, 8, [8000, 100, 4100], [64, 200, 3]),  # long units are cut, short ones are not
    ("cut_edge", "causal", 8, 8, [4091, 4096, 4000, 1800], [5, 5, 200, 300]),  # 64 tiles: just cut; 63: not cut;
                                                                    # a last piece that would start on the diagonal
    ("cut_short", "causal", 28, 4, [1056], [300]),                  # 9 units per XCD, too short to cut
    ("cut_gqa1", "causal", 8, 8, [4100], [300]),                    # one head per group: 256 tokens per row tile
    # units too short to cut along the keys are halved along their rows (two workgroups of four working waves)
    ("halve_one", "causal", 28, 4, [700], [36]),                    # 252 rows: one unit per head, halved
    ("halve_small", "causal", 28, 4, [700, 50], [18, 19]),          # 126 and 133 rows: nothing to halve / halved
    ("halve_cross", "cross", 32, 8, [900, 333], [60, 61]),          # 240 and 244 rows, no mask
    ("halve_14", "causal", 56, 8, [100], [512]),                    # 14 units per XCD, short context: halved
    ("halve_14_long", "causal", 56, 8, [9000], [512]),              # 14 units per XCD, long context: two pieces along the keys
    ("halve_46_long", "causal", 56, 8, [9000], [1670]),             # 46 units per XCD = a full round + 14: those are halved, never cut
    # 17 .. 30 units in an XCD's last round: each cut in two uneven pieces (k short ones per otherwise idle compute unit)
    ("uneven_25", "causal", 28, 4, [6000, 6100], [878, 870]),       # 25 units per XCD: k = 4, cut at 4/5 of 108+ tiles
    ("uneven_17", "causal", 32, 8, [4000], [1088]),                 # 17 units per XCD: k = 2, cut at 2/3
    ("uneven_30", "causal", 32, 8, [17000], [1920]),                # 30 units per XCD: k = 15, short pieces of 16-18 tiles
    ("uneven_short", "causal", 28, 4, [500, 520], [878, 878]),      # 25 units per XCD, too short to cut: whole units
    ("uneven_cross", "cross", 32, 8, [9000], [1088]),               # 17 units per XCD, no mask
    ("uneven_after_round", "causal", 56, 8, [5000], [2100]),        # 58 units per XCD = a full round + 26: k = 5
    # one long request and many short ones: the grid is sized by the batch's row tiles, not by the longest request
    ("long_and_short", "causal", 32, 8, [0] + [100] * 31, [2048] + [1] * 31),
    ("long_and_short_h4", "causal", 28, 4, [300] + [50] * 20, [1500] + [3] * 20),
    ("many_pairs", "causal", 28, 4, [int(x) for x in np.random.default_rng(5).integers(0, 2500, 100)],
     [int(x) for x in np.random.default_rng(6).integers(0, 400, 100)]),          # 400 pairs: 50 per XCD, one per lane of the scan
    ("too_many_pairs", "causal", 32, 8, [int(x) for x in np.random.default_rng(7).integers(0, 900, 70)],
     [int(x) for x in np.random.default_rng(8).integers(1, 300, 70)]),           # 560 pairs: 70 per XCD, no scan, no cuts
    ("far_too_many_pairs", "causal", 8, 8, [int(x) for x in np.random.default_rng(11).integers(0, 200, 280)],
     [int(x) for x in np.random.default_rng(12).integers(0, 40, 280)]),          # 2240 pairs: 280 per XCD, some requests empty
    ("long_and_empty", "causal", 16, 16, [40, 0, 7, 5000], [0, 0, 0, 700]),     # 16 KV heads: two pairs of a request per XCD
    ("halve_ragged", "causal", 28, 4, [300, 1056, 0, 77], [100, 37, 150, 3]),   # last row tiles of 188, 3, 26, 21 rows
]


@pytest.mark.parametrize("name,kind,H,Hkv,prefix,new", CUT_CASES)
def test_cut_units_parity(name, kind, H, Hkv, prefix, new):
    print("case", name, flush=True)
    wl = W.build_workload(name, kind, "bf16", 950 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=prefix, new_lens=new)
    dw = _gpu_run(wl)
    tokens = None if wl.total_new_tokens <= 160 else _sample_tokens(wl, 96, seed=len(name))
    print("   errors (max, mean, lse):", _compare(wl, dw, tokens), flush=True)
    # a second launch on the same workspace (stale pieces of the first) gives the same bits
    first = B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()
    dw.attention()
    torch.cuda.synchronize()
    assert B.DeviceWorkload.to_numpy_bits(dw.out).tobytes() == first


@pytest.mark.parametrize("kind,n_req", [("causal", 1), ("causal", 2), ("cross", 1), ("cross", 3)])
def test_cut_thresholds_sweep(kind, n_req):
    """Contexts whose key-tile counts sit on and around every threshold of the cutting rule (pieces of at least
    2 or 16 tiles, 2 .. 32 of them), with the page table exactly as wide as the context needs: one and two
    requests, so that an XCD holds one unit (32 pieces planned) or two (16); three for cross-attention (8)."""
    for tiles in (7, 8, 9, 15, 16, 17, 23, 24, 25, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257):
        for slack in (0, 1, 63):                           # the last tile full, one key short, one key only
            ctx = tiles * 64 - slack
            new = 3
            print("case thresholds", n_req, tiles, slack, flush=True)
            wl = W.build_workload("thresholds", kind, "bf16", 7000 + tiles, num_q_heads=8, num_kv_heads=4,
                                  head_dim=128, page_size=16, prefix_lens=[ctx - new if kind == "causal" else ctx] * n_req,
                                  new_lens=[new] * n_req, spare_pages=0)
            dw = _gpu_run(wl)
            _compare(wl, dw)


@pytest.mark.parametrize("H,Hkv,prefix,new", [(4, 1, [300], [700]), (8, 2, [0], [1500]), (6, 1, [70, 0, 513], [300, 90, 64]),
                                              (8, 4, [129], [1]), (2, 1, [5000], [1100])])
def test_few_pairs_spread_over_xcds(H, Hkv, prefix, new):
    """Fewer than 8 (request, KV head) pairs: each pair's row tiles are dealt to several XCDs."""
    print("case few pairs", H, Hkv, prefix, new, flush=True)
    wl = W.build_workload("few_pairs", "causal", "bf16", 990 + H, num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=prefix, new_lens=new)
    dw = _gpu_run(wl)
    tokens = None if wl.total_new_tokens <= 200 else _sample_tokens(wl, 128, seed=H)
    print("   errors (max, mean, lse):", _compare(wl, dw, tokens), flush=True)


@pytest.mark.parametrize("seed", range(10))
def test_random_batches_sampled(seed):
    """Random batch shapes (request count, head grouping, prefix and new-token lengths from a few tokens to
    several thousand, empty requests, both kinds): every launch shape the planner can produce -- whole and
    cut units, pairs fanned out over XCDs, ragged last tiles -- against the oracle on sampled tokens."""
    rng = np.random.default_rng(4000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 7]))
    n_req = int(rng.choice([1, 1, 2, 3, 5, 9, 20]))
    kind = "cross" if seed % 4 == 3 else "causal"
    scale = int(rng.choice([40, 400, 3000, 9000]))
    prefix = [int(x) for x in rng.integers(0, scale + 1, size=n_req)]
    new = [int(x) for x in rng.integers(0, max(2, scale // int(rng.choice([1, 4, 30]))) + 1, size=n_req)]
    if sum(new) == 0:
        new[0] = 17
    print("case random", seed, kind, "H", Hkv * G, "Hkv", Hkv, "prefix", prefix, "new", new, flush=True)
    wl = W.build_workload("random%d" % seed, kind, "bf16", 4100 + seed, num_q_heads=Hkv * G, num_kv_heads=Hkv,
                          head_dim=128, page_size=16, prefix_lens=prefix, new_lens=new)
    dw = _gpu_run(wl)
    tokens = None if wl.total_new_tokens <= 96 else _sample_tokens(wl, 64, seed=seed)
    print("   errors (max, mean, lse):", _compare(wl, dw, tokens), flush=True)


DECODE_CASES = [
    # name, kind, H, Hkv, context lengths before the new token, new lens (0 = request without a query token)
    ("decode_mixed", "causal", 28, 4, [0, 1, 15, 16, 62, 63, 64, 65, 127, 128, 500, 1056, 4095, 4096, 9000], [1] * 15),
    ("decode_long", "causal", 32, 8, [20000, 18431, 3, 7000], [1, 1, 1, 1]),        # several pieces per request
    ("decode_holes", "causal", 8, 8, [300, 40, 0, 2000, 77], [1, 0, 1, 1, 0]),      # G = 1; requests without a token
    ("decode_g16", "causal", 16, 1, [1500, 64], [1, 1]),                             # 16 heads on one KV head
    ("decode_g17", "causal", 34, 2, [700, 129], [1, 1]),                             # too wide: the prefill kernel does it
    ("decode_cross", "cross", 32, 8, [6404, 0, 17, 1601], [1, 1, 1, 1]),             # one text query over image K/V
    ("decode_single", "causal", 28, 4, [16384], [1]),                                # one request, long context
]


@pytest.mark.parametrize("name,kind,H,Hkv,ctx,new", DECODE_CASES)
def test_decode_step_parity(name, kind, H, Hkv, ctx, new):
    """The decode step (at most one new token per request) through emm_decode_attn and, for the same batch,
    through emm_prefill_attn, against the oracle; the two entry points must agree bit for bit."""
    print("case", name, flush=True)
    wl = W.build_workload(name, kind, "bf16", 1200 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=ctx, new_lens=new)
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)
    if kind == "causal":
        first = B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()
        dw.out.zero_()
        B.emm_decode_attn(dw.batch, dw.q, dw.k_cache, dw.v_cache, dw.out, dw.lse, dw.workspace)
        torch.cuda.synchronize()
        assert B.DeviceWorkload.to_numpy_bits(dw.out).tobytes() == first


SHARED_CASES = [
    # name, H, Hkv, context lengths, new lens, share group per request, shared tokens per request, units expected
    ("shared_pairs", 28, 4, [700, 650, 900, 300, 1300], [1] * 5, [0, 0, 1, 2, 2], [512, 512, 0, 290, 290], 2),
    ("shared_wide", 32, 8, [2100 + 37 * i for i in range(19)], [1] * 19, [0] * 19, [2048] * 19, 3),   # 8 + 8 + 3 requests
    ("shared_g16", 16, 1, [800, 801, 400], [1, 1, 1], [0, 0, 0], [384, 384, 384], 1),      # two requests fill a tile
    ("shared_g1", 8, 8, [100 * i + 640 for i in range(12)], [1] * 12, [0] * 12, [640] * 12, 1),
    ("shared_exact", 28, 4, [1024, 1024, 1024], [1, 1, 1], [0, 0, 0], [1024, 1024, 1024], 1),   # own part: the new token only
    ("shared_holes", 28, 4, [600, 600, 600, 600, 600], [1, 1, 0, 1, 1], [0] * 5, [512] * 5, 2),  # a request without a token
    ("shared_none", 32, 8, [300, 500], [1, 1], [0, 1], [0, 0], 0),                               # nothing shared
    ("shared_long", 28, 4, [18432, 18000, 17000, 16500], [1] * 4, [0] * 4, [16384] * 4, 1),      # several pieces per unit
]


@pytest.mark.parametrize("name,H,Hkv,ctx,new,group,shared", [
    ("xshared_same_image", 32, 8, [6404] * 6, [1] * 6, [0] * 6, [6404] * 6),           # all tokens shared: 6400 by the unit, 4 own
    ("xshared_exact", 32, 8, [1600] * 3, [1, 1, 1], [0] * 3, [1600] * 3),               # a multiple of 32: no own part at all
    ("xshared_mixed", 28, 4, [1601, 1601, 500, 3202, 3202, 3202], [1] * 6, [0, 0, 1, 2, 2, 2], [1601, 1601, 0, 3202, 3202, 3202]),
    ("xshared_holes", 32, 8, [800, 800, 0, 800], [1, 1, 1, 0], [0, 0, 1, 0], [800, 800, 0, 800]),    # nothing cached; no query
])
def test_cross_decode_shared_prefix_parity(name, H, Hkv, ctx, new, group, shared):
    """Decode step of a cross-attention layer (one text query per request over cached image K/V, unmasked) with the
    image pages of requests that show the same image read once per unit."""
    print("case", name, flush=True)
    wl = W.build_workload(name, "cross", "bf16", 1600 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=ctx, new_lens=new, share_group=group, shared_len=shared)
    dw = _gpu_run(wl)
    _compare(wl, dw)
    plain = as_f64(B.DeviceWorkload.to_numpy_bits(dw.out))
    plan = dw.plan_shared()
    print("   units:", plan["num_units"], plan["unit_num_reqs"].tolist(), plan["unit_shared_len"].tolist(), flush=True)
    assert plan["num_units"] >= 1
    dw.out.zero_()
    dw.lse.zero_()
    dw.attention_shared()
    torch.cuda.synchronize()
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)
    assert np.abs(as_f64(B.DeviceWorkload.to_numpy_bits(dw.out)) - plain).max() <= BF16_MAX_ABS


@pytest.mark.parametrize("name,H,Hkv,ctx,new,group,shared,n_units", SHARED_CASES)
def test_decode_shared_prefix_parity(name, H, Hkv, ctx, new, group, shared, n_units):
    """emm_decode_attn_shared with the units found by emm_shared_prefix_plan_host, against the oracle (which
    knows nothing of units) and, loosely, against emm_decode_attn on the same batch."""
    print("case", name, flush=True)
    wl = W.build_workload(name, "causal", "bf16", 1300 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=ctx, new_lens=new, share_group=group, shared_len=shared)
    dw = _gpu_run(wl)                                   # scatter + plain decode path
    plain = as_f64(B.DeviceWorkload.to_numpy_bits(dw.out))
    plan = dw.plan_shared()
    print("   units:", plan["num_units"], plan["unit_first_req"].tolist(), plan["unit_num_reqs"].tolist(),
          plan["unit_shared_len"].tolist(), flush=True)
    assert plan["num_units"] == n_units
    dw.out.zero_()
    dw.lse.zero_()
    dw.attention_shared()
    torch.cuda.synchronize()
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)
    assert np.abs(as_f64(B.DeviceWorkload.to_numpy_bits(dw.out)) - plain).max() <= BF16_MAX_ABS
    first = B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()
    dw.attention_shared()                               # again into the same workspace: same bits
    torch.cuda.synchronize()
    assert B.DeviceWorkload.to_numpy_bits(dw.out).tobytes() == first
    dw.plan_shared(use_hint=False)                      # without the hint and the bounds: the page table's width rules
    dw.out.zero_()
    dw.attention_shared()
    torch.cuda.synchronize()
    _compare(wl, dw)


FUSED_CASES = [(c[0], c[2], c[3], c[4], c[5], None, None) for c in DECODE_CASES if c[1] == "causal" and c[0] != "decode_g17"] + \
              [(c[0], c[1], c[2], c[3], c[4], c[5], c[6]) for c in SHARED_CASES]


@pytest.mark.parametrize("name,H,Hkv,ctx,new,group,shared", FUSED_CASES)
def test_fused_decode_step_equals_scatter_then_attention(name, H, Hkv, ctx, new, group, shared):
    """emm_decode_step (the new tokens' K/V rows taken from k_new / v_new inside the attention kernel and stored
    by it) against emm_kv_scatter followed by the attention call: same output bits, same pool bytes; with and
    without shared-prefix units."""
    print("case fused", name, flush=True)
    def build():
        return W.build_workload(name, "causal", "bf16", 1400 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                                page_size=16, prefix_lens=ctx, new_lens=new, share_group=group, shared_len=shared)
    bits = B.DeviceWorkload.to_numpy_bits
    ref = _gpu_run(build())                             # scatter, then plain decode attention
    _compare(ref.wl, ref)
    dw = B.DeviceWorkload(build())
    dw.out.zero_()
    dw.decode_step()
    torch.cuda.synchronize()
    assert bits(dw.out).tobytes() == bits(ref.out).tobytes()
    assert bits(dw.k_cache).tobytes() == bits(ref.k_cache).tobytes() and bits(dw.v_cache).tobytes() == bits(ref.v_cache).tobytes()
    assert np.array_equal(dw.lse.cpu().numpy(), ref.lse.cpu().numpy())
    if group is not None:
        ref.plan_shared()
        ref.out.zero_()
        ref.attention_shared()                          # pools already hold the new rows
        dw2 = B.DeviceWorkload(build())
        dw2.plan_shared()
        dw2.out.zero_()
        dw2.decode_step(shared=True)
        torch.cuda.synchronize()
        assert bits(dw2.out).tobytes() == bits(ref.out).tobytes()
        assert bits(dw2.k_cache).tobytes() == bits(ref.k_cache).tobytes() and bits(dw2.v_cache).tobytes() == bits(ref.v_cache).tobytes()


@pytest.mark.parametrize("seed", range(10))
def test_random_decode_batches(seed):
    """Random decode batches (head groupings, batch sizes, ragged contexts, runs of requests that share pages,
    requests without a token): the plain path, the path with units, and emm_decode_step for both, each against
    the oracle or, bit for bit, against its two-call counterpart."""
    rng = np.random.default_rng(5000 + seed)
    H, Hkv = [(8, 8), (28, 4), (32, 8), (16, 1), (12, 4), (6, 2)][int(rng.integers(6))]
    n_req = int(rng.integers(1, 21))
    ctx, new, group, shared = [], [], [], []
    g = 0
    while len(ctx) < n_req:
        run = int(min(rng.integers(1, 7), n_req - len(ctx)))           # a run of requests with common leading pages
        common = int(rng.choice([0, 0, 17, 32, 100, 512, 1500]))
        for _ in range(run):
            own = int(rng.choice([0, 1, 15, 31, 33, 200, 900, 2500]))
            ctx.append(common + own)
            new.append(0 if rng.random() < 0.1 else 1)
            group.append(g)
            shared.append(common)
        g += 1
    print("case random decode", seed, (H, Hkv), ctx, new, flush=True)
    bits = B.DeviceWorkload.to_numpy_bits

    def build():
        return W.build_workload("rnd_decode", "causal", "bf16", 5100 + seed, num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                                page_size=16, prefix_lens=ctx, new_lens=new, share_group=group, shared_len=shared)
    if sum(new) == 0:
        new[0] = 1
    ref = _gpu_run(build())
    _compare(ref.wl, ref)
    plain_out = bits(ref.out).copy()
    plan = ref.plan_shared()
    print("   units:", plan["num_units"], plan["unit_num_reqs"].tolist(), plan["unit_shared_len"].tolist(), flush=True)
    ref.out.zero_()
    ref.attention_shared()
    torch.cuda.synchronize()
    _compare(ref.wl, ref)
    shared_out = bits(ref.out).copy()
    for use_units, want in ((False, plain_out), (True, shared_out)):
        dw = B.DeviceWorkload(build())
        dw.plan_shared()
        dw.out.zero_()
        dw.decode_step(use_units)
        torch.cuda.synchronize()
        assert bits(dw.out).tobytes() == want.tobytes(), use_units
        assert bits(dw.k_cache).tobytes() == bits(ref.k_cache).tobytes()
        assert bits(dw.v_cache).tobytes() == bits(ref.v_cache).tobytes()


PAGE_SIZES = [32, 64, 128, 256]


@pytest.mark.parametrize("ps", PAGE_SIZES)
def test_page_sizes_prefill_and_cross(ps):
    """Pages of 32 .. 256 tokens (a page then holds 2 .. 16 of the 16-key blocks the kernels fetch): ragged
    lengths around page and tile edges, units cut along the keys, cross-attention, and the fp32 kernels."""
    print("case page size", ps, "prefill", flush=True)
    wl = W.build_workload("ps_prefill", "causal", "bf16", 6000 + ps, num_q_heads=28, num_kv_heads=4, head_dim=128,
                          page_size=ps, prefix_lens=[5000, 300, 0, 77, 1056, ps - 1, ps, 4 * ps + 1],
                          new_lens=[64, 200, 150, 3, 300, 2, ps + 1, 40])
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw, _sample_tokens(wl, 96, seed=ps)), flush=True)
    print("case page size", ps, "cut into 16 pieces", flush=True)
    wl = W.build_workload("ps_cut16", "causal", "bf16", 6100 + ps, num_q_heads=28, num_kv_heads=4, head_dim=128,
                          page_size=ps, prefix_lens=[17000], new_lens=[36])
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)
    print("case page size", ps, "cross", flush=True)
    wl = W.build_workload("ps_cross", "cross", "bf16", 6200 + ps, num_q_heads=32, num_kv_heads=8, head_dim=128,
                          page_size=ps, prefix_lens=[6404, 333, 0, 6404], new_lens=[100, 61, 5, 37],
                          share_group=[0, 1, 2, 0], shared_len=[6404, 0, 0, 6404])
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)
    print("case page size", ps, "fp32", flush=True)
    wl = W.build_workload("ps_f32", "causal", "f32", 6300 + ps, num_q_heads=4, num_kv_heads=1, head_dim=64,
                          page_size=ps, prefix_lens=[256, 100, 0], new_lens=[64, 3, ps + 3])
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)


@pytest.mark.parametrize("ps", PAGE_SIZES)
def test_page_sizes_decode(ps):
    """The decode step on pages of 32 .. 256 tokens: plain, with shared-prefix units, and fused with the scatter."""
    print("case page size", ps, "decode", flush=True)
    bits = B.DeviceWorkload.to_numpy_bits
    ctx = [700, 650, 900, 300, 1300, 18000, 0, ps - 1, ps, 2 * ps + 1]
    group = [0, 0, 1, 2, 2, 3, 4, 5, 6, 7]
    shared = [512, 512, 0, 256, 256, 0, 0, 0, 0, 0]

    def build():
        return W.build_workload("ps_decode", "causal", "bf16", 6400 + ps, num_q_heads=28, num_kv_heads=4, head_dim=128,
                                page_size=ps, prefix_lens=ctx, new_lens=[1] * len(ctx), share_group=group, shared_len=shared)
    ref = _gpu_run(build())                             # scatter, then the plain decode kernels
    print("   errors (max, mean, lse):", _compare(ref.wl, ref), flush=True)
    plain_out = bits(ref.out).copy()
    plan = ref.plan_shared()
    print("   units:", plan["num_units"], plan["unit_num_reqs"].tolist(), plan["unit_shared_len"].tolist(), flush=True)
    assert plan["num_units"] == 2 and plan["unit_shared_len"].tolist() == [512, 256]
    ref.out.zero_()
    ref.attention_shared()
    torch.cuda.synchronize()
    print("   errors (max, mean, lse):", _compare(ref.wl, ref), flush=True)
    shared_out = bits(ref.out).copy()
    for use_units, want in ((False, plain_out), (True, shared_out)):
        dw = B.DeviceWorkload(build())
        dw.plan_shared()
        dw.out.zero_()
        dw.decode_step(use_units)
        torch.cuda.synchronize()
        assert bits(dw.out).tobytes() == want.tobytes(), use_units
        assert bits(dw.k_cache).tobytes() == bits(ref.k_cache).tobytes()
        assert bits(dw.v_cache).tobytes() == bits(ref.v_cache).tobytes()


def test_calls_can_be_captured_in_a_hip_graph_and_replayed():
    """The library only launches kernels on the given stream (no allocation, no memset, no synchronisation), so a
    step can be captured in a HIP graph; every replay, with eager work between the replays, must reproduce the
    eager result bit for bit -- prefill (with cut units and the merge kernel), decode with units, and the fused step."""
    print("case graph capture", flush=True)
    bits = B.DeviceWorkload.to_numpy_bits
    prefill = W.build_workload("graph_prefill", "causal", "bf16", 1700, num_q_heads=28, num_kv_heads=4, head_dim=128,
                               page_size=16, prefix_lens=[5000, 300], new_lens=[64, 200])
    decode = W.build_workload("graph_decode", "causal", "bf16", 1701, num_q_heads=28, num_kv_heads=4, head_dim=128,
                              page_size=16, prefix_lens=[2100, 2200, 900, 40], new_lens=[1, 1, 1, 1],
                              share_group=[0, 0, 1, 2], shared_len=[2048, 2048, 0, 0])
    for wl, step in ((prefill, lambda d: d.step()), (decode, lambda d: (d.scatter(), d.attention_shared())),
                     (decode, lambda d: d.decode_step(True))):
        eager = _gpu_run(wl)
        if wl is decode:
            eager.plan_shared()
            eager.out.zero_()
            step(eager)
            torch.cuda.synchronize()
        want_out, want_k = bits(eager.out).tobytes(), bits(eager.k_cache).tobytes()
        dw = B.DeviceWorkload(wl)
        if wl is decode:
            dw.plan_shared()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step(dw)                                    # warm up on the capture stream
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step(dw)
        for replay in range(3):
            dw.out.zero_()                              # eager work and a synchronisation between the replays
            if dw.workspace is not None:
                dw.workspace.fill_(0x5A)                # stale workspace contents must not matter
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert bits(dw.out).tobytes() == want_out, replay
            assert bits(dw.k_cache).tobytes() == want_k, replay


def test_kv_page_migration_is_exact_and_checksummed():
    """Appendix B.5 on one GPU: a request's pages are packed, checksummed, unpacked into other pages of another
    pool; bytes and Adler-32 values must equal the reference's, a corrupted buffer must be reported, and decode
    attention over the migrated pages must give the same bits as over the original ones."""
    from oracle import kv_migrate_model as KM
    print("case kv page migration", flush=True)
    wl = W.build_workload("migrate", "causal", "bf16", 1500, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16,
                          prefix_lens=[3000, 37, 1200], new_lens=[1, 1, 1])
    dw = _gpu_run(wl)                                   # scatter + decode on the source pools
    src_out = B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()
    page_bytes = 4 * 16 * 128 * 2
    kc, vc = B.DeviceWorkload.to_numpy_bits(dw.k_cache), B.DeviceWorkload.to_numpy_bits(dw.v_cache)
    rng = np.random.default_rng(9)
    dst_pages = wl.num_pages + 11
    free = rng.permutation(dst_pages)
    new_table = np.full_like(wl.page_table, -1)
    kd = torch.full((dst_pages, 4, 16, 128), 7.0, dtype=torch.bfloat16, device="cuda:0")
    vd = torch.full_like(kd, -3.0)
    kd_ref, vd_ref = B.DeviceWorkload.to_numpy_bits(kd).copy(), B.DeviceWorkload.to_numpy_bits(vd).copy()
    taken = 0
    for r in range(wl.num_reqs):                        # one request at a time, as a migration would go
        n = -(-(int(wl.prefix_lens[r]) + 1) // 16)
        src_ids = wl.page_table[r, :n].astype(np.int32)
        dst_ids = free[taken:taken + n].astype(np.int32)
        taken += n
        new_table[r, :n] = dst_ids
        ids_d, dst_d = torch.from_numpy(src_ids).to("cuda:0"), torch.from_numpy(dst_ids).to("cuda:0")
        staging = torch.zeros(n * 2 * page_bytes, dtype=torch.uint8, device="cuda:0")
        sums = torch.zeros(n, dtype=torch.int32, device="cuda:0")
        B.emm_kv_pages_pack(dw.k_cache, dw.v_cache, wl.num_pages, page_bytes, ids_d, n, staging, sums)
        ref_staging, ref_sums = KM.pack(kc, vc, src_ids)
        assert staging.cpu().numpy().tobytes() == ref_staging.tobytes()
        assert (sums.cpu().numpy().view(np.uint32) == ref_sums).all()
        sums2 = torch.zeros_like(sums)
        bad = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        B.emm_kv_pages_unpack(staging, dst_d, n, kd, vd, dst_pages, page_bytes, sums2, sums, bad)
        kd_ref, vd_ref, ref_sums2 = KM.unpack(ref_staging, dst_ids, kd_ref, vd_ref)
        assert (sums2.cpu().numpy().view(np.uint32) == ref_sums2).all() and int(bad.item()) == 0
        if r == 0:                                      # a bit flipped in transit is counted, once per damaged page
            hurt = staging.clone()
            hurt[5 * 2 * page_bytes + 123] ^= 4
            hurt[(n - 1) * 2 * page_bytes] ^= 1
            scratch_k, scratch_v = kd.clone(), vd.clone()
            B.emm_kv_pages_unpack(hurt, dst_d, n, scratch_k, scratch_v, dst_pages, page_bytes, None, sums, bad)
            assert int(bad.item()) == 2
    torch.cuda.synchronize()
    assert B.DeviceWorkload.to_numpy_bits(kd).tobytes() == kd_ref.tobytes()
    assert B.DeviceWorkload.to_numpy_bits(vd).tobytes() == vd_ref.tobytes()
    # the destination instance continues decoding: same query, migrated pages, other page ids -> same bits
    pt_d = torch.from_numpy(new_table).to("cuda:0")
    batch = B.make_batch(num_reqs=wl.num_reqs, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16,
                         num_pages=dst_pages, max_pages_per_req=wl.max_pages_per_req, total_new_tokens=3, max_new_len=1,
                         dtype="bf16", softmax_scale=wl.softmax_scale, page_table=pt_d, prefix_lens=dw.prefix_lens,
                         new_lens=dw.new_lens, cu_new_lens=dw.cu_new_lens)
    out = torch.zeros_like(dw.out)
    ws = torch.empty(B.emm_prefill_attn_workspace_size(batch), dtype=torch.uint8, device="cuda:0")
    B.emm_decode_attn(batch, dw.q, kd, vd, out, None, ws)
    torch.cuda.synchronize()
    assert B.DeviceWorkload.to_numpy_bits(out).tobytes() == src_out


def test_kv_page_checksum_of_the_largest_page():
    """Pages of 1 MiB per pool (the largest admitted: e.g. 16 KV heads x 256 tokens x 128 channels in bf16) filled
    with large byte values: the position-weighted sum of a 16-byte chunk alone passes 2^32 there.  Bytes and
    Adler-32 values against the reference, pack and unpack."""
    from oracle import kv_migrate_model as KM
    print("case kv page checksum, 1 MiB pages", flush=True)
    page_bytes = 1 << 20
    rng = np.random.default_rng(12)
    kc = rng.integers(200, 256, (3, page_bytes), dtype=np.uint8)
    vc = rng.integers(0, 256, (3, page_bytes), dtype=np.uint8)
    kc[1, :] = 0xFF
    vc[1, :] = 0xFF
    kc[2, :] = 0
    vc[2, :] = 0
    kc[2, :4096] = 0xFF
    k_d, v_d = torch.from_numpy(kc).to("cuda:0"), torch.from_numpy(vc).to("cuda:0")
    ids = np.array([2, 0, 1], np.int32)
    ids_d = torch.from_numpy(ids).to("cuda:0")
    staging = torch.zeros(3 * 2 * page_bytes, dtype=torch.uint8, device="cuda:0")
    sums = torch.zeros(3, dtype=torch.int32, device="cuda:0")
    B.emm_kv_pages_pack(k_d, v_d, 3, page_bytes, ids_d, 3, staging, sums)
    ref_staging, ref_sums = KM.pack(kc, vc, ids)
    assert staging.cpu().numpy().tobytes() == ref_staging.tobytes()
    assert (sums.cpu().numpy().view(np.uint32) == ref_sums).all(), (sums.cpu().numpy().view(np.uint32), ref_sums)
    k2, v2 = torch.zeros_like(k_d), torch.zeros_like(v_d)
    sums2 = torch.zeros_like(sums)
    bad = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    dst = np.array([1, 2, 0], np.int32)
    B.emm_kv_pages_unpack(staging, torch.from_numpy(dst).to("cuda:0"), 3, k2, v2, 3, page_bytes, sums2, sums, bad)
    k_ref, v_ref, ref_sums2 = KM.unpack(ref_staging, dst, np.zeros_like(kc), np.zeros_like(vc))
    assert (sums2.cpu().numpy().view(np.uint32) == ref_sums2).all() and int(bad.item()) == 0
    assert k2.cpu().numpy().tobytes() == k_ref.tobytes() and v2.cpu().numpy().tobytes() == v_ref.tobytes()


def _plant_key(wl, r, pos, value):
    """Every channel of key `pos` of request r (all KV heads) becomes `value`: in the pool if the key is cached,
    else in k_new."""
    bits = W.to_bf16_bits(np.full((wl.num_kv_heads, wl.head_dim), value, np.float32))
    P = int(wl.prefix_lens[r])
    if wl.kind == "cross" or pos < P:
        wl.k_cache[wl.page_table[r, pos // wl.page_size], :, pos % wl.page_size, :] = bits
    else:
        wl.k_new[int(wl.cu_new_lens[r]) + pos - P] = bits


STEEP_CASES = [
    # name, kind, H, Hkv, prefix lens, new lens, planted keys (request, position, value of every channel)
    # With every query channel 4.0, a key of all 0.6 scores 39 powers of two and a key of all 4.0 scores 261 powers of two
    # above the usual ones: the first makes the kernel raise its reference exponent on the way (row sums past 2^20), the
    # second overflows single precision between two tiles, which the kernel must notice and do the unit again with true
    # running maxima.
    ("steep_mid", "causal", 28, 4, [100, 0], [300, 500], [(0, 250, 0.6), (1, 130, 0.6), (1, 390, 0.6)]),
    ("steep_big", "causal", 28, 4, [100, 0], [300, 500], [(0, 250, 4.0), (1, 130, 0.6), (1, 390, 4.0)]),
    ("steep_big_prefix", "causal", 8, 2, [4000, 700], [200, 40], [(0, 3000, 4.0), (0, 600, 0.6), (1, 699, 4.0)]),
    ("steep_cut", "causal", 28, 4, [5000], [64], [(0, 3000, 4.0), (0, 900, 0.6)]),         # pieces of cut units, merged
    ("steep_cut_mid", "causal", 28, 4, [5000], [64], [(0, 3000, 0.6), (0, 4500, 0.6)]),
    ("steep_cross", "cross", 32, 8, [6404, 1601], [100, 300], [(0, 5000, 4.0), (1, 1600, 4.0), (1, 70, 0.6)]),
    ("steep_first_tile", "causal", 28, 4, [0], [400], [(0, 3, 4.0)]),                       # the dominant key comes first
]


@pytest.mark.parametrize("name,kind,H,Hkv,prefix,new,planted", STEEP_CASES)
def test_scores_that_jump_between_tiles(name, kind, H, Hkv, prefix, new, planted):
    """The prefill kernel takes no row maxima on the way (it watches the row sums); scores that rise steeply from one
    key tile to a later one must still come out right: by raising the reference exponent, or, past the range of
    single precision, by the second, careful pass."""
    print("case", name, flush=True)
    wl = W.build_workload(name, kind, "bf16", 1700 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=prefix, new_lens=new)
    wl.q[...] = W.to_bf16_bits(np.full(wl.q.shape, 4.0, np.float32))
    for r, pos, value in planted:
        _plant_key(wl, r, pos, value)
    dw = _gpu_run(wl)
    print("   errors (max, mean, lse):", _compare(wl, dw), flush=True)
    first = B.DeviceWorkload.to_numpy_bits(dw.out).tobytes()
    dw.out.zero_()
    dw.attention()                                      # same bits on a second run (stale workspace, same decisions)
    torch.cuda.synchronize()
    assert B.DeviceWorkload.to_numpy_bits(dw.out).tobytes() == first


def test_f32_head_dim_128_and_cross():
    print("case f32 d=128 causal + cross", flush=True)
    wl = W.build_workload("f32_128", "causal", "f32", 700, num_q_heads=6, num_kv_heads=2, head_dim=128,
                          page_size=16, prefix_lens=[33, 0, 70], new_lens=[17, 65, 1])
    _compare(wl, _gpu_run(wl))
    wl = W.build_workload("f32_cross", "cross", "f32", 701, num_q_heads=4, num_kv_heads=1, head_dim=64,
                          page_size=16, prefix_lens=[0, 70, 16], new_lens=[3, 9, 66])
    _compare(wl, _gpu_run(wl))


def test_garbage_in_unused_slots_is_ignored():
    """Slots past a request's tokens (tail of the last page) and unreferenced pages may hold anything,
    including NaN and Inf bit patterns; results must not change."""
    print("case garbage slots", flush=True)
    wl = W.build_workload("garbage", "causal", "bf16", 800, num_q_heads=8, num_kv_heads=2, head_dim=128,
                          page_size=16, prefix_lens=[37, 0, 64], new_lens=[70, 5, 130])
    ref = _gpu_run(wl)
    ref_out = B.DeviceWorkload.to_numpy_bits(ref.out)
    for pattern in (0x7FC0, 0x7F80, 0xFF80):            # NaN, +Inf, -Inf
        wl2 = W.build_workload("garbage", "causal", "bf16", 800, num_q_heads=8, num_kv_heads=2, head_dim=128,
                               page_size=16, prefix_lens=[37, 0, 64], new_lens=[70, 5, 130])
        for pool in (wl2.k_cache, wl2.v_cache):
            pool[pool == W.SENTINEL_BF16_BITS] = pattern
        dw = _gpu_run(wl2)
        assert B.DeviceWorkload.to_numpy_bits(dw.out).tobytes() == ref_out.tobytes(), hex(pattern)
    wl3 = W.build_workload("garbage_x", "cross", "bf16", 801, num_q_heads=8, num_kv_heads=2, head_dim=128,
                           page_size=16, prefix_lens=[37, 100], new_lens=[40, 3])
    ref = B.DeviceWorkload.to_numpy_bits(_gpu_run(wl3).out)
    for pool in (wl3.k_cache, wl3.v_cache):
        pool[pool == W.SENTINEL_BF16_BITS] = 0x7FC0
    assert B.DeviceWorkload.to_numpy_bits(_gpu_run(wl3).out).tobytes() == ref.tobytes()


def test_scatter_bit_exact_with_arbitrary_bit_patterns():
    """The scatter moves bytes: NaN payloads, denormals and negative zeros survive unchanged."""
    print("case scatter bit patterns", flush=True)
    for dtype, cfg in (("bf16", 2), ("f32", 1)):
        wl = W.config(cfg, 4)
        rng = np.random.default_rng(900)
        bits = rng.integers(0, 2 ** 16, size=wl.k_new.shape, dtype=np.uint16) if dtype == "bf16" else None
        if dtype == "bf16":
            wl.k_new = bits
            wl.v_new = rng.integers(0, 2 ** 16, size=wl.v_new.shape, dtype=np.uint16)
        else:
            wl.k_new = rng.integers(0, 2 ** 32, size=wl.k_new.shape, dtype=np.uint32).view(np.float32)
            wl.v_new = rng.integers(0, 2 ** 32, size=wl.v_new.shape, dtype=np.uint32).view(np.float32)
        dw = B.DeviceWorkload(wl)
        dw.scatter()
        torch.cuda.synchronize()
        kc, vc = oracle.kv_scatter(wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, wl.k_new,
                                   wl.v_new, wl.k_cache, wl.v_cache)
        if dtype == "bf16":
            got_k, got_v = B.DeviceWorkload.to_numpy_bits(dw.k_cache), B.DeviceWorkload.to_numpy_bits(dw.v_cache)
        else:
            got_k, got_v = dw.k_cache.cpu().numpy(), dw.v_cache.cpu().numpy()
        assert got_k.tobytes() == kc.tobytes() and got_v.tobytes() == vc.tobytes()


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 4), (5, 8)])
def test_page_permutation_invariance_bitwise(cfg, shrink):
    """Relabelling physical pages (pool and table together) must not change a single output bit."""
    print("case permutation cfg=%d" % cfg, flush=True)
    wl = W.config(cfg, shrink)
    out = B.DeviceWorkload.to_numpy_bits(_gpu_run(wl).out)
    perm = np.random.default_rng(5).permutation(wl.num_pages)
    wl2 = W.config(cfg, shrink)
    wl2.k_cache = np.empty_like(wl.k_cache)
    wl2.v_cache = np.empty_like(wl.v_cache)
    wl2.k_cache[perm] = wl.k_cache
    wl2.v_cache[perm] = wl.v_cache
    wl2.page_table = np.where(wl.page_table >= 0, perm[np.maximum(wl.page_table, 0)], -1).astype(np.int32)
    out2 = B.DeviceWorkload.to_numpy_bits(_gpu_run(wl2).out)
    assert out.tobytes() == out2.tobytes()


def test_run_to_run_determinism_and_constant_v():
    print("case determinism", flush=True)
    wl = W.config(4, 8)
    a = _gpu_run(wl)
    b = _gpu_run(wl)
    assert B.DeviceWorkload.to_numpy_bits(a.out).tobytes() == B.DeviceWorkload.to_numpy_bits(b.out).tobytes()
    assert a.lse.cpu().numpy().tobytes() == b.lse.cpu().numpy().tobytes()
    # V == 1 everywhere the request has tokens: the output is the sum of the softmax weights
    wl.v_cache[wl.v_cache != W.SENTINEL_BF16_BITS] = 0x3F80
    wl.v_new[...] = 0x3F80
    out = as_f64(B.DeviceWorkload.to_numpy_bits(_gpu_run(wl).out))
    assert np.abs(out - 1.0).max() <= 8e-3


def test_error_codes_on_device():
    """Status codes through the binding with real device tensors."""
    wl = W.config(1, 1)
    dw = B.DeviceWorkload(wl)
    with pytest.raises(B.EmmError) as e:
        B.emm_prefill_attn(dw.batch, dw.q, dw.k_cache, dw.v_cache, None)
    assert e.value.status == B.EMM_ERR_NULL
    bad = B.DeviceWorkload(wl)
    bad.batch.page_size = 8
    with pytest.raises(B.EmmError) as e:
        bad.scatter()
    assert e.value.status == B.EMM_ERR_UNSUPPORTED


@pytest.mark.parametrize("name,kind,H,Hkv,prefix,new", [
    ("ws_cut32", "causal", 28, 4, [16384], [36]),                    # uniform: one unit per second XCD, 32 pieces: exact size
    ("ws_ragged", "causal", 28, 4, [9000, 300, 5000], [64, 200, 36]),   # ragged: sized from bounds
    ("ws_uneven", "cross", 32, 8, [6404] * 7, [600, 350, 700, 280, 512, 90, 768]),   # 22 units left over: two uneven pieces each
])
def test_workspace_of_exactly_the_stated_size_is_enough(name, kind, H, Hkv, prefix, new):
    """The kernels must stay inside emm_prefill_attn_workspace_size bytes: a buffer of exactly that size followed by a
    guard region, which must come back untouched, and the same output bits as with a roomy workspace."""
    print("case", name, flush=True)
    wl = W.build_workload(name, kind, "bf16", 2300 + len(name), num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=prefix, new_lens=new)
    ref = _gpu_run(wl)
    _compare(wl, ref)
    need = B.emm_prefill_attn_workspace_size(ref.batch)
    assert need > 0
    guard = 1 << 16
    buf = torch.full((need + guard,), 0xA5, dtype=torch.uint8, device="cuda:0")
    dw = B.DeviceWorkload(wl)
    dw.workspace = buf[:need]
    dw.out.zero_()
    dw.step()
    torch.cuda.synchronize()
    assert bool((buf[need:] == 0xA5).all()), "the kernels wrote past the stated workspace size"
    assert B.DeviceWorkload.to_numpy_bits(dw.out).tobytes() == B.DeviceWorkload.to_numpy_bits(ref.out).tobytes()
    too_small = buf[:need - 16]
    with pytest.raises(B.EmmError) as e:
        (B.emm_prefill_attn if kind == "causal" else B.emm_cross_attn)(dw.batch, dw.q, dw.k_cache, dw.v_cache, dw.out, dw.lse, too_small)
    assert e.value.status == B.EMM_ERR_WORKSPACE


def test_two_streams_with_their_own_workspaces():
    """The library keeps no state between calls: two batches stepped on two streams at the same time, each with
    its own workspace, give the bits they give when stepped one after the other.  (Both streams have the default
    priority.)"""
    print("case two streams", flush=True)
    bits = B.DeviceWorkload.to_numpy_bits
    def build_a():
        return W.build_workload("stream_a", "causal", "bf16", 1800, num_q_heads=28, num_kv_heads=4, head_dim=128,
                                page_size=16, prefix_lens=[9000, 300, 5000], new_lens=[64, 200, 36])      # cut units, merge kernel
    def build_b():
        return W.build_workload("stream_b", "causal", "bf16", 1801, num_q_heads=32, num_kv_heads=8, head_dim=128,
                                page_size=16, prefix_lens=[2100, 2200, 900, 40, 7000], new_lens=[1, 1, 1, 1, 1])   # decode pieces
    ref_a, ref_b = _gpu_run(build_a()), _gpu_run(build_b())
    want_a, want_b = bits(ref_a.out).copy(), bits(ref_b.out).copy()
    dw_a, dw_b = B.DeviceWorkload(build_a()), B.DeviceWorkload(build_b())
    torch.cuda.synchronize()
    s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()
    for _ in range(3):                                  # the later rounds overwrite what the earlier ones wrote
        dw_a.out.zero_()
        dw_b.out.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s_a):
            dw_a.step()
        with torch.cuda.stream(s_b):
            dw_b.step()
        with torch.cuda.stream(s_a):
            dw_a.attention()
        with torch.cuda.stream(s_b):
            dw_b.attention()
        torch.cuda.synchronize()
        assert bits(dw_a.out).tobytes() == want_a.tobytes()
        assert bits(dw_b.out).tobytes() == want_b.tobytes()
