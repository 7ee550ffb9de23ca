"""Seeded synthetic inputs for the prefix-cached paged prefill path.

This module only *draws data*: request lengths, page tables, Q/K/V values and a
pre-filled KV pool.  It contains none of the attention or scatter arithmetic, so
both the CPU oracle's tests and the HIP path's tests can consume it without
sharing any of the method's code.

The five named workloads stand in for the request mixes the paper serves
(ShareGPT-4o / VisualWebInstruct requests on Qwen2.5-VL-7B and
Llama-3.2-Vision-11B, Section 4.1): their head counts and head dimension are
those models' attention shapes, and their prefix lengths are of the size of the
image-token counts in Table 1.  The datasets and weights themselves are not
used; every value is drawn from a numpy ``Generator(PCG64(seed))``.

Layouts (all C-contiguous numpy arrays):
  q            [T][H][d]                 packed over requests by ``cu_new_lens``
  k_new, v_new [T][Hkv][d]               K/V of the new tokens (``None`` for cross-attention)
  k_cache, v_cache [num_pages][Hkv][page_size][d]   the paged pool (Appendix A)
  page_table   [B][max_pages_per_req]    int32 physical page ids, -1 where unused
bf16 tensors are carried as ``uint16`` bit patterns; fp32 tensors as ``float32``.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence

import numpy as np

# Recognisable finite fill for pool slots that hold no token (about 1e30): a
# kernel that wrongly attends to such a slot produces an obviously wrong row,
# and a scatter that writes outside its slots destroys the pattern.
SENTINEL_F32 = np.float32(1.0e30)
SENTINEL_BF16_BITS = np.uint16(0x7149)  # ~9.95e29 in bf16


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 values to bf16 (round-to-nearest-even) and return the bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 (exact)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclasses.dataclass
class Workload:
    name: str
    kind: str                 # "causal" (prefix-cached prefill) or "cross" (mask-free cross-attention)
    dtype: str                # "f32" or "bf16"
    num_reqs: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    max_pages_per_req: int
    softmax_scale: float
    page_table: np.ndarray    # int32 [B][max_pages_per_req]
    prefix_lens: np.ndarray   # int32 [B]  tokens already valid in the pages
    new_lens: np.ndarray      # int32 [B]  new tokens (= query rows) per request
    cu_new_lens: np.ndarray   # int32 [B+1]
    q: np.ndarray
    k_new: Optional[np.ndarray]
    v_new: Optional[np.ndarray]
    k_cache: np.ndarray       # pool *before* the scatter: prefix slots filled, the rest sentinel
    v_cache: np.ndarray
    notes: dict = dataclasses.field(default_factory=dict)

    @property
    def total_new_tokens(self) -> int:
        return int(self.cu_new_lens[-1])

    @property
    def max_new_len(self) -> int:
        return int(self.new_lens.max()) if self.num_reqs else 0

    @property
    def elt_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    def attended_pairs(self) -> int:
        """Number of (query, key) pairs one query head attends to, summed over requests."""
        total = 0
        for p, n in zip(self.prefix_lens.tolist(), self.new_lens.tolist()):
            total += n * p + (n * (n + 1) // 2 if self.kind == "causal" else 0)
        return total

    def attention_flops(self) -> int:
        """Algorithmic FLOPs: 2*d for each score and 2*d for each weighted-V row, unmasked pairs only."""
        return 4 * self.head_dim * self.num_q_heads * self.attended_pairs()

    def kv_read_bytes(self) -> int:
        """Bytes of K and V a step must read at least once: every slot the queries of a request can see,
        all KV heads (what bounds the decode step, where nothing is reused)."""
        total = 0
        for p, n in zip(self.prefix_lens.tolist(), self.new_lens.tolist()):
            if n > 0:
                total += p + (n if self.kind == "causal" else 0)
        return 2 * total * self.num_kv_heads * self.head_dim * self.elt_bytes

    def kv_distinct_read_bytes(self) -> int:
        """As kv_read_bytes, but a physical page that several requests reference counts once (with the most
        slots any of them sees in it): what HBM has to deliver at least when shared pages are read once."""
        ps = self.page_size
        seen = {}
        for r, (p, n) in enumerate(zip(self.prefix_lens.tolist(), self.new_lens.tolist())):
            if n <= 0:
                continue
            ctx = p + (n if self.kind == "causal" else 0)
            for lp in range(-(-ctx // ps)):
                page = int(self.page_table[r, lp])
                seen[page] = max(seen.get(page, 0), min(ps, ctx - lp * ps))
        return 2 * sum(seen.values()) * self.num_kv_heads * self.head_dim * self.elt_bytes

    def scatter_bytes(self) -> int:
        """Bytes the KV scatter must move: read K,V of the new tokens and write them once."""
        if self.kind != "causal":
            return 0
        return 4 * self.total_new_tokens * self.num_kv_heads * self.head_dim * self.elt_bytes


def _draw(rng: np.random.Generator, shape, dtype: str, outlier_frac: float = 0.0,
          outlier_mul: float = 1.0) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if outlier_frac > 0.0:
        mask = rng.random(size=shape, dtype=np.float32) < np.float32(outlier_frac)
        x = np.where(mask, x * np.float32(outlier_mul), x).astype(np.float32)
    return x if dtype == "f32" else to_bf16_bits(x)


def build_workload(name: str, kind: str, dtype: str, seed: int, *, num_q_heads: int, num_kv_heads: int,
                   head_dim: int, page_size: int, prefix_lens: Sequence[int], new_lens: Sequence[int],
                   share_group: Optional[Sequence[int]] = None, shared_len: Optional[Sequence[int]] = None,
                   spare_pages: int = 8, softmax_scale: Optional[float] = None,
                   k_outlier_frac: float = 0.0, k_outlier_mul: float = 1.0,
                   identity_pages: bool = False, notes: Optional[dict] = None) -> Workload:
    """Draw one batch.

    ``share_group[r]`` names the group whose leading ``shared_len[r]`` tokens live in physical pages common to every member of the group; all later pages of
    a request are private.  For ``kind == "causal"`` the new tokens are *not* yet in the pool
    (the scatter puts them there); for ``kind == "cross"`` the pool already holds everything and
    there are no new K/V.
    """
    assert kind in ("causal", "cross") and dtype in ("f32", "bf16")
    rng = np.random.default_rng(np.random.PCG64(seed))
    B = len(prefix_lens)
    prefix = np.asarray(prefix_lens, dtype=np.int64)
    new = np.asarray(new_lens, dtype=np.int64)
    ctx = prefix + (new if kind == "causal" else 0)         # tokens that end up in pages
    pages_per_req = [int(-(-int(c) // page_size)) for c in ctx]
    if share_group is None:
        share_group = list(range(B))
        shared_len = [0] * B
    # a shared page is read-only, so under "causal" (where the scatter appends after the prefix)
    # only whole prefix pages may be shared; under "cross" nothing is written and the trailing
    # partial page is shared as well
    shared_pages = []
    for r in range(B):
        n_tok = min(int(shared_len[r]), int(prefix[r]))
        shared_pages.append(-(-n_tok // page_size) if kind == "cross" else n_tok // page_size)

    # logical -> physical assignment: walk the requests, give each group's shared pages one id
    # each (first member allocates), then private ids; finally relabel through a permutation.
    next_id = 0
    group_pages: dict = {}
    logical_rows: List[List[int]] = []
    for r in range(B):
        g = share_group[r]
        row: List[int] = []
        if shared_pages[r] > 0:
            have = group_pages.setdefault(g, [])
            while len(have) < shared_pages[r]:
                have.append(next_id)
                next_id += 1
            row.extend(have[:shared_pages[r]])
        while len(row) < pages_per_req[r]:
            row.append(next_id)
            next_id += 1
        logical_rows.append(row)
    num_pages = next_id + spare_pages
    perm = np.arange(num_pages) if identity_pages else rng.permutation(num_pages)
    max_pages = max([1] + pages_per_req)
    page_table = np.full((B, max_pages), -1, dtype=np.int32)
    for r, row in enumerate(logical_rows):
        page_table[r, :len(row)] = perm[np.asarray(row, dtype=np.int64)] if row else []

    d, Hkv, H = head_dim, num_kv_heads, num_q_heads
    if dtype == "f32":
        k_cache = np.full((num_pages, Hkv, page_size, d), SENTINEL_F32, dtype=np.float32)
        v_cache = np.full((num_pages, Hkv, page_size, d), SENTINEL_F32, dtype=np.float32)
    else:
        k_cache = np.full((num_pages, Hkv, page_size, d), SENTINEL_BF16_BITS, dtype=np.uint16)
        v_cache = np.full((num_pages, Hkv, page_size, d), SENTINEL_BF16_BITS, dtype=np.uint16)

    # prefix K/V: members of a group see the same values in their shared pages because the
    # pages are physically the same; the private remainder is drawn per request.
    filled = np.zeros(num_pages, dtype=bool)
    for r in range(B):
        P = int(prefix[r])
        if P == 0:
            continue
        kp = _draw(rng, (P, Hkv, d), dtype, k_outlier_frac, k_outlier_mul)
        vp = _draw(rng, (P, Hkv, d), dtype)
        for lp in range(-(-P // page_size)):
            pg = int(page_table[r, lp])
            if lp < shared_pages[r] and filled[pg]:
                continue                                   # already written by an earlier group member
            lo, hi = lp * page_size, min(P, (lp + 1) * page_size)
            k_cache[pg, :, :hi - lo, :] = np.transpose(kp[lo:hi], (1, 0, 2))
            v_cache[pg, :, :hi - lo, :] = np.transpose(vp[lo:hi], (1, 0, 2))
            filled[pg] = True

    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(new)
    T = int(cu[-1])
    q = _draw(rng, (T, H, d), dtype)
    if kind == "causal":
        k_new = _draw(rng, (T, Hkv, d), dtype, k_outlier_frac, k_outlier_mul)
        v_new = _draw(rng, (T, Hkv, d), dtype)
    else:
        k_new = v_new = None
    scale = float(softmax_scale) if softmax_scale is not None else 1.0 / math.sqrt(d)
    return Workload(name=name, kind=kind, dtype=dtype, num_reqs=B, num_q_heads=H, num_kv_heads=Hkv,
                    head_dim=d, page_size=page_size, num_pages=num_pages, max_pages_per_req=max_pages,
                    softmax_scale=scale, page_table=page_table,
                    prefix_lens=prefix.astype(np.int32), new_lens=new.astype(np.int32), cu_new_lens=cu,
                    q=q, k_new=k_new, v_new=v_new, k_cache=k_cache, v_cache=v_cache,
                    notes=dict(notes or {}))


# --------------------------------------------------------------------------------------
# The five named workloads.  ``shrink`` divides every length (kept >= 1) so that tests can
# run the same structure at a size a CPU finishes quickly; the bench always uses shrink=1.
# --------------------------------------------------------------------------------------
SEEDS = {1: 1001, 2: 1002, 3: 1003, 4: 1004, 5: 1005}


def _s(x: int, shrink: int) -> int:
    return max(1, int(x) // shrink)


def config1(shrink: int = 1) -> Workload:
    """Tiny prefix-cached prefill in fp32: 1 request, 4 query heads on 1 KV head, d=64, 256 cached + 64 new.

    The pool has 64 physical pages; the request's 20 logical pages are the first 20 entries of a
    seeded permutation of them."""
    P, N = _s(256, shrink), _s(64, shrink)
    pages = -(-(P + N) // 16)
    return build_workload("cfg1_tiny_f32", "causal", "f32", SEEDS[1], num_q_heads=4, num_kv_heads=1,
                          head_dim=64, page_size=16, prefix_lens=[P], new_lens=[N],
                          spare_pages=64 - pages if shrink == 1 else 4)


def config2(shrink: int = 1) -> Workload:
    """Image-prefix batch: 8 requests, 28/4 heads, d=128; 1024 image + 32 system-text tokens cached,
    requests 0-3 and 4-7 share their prefix pages; 128..512 new text tokens each."""
    rng = np.random.default_rng(np.random.PCG64(SEEDS[2] + 7919))
    P = _s(1024, shrink) + _s(32, shrink)
    new = [int(v) for v in rng.integers(_s(128, shrink), _s(512, shrink) + 1, size=8)]
    return build_workload("cfg2_image_prefix", "causal", "bf16", SEEDS[2], num_q_heads=28, num_kv_heads=4,
                          head_dim=128, page_size=16, prefix_lens=[P] * 8, new_lens=new,
                          share_group=[0, 0, 0, 0, 1, 1, 1, 1], shared_len=[P] * 8, spare_pages=16)


def config3(shrink: int = 1) -> Workload:
    """Long video-prefix prefill: 2 requests, 28/4 heads, d=128; 64 frames x 256 tokens cached plus 2048
    new tokens each; every K element is independently multiplied by 8 with probability 0.01."""
    P, N = _s(64 * 256, shrink), _s(2048, shrink)
    return build_workload("cfg3_video_prefix", "causal", "bf16", SEEDS[3], num_q_heads=28, num_kv_heads=4,
                          head_dim=128, page_size=16, prefix_lens=[P, P], new_lens=[N, N],
                          spare_pages=64, k_outlier_frac=0.01, k_outlier_mul=8.0)


def config4(shrink: int = 1) -> Workload:
    """Mixed varlen batch: 32 requests, 32/8 heads, d=128.  Sixteen text-only requests (no prefix,
    log-uniform 256..2048 new tokens) and sixteen multimodal ones (image prefix of 576..4096 tokens of
    which a fraction 0, 0.5 or 1 is cached, the rest recomputed as new tokens, plus 64..512 new text
    tokens); request order shuffled; all pages private; cached prefixes need not be page aligned."""
    rng = np.random.default_rng(np.random.PCG64(SEEDS[4] + 7919))
    prefix, new = [], []
    for _ in range(16):
        n = int(round(math.exp(rng.uniform(math.log(256), math.log(2048)))))
        prefix.append(0)
        new.append(_s(n, shrink))
    for _ in range(16):
        l_img = int(rng.integers(576, 4096 + 1))
        frac = float(rng.choice([0.0, 0.5, 1.0]))
        text = int(rng.integers(64, 512 + 1))
        p = int(math.floor(frac * l_img))
        prefix.append(p // shrink if shrink > 1 else p)
        new.append(_s((l_img - p) + text, shrink))
    order = rng.permutation(32)
    prefix = [prefix[i] for i in order]
    new = [new[i] for i in order]
    return build_workload("cfg4_mixed_varlen", "causal", "bf16", SEEDS[4], num_q_heads=32, num_kv_heads=8,
                          head_dim=128, page_size=16, prefix_lens=prefix, new_lens=new, spare_pages=32)


def config5(shrink: int = 1) -> Workload:
    """Cross-attention for an encoder-decoder MLLM: 16 requests, 32/8 heads, d=128; 256..1024 text
    queries attend without mask to 6404 cached image tokens (4 tiles x 1601, so the last page holds
    4 valid tokens); requests (0,1), (2,3), ... share all their pages."""
    rng = np.random.default_rng(np.random.PCG64(SEEDS[5] + 7919))
    lkv = 4 * 1601 if shrink == 1 else max(1, (4 * 1601) // shrink) | 1
    nq = [int(v) for v in rng.integers(_s(256, shrink), _s(1024, shrink) + 1, size=16)]
    wl = build_workload("cfg5_cross_attn", "cross", "bf16", SEEDS[5], num_q_heads=32, num_kv_heads=8,
                        head_dim=128, page_size=16, prefix_lens=[lkv] * 16, new_lens=nq,
                        share_group=[r // 2 for r in range(16)], shared_len=[lkv] * 16, spare_pages=16)
    return wl


def decode_config(name: str, shrink: int = 1) -> Workload:
    """Decode-step batches (one new token per request, the stage after prefill): the contexts that the
    prefill workloads leave behind.
      decode_video_b8   8 requests with the video context of config 3 (16384 + 2048 tokens), 28/4 heads
      decode_mixed_b32  the 32 requests of config 4 after their prefill (context = prefix + new), 32/8 heads
      decode_b64_8k     64 requests of 8192 tokens, 28/4 heads
      decode_b1_16k, decode_b1_128k   a single request (latency regime), 28/4 heads
    and two with shared prefix pages (requests about the same video / the same system prompt and image):
      decode_shared_video_b8   as decode_video_b8, the 16384 video tokens in pages common to all 8 requests
      decode_shared_video_b32  8 videos with 4 requests each (402 MB of distinct K/V: more than the caches hold)
      decode_shared_image_b32  32 requests in 4 groups of 8, each group sharing 2880 tokens (system prompt +
                               image), then 200..1500 private tokens, 32/8 heads"""
    share_group = shared_len = None
    if name == "decode_video_b8":
        ctx, H, Hkv, seed = [_s(16384 + 2048, shrink)] * 8, 28, 4, 2001
    elif name == "decode_mixed_b32":
        c4 = config4(shrink)
        ctx, H, Hkv, seed = [int(p) + int(n) for p, n in zip(c4.prefix_lens, c4.new_lens)], 32, 8, 2002
    elif name == "decode_b64_8k":
        ctx, H, Hkv, seed = [_s(8192, shrink)] * 64, 28, 4, 2003
    elif name == "decode_b1_16k":
        ctx, H, Hkv, seed = [_s(16384, shrink)], 28, 4, 2007
    elif name == "decode_b1_128k":
        ctx, H, Hkv, seed = [_s(131072, shrink)], 28, 4, 2008
    elif name == "decode_shared_video_b8":
        ctx, H, Hkv, seed = [_s(16384 + 2048, shrink)] * 8, 28, 4, 2004
        share_group, shared_len = [0] * 8, [_s(16384, shrink)] * 8
    elif name == "decode_shared_video_b32":
        ctx, H, Hkv, seed = [_s(16384 + 2048, shrink)] * 32, 28, 4, 2006
        share_group, shared_len = [r // 4 for r in range(32)], [_s(16384, shrink)] * 32
    elif name == "decode_shared_image_b32":
        rng = np.random.default_rng(np.random.PCG64(2005 + 7919))
        shared = _s(2880, shrink)
        ctx = [shared + _s(int(rng.integers(200, 1501)), shrink) for _ in range(32)]
        H, Hkv, seed = 32, 8, 2005
        share_group, shared_len = [r // 8 for r in range(32)], [shared] * 32
    else:
        raise KeyError(name)
    return build_workload(name, "causal", "bf16", seed, num_q_heads=H, num_kv_heads=Hkv, head_dim=128,
                          page_size=16, prefix_lens=ctx, new_lens=[1] * len(ctx), share_group=share_group,
                          shared_len=shared_len, spare_pages=8)


def suffix_config(name: str, shrink: int = 1) -> Workload:
    """Prefill batches as they look after a large prefix-cache hit: a long cached context and a short new
    suffix (the question about a video or image that was seen before), 28/4 heads.  Few rows, many keys:
    the latency of the long context has to be spread over the chip by cutting along the keys.
      suffix_b1_16k_n36   1 request, 16384 cached + 36 new tokens
      suffix_b8_16k_n36   8 requests of that shape (private pages)
      suffix_b8_16k_n4    8 requests, 16384 cached + 4 new tokens
      suffix_b32_4k_n36   32 requests, 4096 cached + 36 new tokens"""
    shapes = {"suffix_b1_16k_n36": (1, 16384, 36, 2101), "suffix_b8_16k_n36": (8, 16384, 36, 2102),
              "suffix_b8_16k_n4": (8, 16384, 4, 2103), "suffix_b32_4k_n36": (32, 4096, 36, 2104)}
    n_req, P, N, seed = shapes[name]
    return build_workload(name, "causal", "bf16", seed, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16,
                          prefix_lens=[_s(P, shrink)] * n_req, new_lens=[N] * n_req, spare_pages=8)


def prefill_shared_config(name: str, shrink: int = 1) -> Workload:
    """Prefill batches whose requests hold the same physical pages at the head of their page tables (Section 3.3:
    questions about one video or image, one system prompt): a long shared cached part, then what each request
    cached alone, then a short new suffix.  Few rows per request, so the rows of a sharing group fill row tiles
    that single requests leave mostly empty.
      prefill_shared_video_b8_n12   8 requests about one video: 16384 shared tokens, 12 new tokens each, 28/4 heads
      prefill_shared_video_b32_n4   8 videos with 4 requests each, 16384 shared tokens, 4 new tokens each, 28/4 heads
      prefill_shared_video_b64_n4   the same 8 videos with 8 requests each
      prefill_shared_image_b32      32 requests in 4 groups of 8 sharing 2880 tokens (system prompt + image), then
                                    0..600 cached tokens of their own and 6..40 new ones, 32/8 heads"""
    if name == "prefill_shared_video_b8_n12":
        shared, H, Hkv, seed = _s(16384, shrink), 28, 4, 2201
        prefix, new, group = [shared] * 8, [12] * 8, [0] * 8
    elif name == "prefill_shared_video_b32_n4":
        shared, H, Hkv, seed = _s(16384, shrink), 28, 4, 2202
        prefix, new, group = [shared] * 32, [4] * 32, [r // 4 for r in range(32)]
    elif name == "prefill_shared_video_b64_n4":
        shared, H, Hkv, seed = _s(16384, shrink), 28, 4, 2204
        prefix, new, group = [shared] * 64, [4] * 64, [r // 8 for r in range(64)]
    elif name == "prefill_shared_image_b32":
        rng = np.random.default_rng(np.random.PCG64(2203 + 7919))
        shared, H, Hkv, seed = _s(2880, shrink), 32, 8, 2203
        prefix = [shared + _s(int(rng.integers(0, 601)), shrink) for _ in range(32)]
        new = [int(rng.integers(6, 41)) for _ in range(32)]
        group = [r // 8 for r in range(32)]
    else:
        raise KeyError(name)
    return build_workload(name, "causal", "bf16", seed, num_q_heads=H, num_kv_heads=Hkv, head_dim=128, page_size=16,
                          prefix_lens=prefix, new_lens=new, share_group=group, shared_len=[shared] * len(prefix),
                          spare_pages=8)


PREFILL_SHARED_CONFIGS = ("prefill_shared_video_b8_n12", "prefill_shared_video_b32_n4", "prefill_shared_video_b64_n4",
                          "prefill_shared_image_b32")
SUFFIX_CONFIGS = ("suffix_b1_16k_n36", "suffix_b8_16k_n36", "suffix_b8_16k_n4", "suffix_b32_4k_n36")
DECODE_CONFIGS = ("decode_video_b8", "decode_mixed_b32", "decode_b64_8k", "decode_b1_16k", "decode_b1_128k")
DECODE_SHARED_CONFIGS = ("decode_shared_video_b8", "decode_shared_video_b32", "decode_shared_image_b32")
CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def config(i: int, shrink: int = 1) -> Workload:
    return CONFIGS[i](shrink)
