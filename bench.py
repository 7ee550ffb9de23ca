#!/usr/bin/env python3
"""Benchmark of the prefix-cached paged prefill hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: KV scatter of the new tokens,
then prefix-cached causal attention (both through the C ABI, inputs already resident in HBM).  The
timed workload is the long video-prefix prefill (2 requests x [16384 cached + 2048 new tokens],
28 query / 4 KV heads, head_dim 128, page size 16, bf16), the configuration the throughput target
is stated on.  One JSON line is printed on stdout; everything else goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_MFMA_PEAK_TFLOPS = 2500.0     # published dense bf16 MFMA figure of MI355X (256 CUs x 4096 flop/clk x 2.4 GHz = 2516.6)
HBM_PEAK_GBS = 8000.0


W_PREFILL_SHARED = ("prefill_shared_video_b8_n12", "prefill_shared_video_b32_n4", "prefill_shared_video_b64_n4",
                    "prefill_shared_image_b32")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def time_workload(dw, steps, warmup, attention=None):
    """Returns (ms per step, mean attention-kernel ms, mean scatter-kernel ms) from HIP events recorded
    on the stream the kernels are launched on (torch's current stream).  `attention` replaces dw.attention."""
    import torch
    attention = attention or dw.attention
    for _ in range(warmup):
        dw.scatter()
        attention()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i][0].record()
        dw.scatter()
        ev[i][1].record()
        attention()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    scat = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
    attn = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
    dev_ms = ev[0][0].elapsed_time(ev[-1][2]) / steps
    return max(wall_ms, dev_ms), attn, scat


def cpu_baseline(wl, target_tokens):
    """The fp64 oracle, as it stands, on an evenly spaced sample of the workload's query tokens."""
    import numpy as np
    import oracle
    T = wl.total_new_tokens
    tokens = np.unique(np.linspace(0, T - 1, num=min(T, target_tokens)).astype(np.int64))
    kc, vc = oracle.kv_scatter(wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, wl.k_new, wl.v_new,
                               wl.k_cache, wl.v_cache)
    t0 = time.perf_counter()
    oracle.attention(wl.kind, wl.page_table, wl.prefix_lens, wl.new_lens, wl.cu_new_lens, wl.q, kc, vc,
                     wl.softmax_scale, tokens)
    dt = time.perf_counter() - t0
    # algorithmic flops of exactly the sampled rows
    cu = wl.cu_new_lens
    flops = 0
    for t in tokens.tolist():
        r = int(np.searchsorted(cu, t, side="right") - 1)
        flops += 4 * wl.head_dim * wl.num_q_heads * (int(wl.prefix_lens[r]) + (t - int(cu[r])) + 1)
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "%d of %d query tokens evenly spaced (all %d heads), %.1f s of fp64 oracle time, "
                      "%.3g tokens/s" % (len(tokens), T, wl.num_q_heads, dt, len(tokens) / dt),
            "new_tokens_per_s": len(tokens) / dt}


def source_digest(*names):
    """sha256 over the named kernel sources: a recorded counter figure is only shown next to measurements of the
    kernels it was taken on."""
    import hashlib
    h = hashlib.sha256()
    for n in names:
        with open(os.path.join(ROOT, "paper_2507_10069_amd", "csrc", n), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def recorded_traffic(path, key, sources):
    """HBM bytes per launch of the dominant kernel from a rocprofv3 --pmc run recorded under profiles/ (FETCH_SIZE and
    WRITE_SIZE, each scaled by what the counter reads for a plain copy of known size).  It is a figure from an
    EARLIER run of the same workload, not of this one: returned with its provenance, and dropped (None) when the
    kernel sources have changed since it was recorded.  Returns (bytes or None, provenance dict or None)."""
    try:
        with open(os.path.join(ROOT, "profiles", path)) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None, None
    rec = rec.get(key, rec) if key else rec
    if not isinstance(rec, dict) or "traffic_bytes_per_launch" not in rec:
        return None, None
    prov = {"file": "profiles/" + path, "recorded": rec.get("recorded"), "fetch_scale": rec.get("fetch_scale"),
            "write_scale": rec.get("write_scale"), "kernel_sources_sha256": rec.get("kernel_sources_sha256"),
            "measured_in_this_run": False}
    if rec.get("kernel_sources_sha256") != source_digest(*sources):
        prov["stale"] = "kernel sources differ from the recorded ones: figure withheld"
        return None, prov
    return rec["traffic_bytes_per_launch"], prov


PREFILL_SOURCES = ("attn_bf16.hip", "attn_bf16_common.h", "emm_internal.h")
DECODE_SOURCES = ("attn_bf16_decode.hip", "attn_bf16_common.h", "emm_internal.h")


def bench_timeline(workload, suffix=None, prefill_shared=None):
    """One launch of the prefill kernel built with -DEMM_TIMELINE (python -m paper_2507_10069_amd.build --timeline):
    every workgroup leaves start / end time stamps (100 MHz), its shader cycle count, its key tiles and where it ran
    (XCC_ID, HW_ID); printed as a summary per round of workgroups and per XCD."""
    import numpy as np
    import torch
    from paper_2507_10069_amd import binding as B
    from paper_2507_10069_amd import workloads as W
    from paper_2507_10069_amd import build as hip_build
    if not os.path.exists(hip_build.TIMELINE_LIB):
        sys.exit("bench.py --timeline: build the instrumented library first: python -m paper_2507_10069_amd.build --timeline")
    B.LIB_PATH = hip_build.TIMELINE_LIB
    n_rec = 16384
    wl = (W.suffix_config(suffix) if suffix is not None else
          W.prefill_shared_config(prefill_shared) if prefill_shared is not None else W.config(workload))
    dw = B.DeviceWorkload(wl)
    if dw.workspace is None or dw.workspace.numel() < n_rec * 64:
        sys.exit("bench.py --timeline: the instrumented library was not loaded")
    dw.scatter()
    dw.workspace[:n_rec * 64].zero_()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(200):                                # every launch overwrites the records: those of the last of 200
        e0.record()                                     # launches back to back are read, with the clock where a
        dw.attention()                                  # sustained run leaves it
        e1.record()
    torch.cuda.synchronize()
    rec = dw.workspace[:n_rec * 64].view(torch.int64).cpu().numpy().reshape(n_rec, 8)
    idx = np.nonzero(rec[:, 1] > 0)[0]
    r = rec[idx]
    t0 = r[:, 0].min()
    start, end = (r[:, 0] - t0) / 100.0, (r[:, 1] - t0) / 100.0            # microseconds
    dur, cyc, tiles = end - start, r[:, 2].astype(np.float64), r[:, 3].astype(np.float64)
    xcc, cu, sh, se = r[:, 5] & 15, (r[:, 4] >> 8) & 15, (r[:, 4] >> 12) & 1, (r[:, 4] >> 13) & 7
    mfma = tiles * 64.0                                 # per SIMD: two waves x 32 MFMAs per key tile
    print("workload %s: kernel %.1f us by HIP events; %d workgroups with work, first start to last end %.1f us"
          % (wl.name, e0.elapsed_time(e1) * 1e3, len(r), end.max()))
    print("XCC_ID equals workgroup index mod 8 for %d of %d workgroups" % (int((xcc == idx % 8).sum()), len(r)))
    first_end = end.min()
    for name, sel in (("first round (started before any workgroup ended)", start < first_end), ("later rounds", start >= first_end)):
        if sel.sum() == 0:
            continue
        busy = len(set(zip(xcc[sel].tolist(), se[sel].tolist(), sh[sel].tolist(), cu[sel].tolist())))
        print("%s: %d workgroups on %d compute units; start %.1f .. %.1f us, end %.1f .. %.1f us; mean duration %.1f us; "
              "%.3f us per key tile; shader clock %.0f MHz; %.1f cycles per MFMA (32 = matrix pipe always busy)"
              % (name, int(sel.sum()), busy, start[sel].min(), start[sel].max(), end[sel].min(), end[sel].max(), dur[sel].mean(),
                 (dur[sel] / tiles[sel]).mean(), (cyc[sel] / dur[sel]).mean(), (cyc[sel] / mfma[sel]).mean()))
    for x in range(8):
        sel = xcc == x
        if sel.sum():
            print("  XCD %d: %3d workgroups, first start %.1f us, last end %.1f us" % (x, int(sel.sum()), start[sel].min(), end[sel].max()))
    print("XCD finish spread: %.1f us (%.1f %% of the span)" % (max(end[xcc == x].max() for x in set(xcc.tolist())) -
          min(end[xcc == x].max() for x in set(xcc.tolist())), 100.0 * (max(end[xcc == x].max() for x in set(xcc.tolist())) -
          min(end[xcc == x].max() for x in set(xcc.tolist()))) / end.max()))


def bench_prefix_cache(with_model: bool):
    """Host-side prefix cache on a stream shaped like the paper's multimodal traffic: a few system prompts,
    a catalogue of images (576..4096 vision tokens) and videos (16384), a private question per request, four
    requests alive at a time, a pool that holds about 1 M tokens so that eviction is constant.  Times
    begin (match + allocate), commit (publish) and release through the C ABI; the reference model is timed on
    a bounded sample of the same stream."""
    import numpy as np
    from paper_2507_10069_amd import prefix_cache as PC

    rng = np.random.default_rng(31)
    ps, num_pages, max_pages = 16, 65536, 2048
    prompts = [rng.integers(0, 150000, int(n)) for n in (40, 120, 300)]
    images = [PC.emm_mm_token_ids(PC.emm_mm_content_hash(b"image-%d" % i), int(rng.integers(576, 4097))) for i in range(300)]
    videos = [PC.emm_mm_token_ids(PC.emm_mm_content_hash(b"video-%d" % i), 16384) for i in range(24)]

    def stream(n):
        out = []
        for _ in range(n):
            item = videos[rng.integers(len(videos))] if rng.random() < 0.15 else images[rng.integers(len(images))]
            out.append(np.concatenate([prompts[rng.integers(3)], item, rng.integers(0, 150000, int(rng.integers(16, 257)))]))
        return out

    def drive(begin, commit, release, reqs):
        t = {"begin": 0.0, "commit": 0.0, "release": 0.0}
        live = []
        for tok in reqs:
            t0 = time.perf_counter()
            rid = begin(tok)
            t1 = time.perf_counter()
            commit(rid, len(tok))
            t2 = time.perf_counter()
            t["begin"] += t1 - t0
            t["commit"] += t2 - t1
            live.append(rid)
            if len(live) > 4:
                t0 = time.perf_counter()
                release(live.pop(0))
                t["release"] += time.perf_counter() - t0
        for rid in live:
            release(rid)
        return t

    reqs = stream(4000)
    tokens = int(sum(len(r) for r in reqs))
    cache = PC.emm_prefix_cache_create(num_pages, ps)
    t = drive(lambda tok: PC.emm_prefix_cache_begin(cache, tok, max_pages)[2],
              lambda rid, n: PC.emm_prefix_cache_commit(cache, rid, n),
              lambda rid: PC.emm_prefix_cache_release(cache, rid), reqs)
    st = PC.emm_prefix_cache_get_stats(cache)
    PC.emm_prefix_cache_destroy(cache)
    total = sum(t.values())
    result = {
        "metric": "prefix_cache_tokens_per_s", "value": tokens / total, "unit": "tokens/s", "n_gpus": 0,
        "steps": len(reqs), "warmup": 0, "ms_per_step": 1e3 * total / len(reqs), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
        "config": {"workload": "4000 requests: system prompt + image (576..4096 tokens) or video (16384) + question, "
                               "page 16, pool 65536 pages, 5 live requests", "tokens": tokens},
        "us_per_request": {k: 1e6 * v / len(reqs) for k, v in t.items()},
        "requests_per_s": len(reqs) / total, "hit_rate": st["hit_tokens"] / st["lookup_tokens"],
        "evictions": st["evictions"],
    }
    if with_model:
        from oracle import prefix_cache_model as M
        sample = reqs[:150]
        model = M.PrefixCacheModel(num_pages, ps)
        tm = drive(lambda tok: model.begin(tok.tolist(), max_pages)[2], lambda rid, n: model.commit(rid, n),
                   lambda rid: model.release(rid), sample)
        result["cpu_baseline"] = {"value": sum(len(r) for r in sample) / sum(tm.values()), "unit": "tokens/s", "cores": 1,
                                  "kind": "oracle", "sample": "first 150 requests of the stream on the reference model"}
    log("prefix cache: %.0f requests/s, %.1f M tokens/s, hit rate %.3f, %d evictions; us per request %s"
        % (result["requests_per_s"], result["value"] / 1e6, result["hit_rate"], st["evictions"], result["us_per_request"]))
    print(json.dumps(result), flush=True)


def bench_kv_migrate(torch, B, steps, warmup):
    """Pack and unpack (with Adler-32 per page) the pages of one long video context and of a whole instance's
    worth of requests: 16 KB per page in each pool (4 KV heads, bf16, one layer), scattered page ids.  Bytes moved = read +
    write = 2 x the pages' bytes per call."""
    import numpy as np
    page_bytes, pool_pages = 4 * 16 * 128 * 2, 40000
    k = torch.randint(-2 ** 15, 2 ** 15, (pool_pages, page_bytes // 2), dtype=torch.int16, device="cuda:0")
    v = torch.randint(-2 ** 15, 2 ** 15, (pool_pages, page_bytes // 2), dtype=torch.int16, device="cuda:0")
    k2, v2 = torch.zeros_like(k), torch.zeros_like(v)
    rng = np.random.default_rng(5)
    out = {}
    for name, n in (("one_video_context_18432_tokens", 1152), ("64_contexts_of_8192_tokens", 32768)):
        src = torch.from_numpy(rng.permutation(pool_pages)[:n].astype(np.int32)).to("cuda:0")
        dst = torch.from_numpy(rng.permutation(pool_pages)[:n].astype(np.int32)).to("cuda:0")
        staging = torch.empty(n * 2 * page_bytes, dtype=torch.uint8, device="cuda:0")
        sums, sums2 = torch.zeros(n, dtype=torch.int32, device="cuda:0"), torch.zeros(n, dtype=torch.int32, device="cuda:0")
        bad = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
        for i in range(-warmup, steps):
            if i >= 0:
                ev[i][0].record()
            B.emm_kv_pages_pack(k, v, pool_pages, page_bytes, src, n, staging, sums)
            if i >= 0:
                ev[i][1].record()
            B.emm_kv_pages_unpack(staging, dst, n, k2, v2, pool_pages, page_bytes, sums2, sums, bad)
            if i >= 0:
                ev[i][2].record()
        torch.cuda.synchronize()
        assert int(bad.item()) == 0 and torch.equal(sums, sums2)
        assert torch.equal(k2[dst.long()], k[src.long()]) and torch.equal(v2[dst.long()], v[src.long()])
        pack_ms = sum(e[0].elapsed_time(e[1]) for e in ev) / steps
        unpack_ms = sum(e[1].elapsed_time(e[2]) for e in ev) / steps
        moved = 2 * n * 2 * page_bytes
        out[name] = {"pages": n, "bytes": n * 2 * page_bytes, "pack_ms": pack_ms, "unpack_ms": unpack_ms,
                     "pack_gbs": moved / (pack_ms * 1e-3) / 1e9, "unpack_gbs": moved / (unpack_ms * 1e-3) / 1e9}
        log("kv migrate %s: pack %.4f ms (%.0f GB/s read+write), unpack %.4f ms (%.0f GB/s)"
            % (name, pack_ms, out[name]["pack_gbs"], unpack_ms, out[name]["unpack_gbs"]))
    # for scale: a plain device-to-device copy of 1 GiB by the runtime
    a1 = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    a2 = torch.empty_like(a1)
    for _ in range(3):
        a2.copy_(a1)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        a2.copy_(a1)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * (1 << 30) / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9
    log("plain copy of 1 GiB: %.0f GB/s read+write" % copy_gbs)
    big = out["64_contexts_of_8192_tokens"]
    gbs = 2 * 2 * big["bytes"] / ((big["pack_ms"] + big["unpack_ms"]) * 1e-3) / 1e9
    print(json.dumps({
        "metric": "kv_page_migration_gbs", "value": gbs, "unit": "GB/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": big["pack_ms"] + big["unpack_ms"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u8", "data": "synthetic",
        "config": {"workload": "pack + unpack of 32768 pages of 2 x 16 KB (64 contexts of 8192 tokens, 4 KV heads, bf16), "
                               "Adler-32 per page on both sides", "parallelism": "single-gpu"},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                     "traffic": None, "kernel": "kv_pages_kernel<false> + kv_pages_kernel<true>"},
        "cases": out, "plain_copy_gbs": copy_gbs,
    }), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=3, help="named workload 1..5 (default 3, the target)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-tokens", type=int, default=2048)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy 5 times (a kernel of known HBM traffic, used to "
                         "scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--others", action="store_true", help="also time the other named workloads (stderr + JSON)")
    ap.add_argument("--decode", default=None, metavar="NAME",
                    help="time one decode-step workload instead (one query token per request; HBM-bound): "
                         "decode_video_b8, decode_mixed_b32 or decode_b64_8k")
    ap.add_argument("--suffix", default=None, metavar="NAME",
                    help="time one short-suffix prefill workload instead (the batch a large cache hit leaves): "
                         "suffix_b1_16k_n36, suffix_b8_16k_n36, suffix_b8_16k_n4 or suffix_b32_4k_n36")
    ap.add_argument("--prefill-shared", default=None, metavar="NAME",
                    help="time a prefill batch with shared prefix pages (%s): emm_prefill_attn against "
                         "emm_prefill_attn_shared" % ", ".join(W_PREFILL_SHARED))
    ap.add_argument("--kv-migrate", action="store_true",
                    help="time the KV page migration primitive (pack and unpack with checksums) instead")
    ap.add_argument("--timeline", action="store_true",
                    help="per-workgroup timeline of one plain prefill launch on the batch that --workload, --suffix or "
                         "--prefill-shared names (needs the build made by python -m paper_2507_10069_amd.build --timeline)")
    ap.add_argument("--prefix-cache", action="store_true",
                    help="time the host-side prefix cache (no GPU work) on a synthetic request stream")
    args = ap.parse_args()
    if args.prefix_cache:
        return bench_prefix_cache(not args.no_cpu_baseline)
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path needs no exchange between requests); "
                 "run with --gpus 1")

    import torch
    from paper_2507_10069_amd import binding as B
    from paper_2507_10069_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    torch.cuda.set_device(0)
    if args.timeline:
        return bench_timeline(args.workload, args.suffix, args.prefill_shared)
    B.load()                                            # fails loudly if libemm.so has not been built

    if args.copy_calibration:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    if args.kv_migrate:
        return bench_kv_migrate(torch, B, args.steps, args.warmup)
    if args.suffix is not None:
        wl = W.suffix_config(args.suffix)
        dw = B.DeviceWorkload(wl)
        ms, attn_ms, scat_ms = time_workload(dw, args.steps, args.warmup)
        tflops = wl.attention_flops() / (attn_ms * 1e-3) / 1e12
        gbs = wl.kv_read_bytes() / (attn_ms * 1e-3) / 1e9
        log("workload %s: %.4f ms/step (attention %.4f ms, scatter %.4f ms), %.1f TFLOP/s, %.0f GB/s of K/V read"
            % (wl.name, ms, attn_ms, scat_ms, tflops, gbs))
        # few rows over long contexts: neither roof is near; the one that is closer is reported
        mfma_frac, hbm_frac = tflops / BF16_MFMA_PEAK_TFLOPS, gbs / HBM_PEAK_GBS
        roof = ({"bound": "mfma", "achieved": tflops, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": mfma_frac}
                if mfma_frac >= hbm_frac else
                {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac})
        roof.update({"traffic": None, "kernel": "attn_bf16_d128_kernel + attn_bf16_merge_kernel"})
        print(json.dumps({
            "metric": "prefill_attention_tflops", "value": wl.attention_flops() / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
            "config": {"workload": wl.name, "requests": wl.num_reqs, "total_new_tokens": wl.total_new_tokens,
                       "algorithmic_flops_per_step": wl.attention_flops(), "kv_read_bytes_per_step": wl.kv_read_bytes(),
                       "parallelism": "single-gpu"},
            "new_tokens_per_s": wl.total_new_tokens / (ms * 1e-3), "attention_ms": attn_ms, "scatter_ms": scat_ms,
            "roofline": roof,
        }), flush=True)
        return
    if args.prefill_shared is not None:
        wl = W.prefill_shared_config(args.prefill_shared)
        dw = B.DeviceWorkload(wl)
        ms, attn_ms, scat_ms = time_workload(dw, args.steps, args.warmup)
        keeps = dw.plan_prefill_shared()["num_groups"] > 0          # what the planner does with its default threshold
        plan = dw.plan_prefill_shared(min_saved_key_tiles=0)        # timed with the groups in any case
        ms_s, attn_s, scat_s = time_workload(dw, args.steps, args.warmup, dw.attention_prefill_shared)
        flops = wl.attention_flops()
        log("workload %s: plain %.4f ms/step (attention %.4f ms); %d sharing groups, row tiles %d -> %d, key tiles %d -> %d: "
            "%.4f ms/step (attention %.4f ms, %.2fx); by default the planner %s the groups"
            % (wl.name, ms, attn_ms, plan["num_groups"], plan["rows_tiles_plain"], plan["rows_tiles_shared"],
               plan["key_tiles_plain"], plan["key_tiles_shared"], ms_s, attn_s, attn_ms / attn_s, "keeps" if keeps else "gives up"))
        tflops = flops / (attn_s * 1e-3) / 1e12
        distinct_gbs = wl.kv_distinct_read_bytes() / (attn_s * 1e-3) / 1e9
        mfma_frac, hbm_frac = tflops / BF16_MFMA_PEAK_TFLOPS, distinct_gbs / HBM_PEAK_GBS
        roof = ({"bound": "mfma", "achieved": tflops, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": mfma_frac}
                if mfma_frac >= hbm_frac else
                {"bound": "hbm", "achieved": distinct_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_frac})
        roof.update({"traffic": None, "kernel": "attn_bf16_d128_kernel (two passes) + attn_bf16_merge_kernel + attn_merge_parts_kernel"})
        print(json.dumps({
            "metric": "prefill_attention_tflops", "value": flops / (ms_s * 1e-3) / 1e12, "unit": "TFLOP/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_s, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
            "config": {"workload": wl.name, "requests": wl.num_reqs, "total_new_tokens": wl.total_new_tokens,
                       "algorithmic_flops_per_step": flops, "kv_distinct_bytes_per_step": wl.kv_distinct_read_bytes(),
                       "parallelism": "single-gpu"},
            "new_tokens_per_s": wl.total_new_tokens / (ms_s * 1e-3), "attention_ms": attn_s, "scatter_ms": scat_s,
            "sharing_groups": plan["num_groups"], "row_tiles_plain": plan["rows_tiles_plain"],
            "row_tiles_shared": plan["rows_tiles_shared"], "key_tiles_plain": plan["key_tiles_plain"],
            "key_tiles_shared": plan["key_tiles_shared"], "planner_default_keeps_groups": keeps,
            "plain_path": {"ms_per_step": ms, "attention_ms": attn_ms},
            "speedup_over_plain_attention": attn_ms / attn_s, "roofline": roof,
        }), flush=True)
        return
    if args.decode is not None:
        wl = W.decode_config(args.decode)
        dw = B.DeviceWorkload(wl)
        ms, attn_ms, scat_ms = time_workload(dw, args.steps, args.warmup)
        gbs = wl.kv_read_bytes() / (attn_ms * 1e-3) / 1e9
        # pages that several requests share have to come from HBM once only: the roofline figure counts them once
        # (for a batch without shared pages the two are the same number)
        distinct = wl.kv_distinct_read_bytes()
        distinct_gbs = distinct / (attn_ms * 1e-3) / 1e9
        log("workload %s: %.4f ms/step (attention %.4f ms, scatter %.4f ms), %.0f GB/s of K/V consumed, %.0f GB/s of distinct K/V"
            % (wl.name, ms, attn_ms, scat_ms, gbs, distinct_gbs))
        # the same batch through emm_decode_attn_shared with what the host knows of it: shared pages are
        # read once per unit, and pieces are sized for the real amount of work, not for the longest context
        plan = dw.plan_shared()
        ms_s, attn_s, scat_s = time_workload(dw, args.steps, args.warmup, dw.attention_shared)
        elt = 2 * wl.num_kv_heads * wl.head_dim * wl.elt_bytes          # K and V bytes per context token
        saved = int(sum(int(l) * (int(n) - 1) for l, n in zip(plan["unit_shared_len"], plan["unit_num_reqs"]))) * elt
        read = wl.kv_read_bytes() - saved
        shared = {"num_units": plan["num_units"], "planned_tiles": plan["planned_tiles"], "ms_per_step": ms_s, "attention_ms": attn_s,
                  "kv_bytes_read_per_step": read, "read_gbs": read / (attn_s * 1e-3) / 1e9,
                  "frac_hbm_peak": read / (attn_s * 1e-3) / 1e9 / HBM_PEAK_GBS,
                  "speedup_over_unshared_attention": attn_ms / attn_s}
        log("  planned (%d shared-prefix units, %d tiles): attention %.4f ms (%.2fx), %.0f GB/s of the %.0f MB it reads"
            % (plan["num_units"], plan["planned_tiles"], attn_s, attn_ms / attn_s, shared["read_gbs"], read / 1e6))
        # the whole step (scatter + attention) as ONE call, emm_decode_step, without and with the units
        # (both timed the same way here: K steps back to back between two events)
        def two_calls(attention):
            dw.scatter()
            attention()
        fused = {}
        for key, fn in (("plain", lambda: dw.decode_step(False)), ("planned", lambda: dw.decode_step(True)),
                        ("plain_two_calls", lambda: two_calls(dw.attention)),
                        ("planned_two_calls", lambda: two_calls(dw.attention_shared))):
            for _ in range(args.warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0 = time.perf_counter()
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            fused[key] = max(e0.elapsed_time(e1), (time.perf_counter() - t0) * 1e3) / args.steps
        log("  step as one call (emm_decode_step): %.4f ms plain (scatter + attention: %.4f), %.4f ms planned (%.4f)"
            % (fused["plain"], fused["plain_two_calls"], fused["planned"], fused["planned_two_calls"]))
        # the planned step captured in a HIP graph and replayed: what a serving loop that captures its layers sees
        side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            dw.decode_step(True)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                dw.decode_step(True)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        fused["planned_graph_replay"] = e0.elapsed_time(e1) / args.steps
        log("  the planned step replayed from a HIP graph: %.4f ms" % fused["planned_graph_replay"])
        decode_traffic, decode_traffic_source = recorded_traffic("attn_bf16_decode_hbm_traffic.json", wl.name, DECODE_SOURCES)
        print(json.dumps({
            "metric": "decode_attention_kv_read_gbs", "value": distinct / (ms * 1e-3) / 1e9, "unit": "GB/s",
            "kv_consumed_gbs": wl.kv_read_bytes() / (ms * 1e-3) / 1e9,     # shared pages counted once per request
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
            "config": {"workload": wl.name, "requests": wl.num_reqs, "kv_read_bytes_per_step": wl.kv_read_bytes(),
                       "parallelism": "single-gpu"},
            "new_tokens_per_s": wl.total_new_tokens / (ms * 1e-3), "attention_ms": attn_ms, "scatter_ms": scat_ms,
            "kv_distinct_bytes_per_step": distinct,
            "roofline": {"bound": "hbm", "achieved": distinct_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": distinct_gbs / HBM_PEAK_GBS, "traffic": decode_traffic, "traffic_source": decode_traffic_source,
                         "kernel": "attn_bf16_decode_kernel + attn_bf16_decode_merge_kernel"},
            "shared_prefix": shared, "fused_step_ms": fused,
        }), flush=True)
        return

    wl = W.config(args.workload)
    dw = B.DeviceWorkload(wl)
    ms, attn_ms, scat_ms = time_workload(dw, args.steps, args.warmup)
    flops = wl.attention_flops()
    T = wl.total_new_tokens
    tflops = flops / (ms * 1e-3) / 1e12
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12
    log("workload %s: %.4f ms/step (attention %.4f ms, scatter %.4f ms), %.1f TFLOP/s whole step, "
        "%.1f TFLOP/s attention kernel" % (wl.name, ms, attn_ms, scat_ms, tflops, attn_tflops))

    traffic, traffic_source = recorded_traffic("attn_bf16_cfg%d_hbm_traffic.json" % args.workload, None, PREFILL_SOURCES)
    result = {
        "metric": "prefill_attention_tflops", "value": tflops, "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d requests, %d cached + %d new tokens each, %d/%d heads, head_dim %d, "
                               "page %d, causal, KV scatter + attention per step"
                               % (wl.name, wl.num_reqs, int(wl.prefix_lens[0]), int(wl.new_lens[0]),
                                  wl.num_q_heads, wl.num_kv_heads, wl.head_dim, wl.page_size)
                   if args.workload == 3 else wl.name,
                   "total_new_tokens": T, "algorithmic_flops_per_step": flops, "parallelism": "single-gpu"},
        "new_tokens_per_s": T / (ms * 1e-3),
        "pct_bf16_mfma_peak": 100.0 * tflops / BF16_MFMA_PEAK_TFLOPS,
        "attention_ms": attn_ms, "scatter_ms": scat_ms,
        "scatter_gbs": (wl.scatter_bytes() / (scat_ms * 1e-3) / 1e9) if scat_ms > 0 else None,
        "roofline": {"bound": "mfma", "achieved": attn_tflops, "peak": BF16_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": attn_tflops / BF16_MFMA_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "attn_bf16_d128_kernel"},
    }
    if args.others:
        others = {}
        for i in (1, 2, 4, 5):
            w = W.config(i)
            d = B.DeviceWorkload(w)
            m, am, sm = time_workload(d, 30, 5)
            others[w.name] = {"ms_per_step": m, "attention_ms": am, "scatter_ms": sm,
                              "tflops": w.attention_flops() / (m * 1e-3) / 1e12,
                              "attention_tflops": w.attention_flops() / (am * 1e-3) / 1e12,
                              "new_tokens_per_s": w.total_new_tokens / (m * 1e-3)}
            if w.dtype == "bf16":
                others[w.name]["frac_bf16_mfma_peak"] = others[w.name]["attention_tflops"] / BF16_MFMA_PEAK_TFLOPS
            log("workload %s: %s" % (w.name, others[w.name]))
            del d
        for name in W.SUFFIX_CONFIGS:                    # short suffixes after a large cache hit
            w = W.suffix_config(name)
            d = B.DeviceWorkload(w)
            m, am, sm = time_workload(d, 30, 5)
            others[name] = {"ms_per_step": m, "attention_ms": am, "scatter_ms": sm,
                            "tflops": w.attention_flops() / (am * 1e-3) / 1e12,
                            "kv_read_gbs": w.kv_read_bytes() / (am * 1e-3) / 1e9,
                            "new_tokens_per_s": w.total_new_tokens / (m * 1e-3)}
            log("workload %s: %s" % (name, others[name]))
            del d
        for name in W.PREFILL_SHARED_CONFIGS:            # short suffixes over shared cached pages: plain call and the grouped one
            w = W.prefill_shared_config(name)
            d = B.DeviceWorkload(w)
            m, am, sm = time_workload(d, 30, 5)
            plan = d.plan_prefill_shared(min_saved_key_tiles=0)
            ms_, ams, _ = time_workload(d, 30, 5, d.attention_prefill_shared)
            others[name] = {"ms_per_step": m, "attention_ms": am, "scatter_ms": sm, "shared_attention_ms": ams,
                            "sharing_groups": plan["num_groups"], "speedup_over_plain_attention": am / ams,
                            "new_tokens_per_s": w.total_new_tokens / (min(m, ms_) * 1e-3)}
            log("workload %s: %s" % (name, others[name]))
            del d
        for name in W.DECODE_CONFIGS:
            w = W.decode_config(name)
            d = B.DeviceWorkload(w)
            m, am, sm = time_workload(d, 30, 5)
            others[name] = {"ms_per_step": m, "attention_ms": am, "scatter_ms": sm,
                            "kv_read_gbs": w.kv_read_bytes() / (am * 1e-3) / 1e9,
                            "frac_hbm_peak": w.kv_read_bytes() / (am * 1e-3) / 1e9 / HBM_PEAK_GBS,
                            "new_tokens_per_s": w.total_new_tokens / (m * 1e-3)}
            log("workload %s: %s" % (name, others[name]))
            del d
        result["other_workloads"] = others
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, args.cpu_sample_tokens)
        log("cpu baseline:", result["cpu_baseline"])
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
