"""The C++ prefix cache (csrc/prefix_cache.cpp, through the C ABI) against the reference model
(oracle/prefix_cache_model.py), call by call and id by id: page-table rows, prefix lengths, statuses and
statistics must be identical on seeded random traffic that includes evictions, duplicates, appends,
overlapping lifetimes and failing calls.  Host code only, so this runs without a GPU."""
from __future__ import annotations

import hashlib
import random

import numpy as np
import pytest

from oracle import prefix_cache_model as M
from paper_2507_10069_amd import binding as B
from paper_2507_10069_amd import prefix_cache as PC

STATUS = {M.INVALID_ARG: B.EMM_ERR_INVALID_ARG, M.NO_SPACE: PC.EMM_ERR_NO_SPACE, M.NOT_FOUND: PC.EMM_ERR_NOT_FOUND}


def test_content_hash_is_sha256():
    rng = random.Random(5)
    for n in list(range(0, 130)) + [255, 256, 257, 1000, 4096, 65537]:
        data = bytes(rng.randrange(256) for _ in range(n))
        assert PC.emm_mm_content_hash(data) == hashlib.sha256(data).digest() == M.mm_content_hash(data), n
    assert PC.emm_mm_content_hash(b"abc").hex() == "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"
    big = bytes(range(256)) * 4096                               # 1 MiB, e.g. an image file
    assert PC.emm_mm_content_hash(big) == hashlib.sha256(big).digest()


def test_placeholder_ids_match_model():
    for seed in range(5):
        digest = hashlib.sha256(b"item%d" % seed).digest()
        ids = PC.emm_mm_token_ids(digest, 700)
        assert ids.tolist() == M.mm_token_ids(digest, 700)
    assert PC.emm_mm_token_ids(bytes(32), 2).tolist() == [-1, -1 - 0x4F1BBCDCBFA53E0A]
    assert PC.emm_mm_token_ids(bytes(32), 0).size == 0
    with pytest.raises(B.EmmError):
        PC.emm_mm_token_ids(bytes(32), -1)


def _sequences(rng, ps, n_seq):
    prompts = [[rng.randrange(0, 50000) for _ in range(rng.randrange(1, 5 * ps))] for _ in range(3)]
    images = [M.mm_token_ids(M.mm_content_hash(b"img%d" % i), rng.randrange(ps, 8 * ps)) for i in range(4)]
    out = []
    for _ in range(n_seq):
        s = list(rng.choice(prompts))
        if rng.random() < 0.7:
            s += rng.choice(images)
        if rng.random() < 0.3:
            s += rng.choice(images)
        s += [rng.randrange(0, 50000) for _ in range(rng.randrange(1, 3 * ps))]
        out.append(s)
    return out


class _Both:
    """Applies every call to the library and to the model and compares what comes back."""

    def __init__(self, num_pages, ps):
        self.model = M.PrefixCacheModel(num_pages, ps)
        self.cache = PC.emm_prefix_cache_create(num_pages, ps)
        self.ids = {}                       # library request id -> model request id

    def close(self):
        PC.emm_prefix_cache_destroy(self.cache)

    def _both(self, lib_call, model_call):
        lib_err = model_err = None
        try:
            lib_out = lib_call()
        except B.EmmError as e:
            lib_err, lib_out = e.status, None
        try:
            model_out = model_call()
        except M.CacheError as e:
            model_err, model_out = STATUS[e.status], None
        assert lib_err == model_err, (lib_err, model_err)
        assert PC.emm_prefix_cache_get_stats(self.cache) == self.model.stats()
        return lib_out, model_out, lib_err

    def begin(self, tokens, max_pages):
        lo, mo, err = self._both(lambda: PC.emm_prefix_cache_begin(self.cache, tokens, max_pages),
                                 lambda: self.model.begin(tokens, max_pages))
        if err is not None:
            return None
        assert lo[0].tolist() == mo[0] and lo[1] == mo[1]
        self.ids[lo[2]] = mo[2]
        return lo[2]

    def append(self, rid, tokens, max_pages):
        lo, mo, err = self._both(lambda: PC.emm_prefix_cache_append(self.cache, rid, tokens, max_pages),
                                 lambda: self.model.append(self.ids.get(rid, -1), tokens, max_pages))
        if err is None:
            assert lo.tolist() == mo
        return err is None

    def commit(self, rid, n):
        return self._both(lambda: PC.emm_prefix_cache_commit(self.cache, rid, n),
                          lambda: self.model.commit(self.ids.get(rid, -1), n))[2] is None

    def release(self, rid):
        ok = self._both(lambda: PC.emm_prefix_cache_release(self.cache, rid),
                        lambda: self.model.release(self.ids.get(rid, -1)))[2] is None
        if ok:
            del self.ids[rid]
        return ok


@pytest.mark.parametrize("seed", range(12))
def test_random_traffic_matches_model(seed):
    rng = random.Random(1000 + seed)
    ps = rng.choice([1, 2, 4, 16, 16])
    both = _Both(rng.randrange(12, 80), ps)
    seqs = _sequences(rng, ps, 10)
    live = {}                               # rid -> tokens
    n_err = 0
    for step in range(1500):
        op = rng.random()
        if op < 0.35 or not live:
            s = list(rng.choice(seqs))
            if rng.random() < 0.5:
                s = s[:rng.randrange(1, len(s) + 1)]
            max_pages = rng.choice([64, 64, 64, -(-len(s) // ps), -(-len(s) // ps) - 1])
            rid = both.begin(s, max_pages)
            if rid is None:
                n_err += 1
            else:
                live[rid] = s
        elif op < 0.55:
            rid = rng.choice(list(live))
            extra = [rng.randrange(0, 5) for _ in range(rng.randrange(0, 2 * ps + 1))]
            if both.append(rid, extra, 64):
                live[rid] = live[rid] + extra
            else:
                n_err += 1
        elif op < 0.80:
            rid = rng.choice(list(live))
            n = rng.choice([len(live[rid]), rng.randrange(0, len(live[rid]) + 2)])
            n_err += not both.commit(rid, n)
        elif op < 0.97:
            rid = rng.choice(list(live))
            if rng.random() < 0.7:
                both.commit(rid, len(live[rid]))
            assert both.release(rid)
            del live[rid]
        else:
            n_err += not both.release(rng.randrange(10 ** 6, 10 ** 7))     # unknown id
            n_err += not both.commit(rng.randrange(10 ** 6, 10 ** 7), 0)
    assert n_err > 0                        # the failing paths were exercised
    assert both.model.stats()["evictions"] > 0 or both.model.num_pages > 60
    for rid in list(live):
        assert both.release(rid)
    st = PC.emm_prefix_cache_get_stats(both.cache)
    assert st["live_requests"] == 0 and st["private_pages"] == 0
    assert st["free_pages"] + st["cached_pages"] == st["num_pages"]
    both.close()


def test_long_sequences_and_heavy_eviction_match_model():
    """Workload-sized: 18k-token video contexts and 1-4k image contexts at page size 16 through a pool that
    holds only a few of them."""
    rng = random.Random(77)
    ps = 16
    both = _Both(4000, ps)
    videos = [M.mm_token_ids(M.mm_content_hash(b"video%d" % i), 16384) for i in range(3)]
    images = [M.mm_token_ids(M.mm_content_hash(b"image%d" % i), rng.randrange(576, 4096)) for i in range(6)]
    system = [rng.randrange(0, 50000) for _ in range(40)]
    live = []
    for step in range(60):
        s = system + (rng.choice(videos) if rng.random() < 0.3 else rng.choice(images))
        s = s + [rng.randrange(0, 50000) for _ in range(rng.randrange(8, 300))]
        rid = both.begin(s, 1200)
        if rid is not None:
            both.commit(rid, len(s))
            live.append(rid)
        while len(live) > 2 or (rid is None and live):
            both.release(live.pop(0))
            rid = 0
    assert both.model.stats()["evictions"] > 0 and both.model.stats()["hit_tokens"] > 0
    both.close()


def test_null_and_argument_errors():
    lib = B.load()
    PC._lib()
    assert lib.emm_prefix_cache_create(4, 4, None) == B.EMM_ERR_NULL
    with pytest.raises(B.EmmError) as e:
        PC.emm_prefix_cache_create(0, 16)
    assert e.value.status == B.EMM_ERR_INVALID_ARG
    with pytest.raises(B.EmmError):
        PC.emm_prefix_cache_create(16, 0)
    c = PC.emm_prefix_cache_create(4, 4)
    assert lib.emm_prefix_cache_begin(c, None, 1, 1, None, None, None) == B.EMM_ERR_NULL
    assert lib.emm_prefix_cache_get_stats(c, None) == B.EMM_ERR_NULL
    assert lib.emm_prefix_cache_release(None, 1) == B.EMM_ERR_NULL
    with pytest.raises(B.EmmError) as e:
        PC.emm_prefix_cache_begin(c, np.zeros(0, dtype=np.int64), 4)
    assert e.value.status == B.EMM_ERR_INVALID_ARG
    assert "page" in B.emm_status_string(PC.EMM_ERR_NO_SPACE) and "request" in B.emm_status_string(PC.EMM_ERR_NOT_FOUND)
    PC.emm_prefix_cache_destroy(c)
    PC.emm_prefix_cache_destroy(None)
