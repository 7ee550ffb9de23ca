"""Pins for the prefix-cache reference model (oracle/prefix_cache_model.py): each compares it with
something that shares none of its code -- published SHA-256 vectors, a hand-worked id, a
content-addressed dictionary (what page sharing means when nothing is evicted), a textbook LRU, and
conservation invariants under random traffic."""
from __future__ import annotations

import random
from collections import OrderedDict

import pytest

from oracle import prefix_cache_model as M


# ---- pool 1: content hash and placeholder ids (Section 3.3; Appendix B.7: cryptographic hash)

def test_sha256_published_vectors():
    # FIPS 180-4 example messages
    assert M.mm_content_hash(b"abc").hex() == \
        "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"
    assert M.mm_content_hash(b"").hex() == \
        "e3b0c44298fc1c149afbf4c8996fb92427ae41e4649b934ca495991b7852b855"
    assert M.mm_content_hash(b"abcdbcdecdefdefgefghfghighijhijkijkljklmklmnlmnomnopnopq").hex() == \
        "248d6a61d20638b8e5c026930c3e6039a33ce45964ff2167f6ecedd419db06c1"


def test_placeholder_ids_worked_example_and_properties():
    # all-zero digest: w0 = w1 = 0, so id_j = -1 - ((j * 0x9E3779B97F4A7C15 mod 2^64) >> 1)
    ids = M.mm_token_ids(bytes(32), 3)
    assert ids[0] == -1
    assert ids[1] == -1 - 0x4F1BBCDCBFA53E0A
    assert ids[2] == -1 - (((2 * 0x9E3779B97F4A7C15) % (1 << 64)) >> 1)
    # w1 only: flips bits of every id the same way
    d = bytes(8) + (0xFF).to_bytes(8, "big") + bytes(16)
    assert M.mm_token_ids(d, 1)[0] == -1 - (0xFF >> 1)
    a = M.mm_token_ids(M.mm_content_hash(b"image-a"), 576)
    b = M.mm_token_ids(M.mm_content_hash(b"image-b"), 576)
    assert all(x < 0 for x in a + b) and all(x >= -(1 << 63) for x in a + b)
    assert len(set(a)) == 576 and not set(a) & set(b)
    assert a == M.mm_token_ids(M.mm_content_hash(b"image-a"), 576)
    assert a[:100] == M.mm_token_ids(M.mm_content_hash(b"image-a"), 100)


# ---- pool 2 without eviction: pages are content addressed

def _make_sequences(rng, n_seq, ps):
    """Sequences that share prefixes the way the paper's workloads do: a few system prompts, a few images
    (runs of placeholder ids), then a private tail; lengths not multiples of the page size."""
    prompts = [[rng.randrange(0, 50000) for _ in range(rng.randrange(1, 4 * ps))] for _ in range(3)]
    images = [M.mm_token_ids(M.mm_content_hash(b"img%d" % i), rng.randrange(ps, 6 * ps)) for i in range(4)]
    seqs = []
    for _ in range(n_seq):
        s = list(rng.choice(prompts))
        if rng.random() < 0.7:
            s += rng.choice(images)
        s += [rng.randrange(0, 50000) for _ in range(rng.randrange(1, 3 * ps))]
        seqs.append(s)
    return seqs


@pytest.mark.parametrize("ps", [1, 4, 16])
def test_hits_equal_content_addressed_pages_when_nothing_is_evicted(ps):
    rng = random.Random(100 + ps)
    seqs = _make_sequences(rng, 60, ps)
    cache = M.PrefixCacheModel(num_pages=100000, page_size=ps)
    published = {}                      # tuple(tokens[0 : (p+1) ps]) -> physical page of the first publisher
    for s in seqs:
        n = len(s)
        row, prefix_len, rid = cache.begin(s, max_pages=-(-n // ps) + 2)
        # expected: longest run of leading full pages whose content is published, last token's page excluded
        exp = 0
        while exp < (n - 1) // ps and tuple(s[:(exp + 1) * ps]) in published:
            exp += 1
        assert prefix_len == exp * ps
        assert row[:exp] == [published[tuple(s[:(p + 1) * ps])] for p in range(exp)]
        n_pages = -(-n // ps)
        assert all(pg >= 0 for pg in row[:n_pages]) and row[n_pages:] == [-1, -1]
        assert len(set(row[:n_pages])) == n_pages
        fresh = row[exp:n_pages]
        assert not set(fresh) & set(published.values())          # new tokens never land in shared pages
        cache.commit(rid, n)
        for p in range(n // ps):
            published.setdefault(tuple(s[:(p + 1) * ps]), row[p])
        cache.release(rid)
    st = cache.stats()
    assert st["cached_pages"] == len(published) and st["evictions"] == 0
    assert st["free_pages"] + st["cached_pages"] == st["num_pages"] and st["private_pages"] == 0


def test_whole_sequence_cached_still_leaves_a_page_to_prefill():
    cache = M.PrefixCacheModel(64, 4)
    s = list(range(16))                                          # exactly 4 pages
    row, pl, rid = cache.begin(s, 4)
    assert pl == 0
    cache.commit(rid, 16)
    cache.release(rid)
    row2, pl2, rid2 = cache.begin(s, 4)
    assert pl2 == 12 and row2[:3] == row[:3] and row2[3] != row[3]
    cache.commit(rid2, 16)                                       # its last page is a duplicate of a cached one
    assert cache.stats()["private_pages"] == 1
    cache.release(rid2)
    assert cache.stats()["cached_pages"] == 4 and cache.stats()["free_pages"] == 60


# ---- eviction: reduces to a textbook LRU when every sequence is one page plus one token

@pytest.mark.parametrize("capacity,n_keys", [(5, 8), (9, 12), (3, 3)])
def test_single_page_sequences_behave_like_a_textbook_lru(capacity, n_keys):
    ps = 4
    rng = random.Random(capacity * 31 + n_keys)
    cache = M.PrefixCacheModel(num_pages=capacity, page_size=ps)
    lru = OrderedDict()                 # holds at most capacity-1 keys: one page is always in use as the tail
    for step in range(400):
        k = rng.randrange(n_keys)
        seq = [1000 * k + i for i in range(ps)] + [7]
        row, prefix_len, rid = cache.begin(seq, 2)
        hit = k in lru
        assert prefix_len == (ps if hit else 0), step
        if hit:
            lru.move_to_end(k)
        else:
            if len(lru) == capacity - 1:
                lru.popitem(last=False)
            lru[k] = True
        cache.commit(rid, ps + 1)
        cache.release(rid)
        assert cache.stats()["cached_pages"] == len(lru)


# ---- user counts (Appendix A): a node in use is never evicted; a failed call changes nothing

def test_pages_of_live_requests_survive_pressure_and_no_space_is_clean():
    ps = 4
    cache = M.PrefixCacheModel(num_pages=12, page_size=ps)
    a = list(range(100, 100 + 4 * ps + 1))                       # 4 full pages + 1 token: 5 pages
    row_a, _, rid_a = cache.begin(a, 8)
    cache.commit(rid_a, len(a))
    for i in range(20):                                          # traffic that needs eviction: 7 pages left
        s = [5000 + 100 * i + j for j in range(2 * ps + 1)]
        _, pl, rid = cache.begin(s, 8)
        assert pl == 0
        cache.commit(rid, len(s))
        cache.release(rid)
    row_b, pl_b, rid_b = cache.begin(a[:4 * ps] + [1, 2, 3], 8)  # A's four pages are still there
    assert pl_b == 4 * ps and row_b[:4] == row_a[:4]
    before = cache.stats()
    with pytest.raises(M.CacheError) as e:                       # 12 pages: A holds 5, B 1 more; 7 needed
        cache.begin([9000 + j for j in range(7 * ps)], 8)
    assert e.value.status == M.NO_SPACE and cache.stats() == before
    with pytest.raises(M.CacheError) as e:
        cache.begin([1, 2, 3], 0)
    assert e.value.status == M.INVALID_ARG
    with pytest.raises(M.CacheError) as e:
        cache.release(12345)
    assert e.value.status == M.NOT_FOUND
    cache.release(rid_a)
    cache.release(rid_b)
    row_c, pl_c, _ = cache.begin([9000 + j for j in range(7 * ps)], 8)   # now the old nodes can go
    assert pl_c == 0 and len(set(row_c[:7])) == 7


def test_children_are_evicted_before_parents_and_least_recent_branch_first():
    ps = 2
    cache = M.PrefixCacheModel(num_pages=8, page_size=ps)

    def run(seq):
        row, pl, rid = cache.begin(seq, 8)
        cache.commit(rid, len(seq))
        cache.release(rid)
        return row, pl

    run([1, 1, 2, 2, 3, 3, 0])          # chain of 3 pages (+ tail page, freed)
    run([1, 1, 4, 4, 0])                # branch below the first page: shares it, adds 1
    run([1, 1, 2, 2, 0])                # touches the first two nodes of the chain again
    assert cache.stats()["cached_pages"] == 4 and cache.stats()["free_pages"] == 4
    # 6 pages wanted: 4 free + 2 evictions.  Evictable leaves: [3,3] (stamped by request 1) and [4,4]
    # (stamped by request 2); [2,2] becomes a leaf only after [3,3] is gone and was stamped later than both.
    run([9, 9, 8, 8, 7, 7, 6, 6, 5, 5, 0])
    _, pl = run([1, 1, 2, 2, 3, 3, 0])
    assert pl == 4                      # [1,1] and [2,2] survived, [3,3] did not
    assert cache.stats()["evictions"] >= 2


def test_a_chain_released_at_once_loses_its_deepest_page_first():
    ps = 2
    cache = M.PrefixCacheModel(num_pages=5, page_size=ps)
    seq = [1, 1, 2, 2, 3, 3, 0]
    row, _, rid = cache.begin(seq, 4)
    cache.commit(rid, len(seq))
    cache.release(rid)                  # three nodes, same stamp; 2 pages free
    _, _, rid2 = cache.begin([5, 5, 6, 6, 0], 4)     # 3 pages: one eviction
    cache.release(rid2)
    assert cache.stats()["evictions"] == 1
    row3, pl3, _ = cache.begin(seq, 4)
    assert pl3 == 2 * ps and row3[:2] == row[:2]     # the parents are intact


def test_recently_used_means_recently_released():
    ps = 4
    cache = M.PrefixCacheModel(num_pages=6, page_size=ps)
    a = [10, 11, 12, 13, 0]
    b = [20, 21, 22, 23, 0]
    _, _, ra = cache.begin(a, 2)
    cache.commit(ra, 5)                 # A's node is created first ...
    _, _, rb = cache.begin(b, 2)
    cache.commit(rb, 5)
    cache.release(rb)
    cache.release(ra)                   # ... but A is released last; 2 nodes, 4 pages free
    _, _, rc = cache.begin(list(range(100, 100 + 5 * ps)), 5)   # 5 pages: one eviction, and it must be B's node
    cache.release(rc)
    assert cache.stats()["evictions"] == 1
    assert cache.begin(a, 2)[1] == ps
    assert cache.begin(b, 2)[1] == 0


def test_page_order_is_a_fifo_queue():
    cache = M.PrefixCacheModel(num_pages=8, page_size=2)
    row, _, rid = cache.begin([1, 2, 3, 4, 5], 4)
    assert row == [0, 1, 2, -1]
    cache.release(rid)                  # nothing committed: the three pages go to the back, in order
    row2, _, rid2 = cache.begin(list(range(12)), 6)
    assert row2 == [3, 4, 5, 6, 7, 0]
    cache.commit(rid2, 4)               # pages 3 and 4 become nodes
    cache.release(rid2)                 # 5, 6, 7, 0 return in page-table order: free = 1 2 5 6 7 0
    row3, _, rid3 = cache.begin([50, 51, 52, 53, 54, 55, 56, 57, 58, 59, 60, 61, 62], 7)
    # 7 pages wanted, 6 free: the deeper of the two nodes (page 4) is evicted when the queue runs dry
    assert row3 == [1, 2, 5, 6, 7, 0, 4]


# ---- conservation under random traffic with appends, overlapping lifetimes and a small pool

@pytest.mark.parametrize("seed", range(6))
def test_random_traffic_conserves_pages_and_never_shares_a_writable_page(seed):
    rng = random.Random(seed)
    ps = rng.choice([1, 2, 4, 16])
    cache = M.PrefixCacheModel(num_pages=rng.randrange(20, 60), page_size=ps)
    seqs = _make_sequences(rng, 12, ps)
    live = {}                           # rid -> (tokens, row, prefix_len)
    for step in range(500):
        op = rng.random()
        try:
            if op < 0.4 or not live:
                s = list(rng.choice(seqs))[:rng.randrange(1, 6 * ps)]
                row, pl, rid = cache.begin(s, 64)
                assert pl % ps == 0 and pl <= len(s) - 1
                live[rid] = [s, row, pl]
            elif op < 0.6:
                rid = rng.choice(list(live))
                extra = [rng.randrange(0, 9) for _ in range(rng.randrange(0, 2 * ps))]
                row = cache.append(rid, extra, 64)
                assert row[:len([x for x in live[rid][1] if x >= 0])] == [x for x in live[rid][1] if x >= 0]
                live[rid][0] = live[rid][0] + extra
                live[rid][1] = row
            elif op < 0.8:
                rid = rng.choice(list(live))
                cache.commit(rid, len(live[rid][0]))
            else:
                rid = rng.choice(list(live))
                cache.release(rid)
                del live[rid]
        except M.CacheError as e:
            assert e.status in (M.NO_SPACE, M.INVALID_ARG)
        st = cache.stats()
        assert st["free_pages"] + st["cached_pages"] + st["private_pages"] == st["num_pages"]
        assert st["live_requests"] == len(live) and 0 <= st["evictable_pages"] <= st["cached_pages"]
        # pages that may still be written (beyond a request's committed full pages) belong to one request only
        writable = []
        for rid, (s, row, pl) in live.items():
            n_pages = -(-len(s) // ps)
            assert all(0 <= pg < st["num_pages"] for pg in row[:n_pages])
            rq = cache.requests[rid]
            writable += [pg for pg, private in zip(rq.pages, rq.private) if private]
        assert len(writable) == len(set(writable)) == st["private_pages"]
        assert not set(writable) & set(cache.free)
        assert not set(writable) & {nd.page for nd in cache.nodes}
