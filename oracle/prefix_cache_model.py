"""Reference model of the host-side unified multimodal prefix cache.  TEST INFRASTRUCTURE ONLY.

Plain Python objects, dictionaries and linear scans: slow and easy to check by eye against the paper
(Section 3.3, "Unified Multimodal Prefix Cache": a hash per multimodal input, a prefix tree over the
unified token sequence, the longest matching prefix skips prefill; Appendix A: every tree node has a
user count, a node is evictable only at zero, eviction is least-recently-used when the pool is full).
Nothing in the product package imports this file and it imports nothing from the product package.

Readings where the paper is silent (the C library states the same ones in its header):
  * a tree node is one FULL page of ``page_size`` tokens, so matches are whole pages;
  * at least one token of a request is left to prefill: prefix_len <= n_tokens - 1;
  * a logical clock advances by one on every successful begin / commit / release; commit stamps the
    nodes it creates and release stamps every node on the request's path (a node in use cannot be
    evicted, so a stamp at begin would never be looked at before release overwrites it);
  * the victim is the evictable node (no users, no children) with the smallest (stamp, creation number);
  * free pages are a FIFO queue, initially 0 .. num_pages-1; release returns private pages in
    page-table order; an evicted node's page goes to the back of the queue;
  * a failed call changes nothing.

Parity of the tree logic is pinned in tests/test_oracle_prefix_cache.py by models that share none of
this code: content-addressed pages without eviction, a textbook LRU, and conservation invariants.
"""
from __future__ import annotations

import hashlib
from collections import deque
from typing import Dict, List, Optional, Sequence, Tuple

OK, INVALID_ARG, NO_SPACE, NOT_FOUND = "ok", "invalid_arg", "no_space", "not_found"
_M64 = (1 << 64) - 1


class CacheError(Exception):
    def __init__(self, status: str):
        super().__init__(status)
        self.status = status


def mm_content_hash(data: bytes) -> bytes:
    """Appendix B.7: identity of a multimodal input is established with a cryptographic hash (SHA-256)."""
    return hashlib.sha256(data).digest()


def mm_token_ids(digest: bytes, n_tokens: int) -> List[int]:
    """Placeholder ids that stand for an item's vision tokens in the unified sequence: negative (text ids
    are >= 0), a function of the digest and the position only."""
    w0 = int.from_bytes(digest[0:8], "big")
    w1 = int.from_bytes(digest[8:16], "big")
    return [-1 - ((((w0 + j * 0x9E3779B97F4A7C15) & _M64) ^ w1) >> 1) for j in range(n_tokens)]


class _Node:
    __slots__ = ("parent", "key", "page", "users", "stamp", "number", "children")

    def __init__(self, parent, key, page, stamp, number):
        self.parent: Optional[_Node] = parent
        self.key: Tuple[int, ...] = key              # the page's tokens
        self.page: int = page
        self.users = 0
        self.stamp = stamp
        self.number = number                         # creation order
        self.children: Dict[Tuple[int, ...], _Node] = {}


class _Request:
    __slots__ = ("tokens", "pages", "private", "path", "resolved_pages", "n_computed")

    def __init__(self):
        self.tokens: List[int] = []
        self.pages: List[int] = []
        self.private: List[bool] = []                # per page: owned by this request alone
        self.path: List[_Node] = []                  # nodes this request is a user of, root excluded
        self.resolved_pages = 0                      # leading pages that have a node on the path
        self.n_computed = 0


class PrefixCacheModel:
    def __init__(self, num_pages: int, page_size: int):
        if num_pages < 1 or page_size < 1:
            raise CacheError(INVALID_ARG)
        self.num_pages, self.page_size = num_pages, page_size
        self.root = _Node(None, (), -1, 0, 0)
        self.nodes: List[_Node] = []                 # every node but the root
        self.free = deque(range(num_pages))
        self.clock = 0
        self.created = 0
        self.requests: Dict[int, _Request] = {}
        self.next_request = 1
        self.lookups = self.lookup_tokens = self.hit_tokens = self.evictions = 0

    # ---- helpers
    def _pages_for(self, n_tokens: int) -> int:
        return -(-n_tokens // self.page_size)

    def _unused(self) -> int:
        return sum(1 for nd in self.nodes if nd.users == 0)

    def _evict_one(self) -> None:
        victims = [nd for nd in self.nodes if nd.users == 0 and not nd.children]
        nd = min(victims, key=lambda x: (x.stamp, x.number))
        del nd.parent.children[nd.key]
        self.nodes.remove(nd)
        self.free.append(nd.page)
        self.evictions += 1

    def _take_page(self) -> int:
        if not self.free:
            self._evict_one()
        return self.free.popleft()

    def _row(self, rq: _Request, max_pages: int) -> List[int]:
        return rq.pages + [-1] * (max_pages - len(rq.pages))

    # ---- the five operations
    def begin(self, tokens: Sequence[int], max_pages: int):
        n, ps = len(tokens), self.page_size
        if n < 1 or max_pages < self._pages_for(n):
            raise CacheError(INVALID_ARG)
        matched: List[_Node] = []
        node = self.root
        for p in range((n - 1) // ps):               # never the page that holds the last token
            child = node.children.get(tuple(tokens[p * ps:(p + 1) * ps]))
            if child is None:
                break
            matched.append(child)
            node = child
        for nd in matched:
            nd.users += 1
        need = self._pages_for(n) - len(matched)
        if need > len(self.free) + self._unused():
            for nd in matched:
                nd.users -= 1
            raise CacheError(NO_SPACE)
        self.clock += 1
        rq = _Request()
        rq.tokens = list(tokens)
        rq.pages = [nd.page for nd in matched] + [self._take_page() for _ in range(need)]
        rq.private = [False] * len(matched) + [True] * need
        rq.path = matched
        rq.resolved_pages = len(matched)
        rq.n_computed = len(matched) * ps
        rid = self.next_request
        self.next_request += 1
        self.requests[rid] = rq
        self.lookups += 1
        self.lookup_tokens += n
        self.hit_tokens += rq.n_computed
        return self._row(rq, max_pages), rq.n_computed, rid

    def append(self, rid: int, tokens: Sequence[int], max_pages: int):
        rq = self.requests.get(rid)
        if rq is None:
            raise CacheError(NOT_FOUND)
        total = self._pages_for(len(rq.tokens) + len(tokens))
        if max_pages < total:
            raise CacheError(INVALID_ARG)
        need = total - len(rq.pages)
        if need > len(self.free) + self._unused():
            raise CacheError(NO_SPACE)
        rq.tokens += list(tokens)
        for _ in range(need):
            rq.pages.append(self._take_page())
            rq.private.append(True)
        return self._row(rq, max_pages)

    def commit(self, rid: int, n_computed: int) -> None:
        rq = self.requests.get(rid)
        if rq is None:
            raise CacheError(NOT_FOUND)
        if n_computed > len(rq.tokens) or n_computed < rq.n_computed:
            raise CacheError(INVALID_ARG)
        ps = self.page_size
        self.clock += 1
        rq.n_computed = n_computed
        for p in range(rq.resolved_pages, n_computed // ps):
            parent = rq.path[-1] if rq.path else self.root
            key = tuple(rq.tokens[p * ps:(p + 1) * ps])
            child = parent.children.get(key)
            if child is None:                        # publish this request's page
                self.created += 1
                child = _Node(parent, key, rq.pages[p], self.clock, self.created)
                parent.children[key] = child
                self.nodes.append(child)
                rq.private[p] = False
            child.users += 1                         # else: someone published the same content first;
            rq.path.append(child)                    # this request keeps its page as a private duplicate
        rq.resolved_pages = max(rq.resolved_pages, n_computed // ps)

    def release(self, rid: int) -> None:
        rq = self.requests.pop(rid, None)
        if rq is None:
            raise CacheError(NOT_FOUND)
        self.clock += 1
        for nd in rq.path:
            nd.users -= 1
            nd.stamp = self.clock
        for page, private in zip(rq.pages, rq.private):
            if private:
                self.free.append(page)

    def stats(self) -> dict:
        return {
            "lookups": self.lookups, "lookup_tokens": self.lookup_tokens, "hit_tokens": self.hit_tokens,
            "evictions": self.evictions, "num_pages": self.num_pages, "free_pages": len(self.free),
            "cached_pages": len(self.nodes), "evictable_pages": self._unused(),
            "private_pages": sum(sum(rq.private) for rq in self.requests.values()),
            "live_requests": len(self.requests),
        }
