/*
 * emm_prefix_cache.h -- C ABI of the host-side unified multimodal prefix cache (ElasticMM, arXiv
 * 2507.10069, Section 3.3 "Unified Multimodal Prefix Cache" and Appendix A), the step that comes
 * before the device path of emm.h: it decides, for every request, how many leading tokens already
 * have their K/V in the paged pool and which physical pages hold them, i.e. it produces the
 * `page_table` rows and `prefix_lens` that emm_kv_scatter / emm_prefill_attn / emm_decode_attn
 * consume.  Everything here is host memory and host arithmetic; no HIP call is made.
 *
 * What the paper fixes, and how it is taken here
 *   - Two pools (Section 3.3).  Pool 1 maps a multimodal input to its encoded tokens, looked up
 *     by a hash of the input ("cryptographic", Appendix B.7): emm_mm_content_hash is SHA-256
 *     (FIPS 180-4) and emm_mm_token_ids turns a digest into the placeholder ids that stand for the
 *     item's vision tokens in the unified sequence, so that identical inputs give identical id
 *     runs.  Storing the encoded tokens themselves is the vision encoder's side and is not here.
 *   - Pool 2 is a prefix tree over the unified token sequence (text ids and multimodal
 *     placeholder ids alike); the longest cached prefix of a new request skips prefill and its
 *     K/V pages are reused.  Appendix A: every tree node carries a user count, a node may be
 *     evicted only when that count is zero, and eviction goes in least-recently-used order when
 *     the pool is full.
 *   - Granularity.  The device kernels read pages of `page_size` tokens, so a tree node is one
 *     FULL page and matches are whole pages: prefix_len is a multiple of page_size.  (The paper
 *     manages its pool token by token; with pages a partially matching page is recomputed.)
 *   - At least one token of every request is left to prefill (its logits are needed), so
 *     prefix_len <= n_tokens - 1.
 *
 * Order of events, all deterministic (needed so that an independent model can be compared id by id)
 *   - A logical clock advances by one on every begin / commit / release call.
 *   - commit stamps the nodes it creates with the clock, release stamps every node on the request's
 *     path.  (A node in use cannot be evicted, so its stamp is not looked at before its last user's
 *     release overwrites it; "recently used" therefore means recently released.)
 *   - Evictable = user count 0 and no children.  The victim is the evictable node with the smallest
 *     (stamp, creation number).  Its page goes to the back of the free queue.
 *   - Free pages are a FIFO queue, initially 0, 1, ..., num_pages-1; release returns a request's
 *     private pages in page-table order.
 *
 * Not thread-safe: one cache belongs to one scheduler thread.
 */
#ifndef EMM_PREFIX_CACHE_H
#define EMM_PREFIX_CACHE_H

#include "emm.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct emm_prefix_cache emm_prefix_cache;   /* opaque; host memory owned by the library */

typedef struct {
    int64_t lookups;          /* successful begin calls                                          */
    int64_t lookup_tokens;    /* tokens of those requests                                        */
    int64_t hit_tokens;       /* of them, tokens served from cached pages (sum of prefix_len)    */
    int64_t evictions;        /* nodes evicted so far                                            */
    int32_t num_pages;        /* pool size                                                       */
    int32_t free_pages;       /* in the free queue                                               */
    int32_t cached_pages;     /* owned by tree nodes (shared, read-only)                         */
    int32_t evictable_pages;  /* of them, nodes with user count 0 (all reclaimable, leaves first)*/
    int32_t private_pages;    /* owned by live requests (not yet published, or duplicates)       */
    int32_t live_requests;
} emm_prefix_cache_stats;

/*
 * SHA-256 of n_bytes at `data` (host) into digest[32] (Appendix B.7: input identity is verified
 * with a cryptographic hash).  data may be NULL iff n_bytes == 0.
 */
emm_status emm_mm_content_hash(const void *data, size_t n_bytes, uint8_t digest[32]);

/*
 * Placeholder ids of the n_tokens vision tokens of a multimodal item with this digest, for use in
 * the unified sequence: with w0, w1 the first two big-endian 64-bit words of the digest,
 *   ids[j] = -1 - (int64)(((w0 + j * 0x9E3779B97F4A7C15) ^ w1) >> 1)       (arithmetic mod 2^64)
 * Always negative, so they never collide with text token ids (>= 0).
 */
emm_status emm_mm_token_ids(const uint8_t digest[32], int32_t n_tokens, int64_t *ids);

/* A cache over a pool of num_pages pages of page_size tokens (both >= 1).  *cache receives the handle. */
emm_status emm_prefix_cache_create(int32_t num_pages, int32_t page_size, emm_prefix_cache **cache);
void emm_prefix_cache_destroy(emm_prefix_cache *cache);   /* NULL is allowed */

/*
 * Admit a request (Section 3.3: find the longest matching prefix; that portion skips prefill).
 *   tokens[n_tokens]        host, the unified sequence, n_tokens >= 1
 *   page_table_row[max_pages]  host, written: entries 0 .. ceil(n_tokens/page_size)-1 are the
 *                           request's pages (the matched prefix pages first, then newly
 *                           allocated private pages), the rest -1
 *   *prefix_len             tokens whose K/V are already in those pages (multiple of page_size,
 *                           <= n_tokens - 1); the caller prefills tokens prefix_len .. n_tokens-1
 *   *request                id for the later calls (> 0)
 * The matched nodes get one more user each.  Pages are taken from the free queue, evicting
 * least-recently-used unused nodes when it runs dry.  EMM_ERR_NO_SPACE if even that is not
 * enough, EMM_ERR_INVALID_ARG if max_pages is too small or n_tokens < 1; on any error the cache is
 * unchanged.
 */
emm_status emm_prefix_cache_begin(emm_prefix_cache *cache, const int64_t *tokens, int32_t n_tokens,
                                  int32_t max_pages, int32_t *page_table_row, int32_t *prefix_len,
                                  int64_t *request);

/*
 * The request grows by n_tokens (decode: the tokens it generated; chunked prefill: the next
 * chunk).  Pages are allocated as for begin; page_table_row is rewritten in full.  On error the
 * cache and the request are unchanged.
 */
emm_status emm_prefix_cache_append(emm_prefix_cache *cache, int64_t request, const int64_t *tokens,
                                   int32_t n_tokens, int32_t max_pages, int32_t *page_table_row);

/*
 * The caller states that the K/V of the request's first n_computed tokens are in their pages.  Every
 * full page among them that is not yet in the tree is published: it becomes a node below the
 * request's path (one more user: this request) and from then on is shared and read-only.  Where
 * the tree already has a node with the same page content below the same path (another request
 * published it first), the request keeps its own page as a private duplicate and its path
 * continues through the existing node.  EMM_ERR_INVALID_ARG if n_computed exceeds the request's
 * tokens or is smaller than at an earlier commit.
 */
emm_status emm_prefix_cache_commit(emm_prefix_cache *cache, int64_t request, int32_t n_computed);

/*
 * The request is finished: every node on its path loses one user (Appendix A: at zero a node
 * becomes eligible for eviction) and is stamped with the clock; its private pages return to the
 * free queue.  Published pages stay cached until evicted.
 */
emm_status emm_prefix_cache_release(emm_prefix_cache *cache, int64_t request);

emm_status emm_prefix_cache_get_stats(const emm_prefix_cache *cache, emm_prefix_cache_stats *stats);

#ifdef __cplusplus
}
#endif
#endif /* EMM_PREFIX_CACHE_H */
