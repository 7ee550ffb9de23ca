/*
 * emm.h -- C ABI of the MI355X (gfx950) prefix-cached paged prefill attention library.
 *
 * The library implements the attention hot path behind a unified multimodal prefix cache
 * (ElasticMM, arXiv 2507.10069, Section 3.3): a request's leading tokens (image or video tokens
 * plus shared text) already have their key/value entries in a paged KV pool (Appendix A), and
 * prefill runs only over the remaining "new" tokens, reading the cached entries instead of
 * recomputing them.  Appendix B.7 states what the result must be: identical to prefilling the
 * whole sequence.  These device operations are exported:
 *
 *   emm_kv_scatter    store the new tokens' K/V rows in their pool slots          (Section 2.2)
 *   emm_prefill_attn  causal grouped-query attention of the new tokens over
 *                     cached prefix + new tokens, read from the pool       (Section 3.3, App. B.7)
 *   emm_cross_attn    unmasked attention of text queries over cached image K/V
 *                     for encoder-decoder models                                  (Section 2.1)
 *   emm_decode_attn   the same attention for the decode step, one new token per request (Section 2.2)
 *   emm_decode_attn_shared  the decode step reading pages that several requests share once (Section 3.3)
 *   emm_decode_step   scatter + decode attention of one step in one launch               (Section 2.2)
 *   emm_kv_pages_pack / emm_kv_pages_unpack  the two ends of a KV cache migration      (Appendix B.5)
 *
 * Conventions common to all calls
 *   - Every pointer marked "device" is memory of the current HIP device, owned by the caller; the
 *     library allocates and frees nothing and keeps no state between calls.
 *   - Calls enqueue work on `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and
 *     return without waiting for it.  Errors are reported by return code only.  Everything a call was
 *     given in device memory, the batch's four arrays included, must stay allocated and unchanged until
 *     that work has finished.
 *   - Host-side checks cover the scalar fields, null pointers and 16-byte alignment of tensor
 *     pointers.  Device-resident arrays (page table, lengths, shared-prefix units) cannot be checked
 *     there: check host copies of them with emm_validate_batch_host.  The kernels force whatever
 *     those arrays hold into the range the scalar fields allow (page ids into the pool, lengths into
 *     the page-table row and the packed tensors), so inconsistent arrays give meaningless results but
 *     no access outside the buffers that were passed.
 *   - Pool layout: [num_pages][num_kv_heads][page_size][head_dim], K and V in separate pools.
 *     Logical token slot i of request r lives in page page_table[r][i / page_size] at offset
 *     i % page_size.  Packed layouts: q, out [T][num_q_heads][head_dim]; k_new, v_new
 *     [T][num_kv_heads][head_dim]; rows of request r are cu_new_lens[r] .. cu_new_lens[r+1]-1.
 *   - Query head h reads KV head h / (num_q_heads / num_kv_heads).
 *   - Element offsets are computed in 64 bits.
 *   - Supported: page_size 16, 32, 64, 128 or 256; EMM_BF16 with head_dim 128 (MFMA kernels); EMM_F32
 *     with head_dim 64 or 128 (plain fp32 kernels).  Anything else returns EMM_ERR_UNSUPPORTED.
 *   - A page that receives new tokens must be referenced by exactly one request: shared pages
 *     (prefix-tree nodes with several users, Appendix A) are read-only.
 */
#ifndef EMM_H
#define EMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    EMM_OK = 0,
    EMM_ERR_NULL = 1,          /* a required pointer is NULL                                   */
    EMM_ERR_INVALID_ARG = 2,   /* a scalar field is out of range or a pointer is misaligned    */
    EMM_ERR_UNSUPPORTED = 3,   /* valid request, but no kernel for this dtype/head_dim/page    */
    EMM_ERR_WORKSPACE = 4,     /* workspace_bytes smaller than emm_prefill_attn_workspace_size */
    EMM_ERR_LAUNCH = 5,        /* the HIP runtime refused the launch                           */
    EMM_ERR_NO_SPACE = 6,      /* prefix cache: every page is held by a live request           */
    EMM_ERR_NOT_FOUND = 7      /* prefix cache: no live request with this id                   */
} emm_status;

typedef enum { EMM_F32 = 0, EMM_BF16 = 1 } emm_dtype;

/* One batch of requests.  Scalars are host values; the four arrays are device memory. */
typedef struct {
    int32_t num_reqs;            /* B >= 0                                                       */
    int32_t num_q_heads;         /* H, a multiple of num_kv_heads                                */
    int32_t num_kv_heads;        /* Hkv                                                          */
    int32_t head_dim;            /* d                                                            */
    int32_t page_size;           /* tokens per page ("block size")                               */
    int32_t num_pages;           /* pages in each pool                                           */
    int32_t max_pages_per_req;   /* row stride of page_table                                     */
    int32_t total_new_tokens;    /* T = cu_new_lens[B]; known to the host so no sync is needed   */
    int32_t max_new_len;         /* max_r new_lens[r]                                            */
    int32_t dtype;               /* emm_dtype of q, k, v, out and both pools                     */
    float softmax_scale;         /* scores are softmax_scale * <q, k>                            */
    int32_t reserved;            /* must be 0                                                    */
    const int32_t *page_table;   /* device [B][max_pages_per_req] physical page ids              */
    const int32_t *prefix_lens;  /* device [B] tokens already valid in the pages                 */
    const int32_t *new_lens;     /* device [B] new tokens = query rows of the request            */
    const int32_t *cu_new_lens;  /* device [B+1] exclusive prefix sum of new_lens                */
} emm_batch;

/*
 * KV scatter (Section 2.2: prefill produces the KV cache of all input tokens; Appendix B.5's
 * exact-copy requirement).  For request r, new token j, KV head h: copy the head_dim elements of
 * k_new[cu_new_lens[r]+j][h] bit for bit to slot prefix_lens[r]+j of request r in k_cache; the same
 * for v_new / v_cache.  No other byte of the pools is written.
 *   k_new, v_new      device, read,  [T][Hkv][d]
 *   k_cache, v_cache  device, write, [num_pages][Hkv][page_size][d]
 * T == 0 is a no-op.
 */
emm_status emm_kv_scatter(const emm_batch *batch, const void *k_new, const void *v_new,
                          void *k_cache, void *v_cache, void *hip_stream);

/* Bytes of device workspace emm_prefill_attn / emm_cross_attn / emm_decode_attn need for this batch: 0 for
 * EMM_F32.  For EMM_BF16 the kernels cut work along the key axis, park the pieces' accumulators in the workspace
 * and merge them with a second kernel on the same stream:
 *   prefill / cross-attention: the work units an XCD has left over after its full rounds of 32 are cut in up to 32
 *     pieces; a piece record is 135168 bytes, and the size is 8 XCDs x the most records an XCD can need: exactly that
 *     of the plan when all requests have the same number of new tokens (0 when that plan cuts nothing, as for 2 x
 *     2048 new tokens on 28 / 4 heads), else a bound from the scalar fields (32 or 64 records per XCD: 34.6 or 69.2
 *     MB), and 0 when no context the page table can hold is long enough to be cut (under 1536 tokens);
 *     emm_prefill_plan_host shows the plan;
 *   decode batch (at most one new token per request and at most 16 query heads per KV head): every context is
 *     cut; 8320 bytes per (request, KV head, piece), a piece being 128 to 1920 keys of the longest context the
 *     page table can hold.
 * The contents need no initialisation and mean nothing afterwards.  Calls on different streams must not share a
 * workspace.  Host-only; reads only the scalar fields. */
emm_status emm_prefill_attn_workspace_size(const emm_batch *batch, size_t *bytes);

/*
 * Prefix-cached causal prefill attention (Section 3.3; Appendix B.7, g_P^remaining).
 * Query row j of request r attends to the request's logical slots 0 .. prefix_lens[r]+j, i.e. to
 * the whole cached prefix and to the new tokens up to and including itself; the new tokens' K/V
 * are read from the pool, so emm_kv_scatter must precede this call on the same stream.
 *   q       device, read,  [T][H][d]
 *   out     device, write, [T][H][d], same dtype as q (bf16 rounded to nearest even)
 *   lse     device, write, [T][H] fp32 natural-log softmax denominators, or NULL
 *   workspace  device scratch of at least emm_prefill_attn_workspace_size bytes, 16-byte aligned (may be
 *              NULL if that size is 0); EMM_ERR_NULL / EMM_ERR_WORKSPACE if missing / too small
 * bf16 path: scores and both products accumulate in fp32, softmax weights are rounded to bf16 for
 * the value product.  Results are run-to-run bitwise deterministic.
 */
emm_status emm_prefill_attn(const emm_batch *batch, const void *q, const void *k_cache,
                            const void *v_cache, void *out, float *lse, void *workspace,
                            size_t workspace_bytes, void *hip_stream);

/*
 * Decode-step attention (Section 2.2: after prefill the decode stage produces one token per iteration
 * from the cached K/V of all earlier tokens, and is memory bound).  emm_prefill_attn for a batch in which
 * every request has at most one new token (max_new_len <= 1, else EMM_ERR_INVALID_ARG): the token of
 * request r attends to slots 0 .. prefix_lens[r], its own K/V having been scattered first.  Arguments,
 * workspace and results as for emm_prefill_attn, which takes the same path for such a batch by itself;
 * the bf16 kernel behind it reads every K/V byte once, cutting each request's context into pieces that
 * fill the chip and merging them through the workspace.
 */
emm_status emm_decode_attn(const emm_batch *batch, const void *q, const void *k_cache,
                           const void *v_cache, void *out, float *lse, void *workspace,
                           size_t workspace_bytes, void *hip_stream);

/*
 * emm_decode_attn for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels and the same results, bit for bit, with the piece
 * records in a fixed array of EMM_DECODE_STATIC_SCRATCH_BYTES inside the library's device image instead of a
 * caller's workspace.  The call allocates and frees nothing.  Every GPU the library is used on holds its own
 * copy of the array until the process ends; its address is looked up on the first call on a device, so the
 * device of `hip_stream` must be the current device.
 *   bf16 decode-shaped batches only (max_new_len <= 1, H / Hkv <= 16), else EMM_ERR_INVALID_ARG /
 *   EMM_ERR_UNSUPPORTED; a batch for which emm_prefill_attn_workspace_size exceeds
 *   EMM_DECODE_STATIC_SCRATCH_BYTES is refused with EMM_ERR_WORKSPACE before anything is launched (64 requests
 *   x 4 KV heads x 8192 tokens need 12.2 MiB).
 * All calls on one GPU share that GPU's array: calls that may overlap there (different streams, several
 * threads) race on it and must be ordered by the caller.  Nothing in the array has to start at zero; a call
 * overwrites what it later reads.
 */
#define EMM_DECODE_STATIC_SCRATCH_BYTES (16u << 20)
emm_status emm_decode_attn_static(const emm_batch *batch, const void *q, const void *k_cache,
                                  const void *v_cache, void *out, float *lse, void *hip_stream);

/*
 * Prefill with shared prefixes (Section 3.3: requests repeat system prompts, images and videos, so several requests
 * of a prefill batch hold the SAME physical pages at the head of their page tables).  When such requests bring few
 * new tokens each (a short question about a video seen before), every one of them on its own fills a small part
 * of a 256-row work unit and streams the whole shared context for it.  Here the query rows of a sharing GROUP are
 * packed into common row tiles for the shared keys, which are then streamed once per group and row tile; each
 * request's remaining keys (the rest of its cached prefix and its new tokens, causal) are done per request; and the
 * two partial results of every row are merged by their softmax denominators -- the same attention as
 * emm_prefill_attn up to rounding (both partial outputs pass through bf16).
 *
 * emm_prefill_shared_plan_host finds the groups from HOST copies of the batch arrays (runs of consecutive requests
 * whose page tables agree on their leading pages; shared length a multiple of 64 tokens, at least
 * max(min_shared_tokens, 64); a group is formed only if its packed rows need fewer 256-row tiles than its members
 * apart).  The three steps cost two more kernel launches and a second pass over every output row than the one plain
 * call, so groups are only worth having when they save enough streaming: with key_tiles_plain / key_tiles_shared
 * the 64-key tiles that all 256-row work units together stream without and with the groups, the plan keeps its
 * groups only if key_tiles_plain - key_tiles_shared >= min_saved_key_tiles (0: always; negative: the library's
 * default, EMM_PREFILL_SHARED_MIN_SAVED_KEY_TILES, measured on MI355X on batches of 8 .. 32 requests).  It writes,
 * into host arrays the caller provides, what the two passes need:
 *   req_shared_len    [B]                        tokens of request r done in its group's pass; 0: in no group
 *   group_page_table  [B / 2][max_pages_per_req] page-table row of each group's first member (*)
 *   group_prefix_lens, group_new_lens [B / 2]    shared length; new tokens of all members together
 *   group_cu_new_lens [B / 2 + 1]                first packed row of each group (members are consecutive)
 *   own_page_table    [B][max_pages_per_req]     each request's row moved left by the pages of its shared part (*)
 *   own_prefix_lens   [B]                        prefix_lens[r] - req_shared_len[r]
 * (*) the sizes are what the caller provides; the rows are written packed, as narrow as what they hold allows, with
 * the row stride that the descriptor states (groups.max_pages_per_req, own.max_pages_per_req <= the batch's): the
 * launches size their grids, and decide whether anything is cut along the keys, from that width.
 * and fills the scalar fields of two descriptors, `groups` (one "request" per group) and `own` (the batch itself
 * with the moved page table), whose four array pointers it leaves NULL: the caller copies the arrays to the
 * device and sets them (own.new_lens and own.cu_new_lens are the batch's).  num_groups == 0: nothing to gain, use
 * emm_prefill_attn (req_shared_len is then all zero and `own` is the batch itself).  rows_tiles_plain /
 * rows_tiles_shared: 256-row tiles per KV head over the shared keys without and with the groups; they and the two
 * key-tile counts describe the grouping that was found, also when it was then given up as not worth it.
 *
 * emm_prefill_attn_shared runs the three steps on the stream: the groups' pass (unmasked, into the workspace), the
 * own pass (emm_prefill_attn of `own`, into out), the merge (into out and lse).  emm_kv_scatter of the ORIGINAL
 * batch must precede it.  req_shared_len: device [B].  Workspace: emm_prefill_attn_shared_workspace_size, 256-byte
 * aligned.  EMM_BF16 only.
 */
#define EMM_PREFILL_SHARED_MIN_SAVED_KEY_TILES 10000
typedef struct {
    int32_t num_groups;
    int64_t rows_tiles_plain, rows_tiles_shared;
    int64_t key_tiles_plain, key_tiles_shared;
    emm_batch groups, own;
    int32_t *req_shared_len;
    int32_t *group_page_table, *group_prefix_lens, *group_new_lens, *group_cu_new_lens;
    int32_t *own_page_table, *own_prefix_lens;
} emm_prefill_shared_plan;
emm_status emm_prefill_shared_plan_host(const emm_batch *batch, const int32_t *host_page_table,
                                        const int32_t *host_prefix_lens, const int32_t *host_new_lens,
                                        const int32_t *host_cu_new_lens, int32_t min_shared_tokens,
                                        int64_t min_saved_key_tiles, emm_prefill_shared_plan *plan);
emm_status emm_prefill_attn_shared_workspace_size(const emm_batch *groups, const emm_batch *own, size_t *bytes);
emm_status emm_prefill_attn_shared(const emm_batch *groups, const emm_batch *own, const int32_t *req_shared_len,
                                   const void *q, const void *k_cache, const void *v_cache, void *out, float *lse,
                                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Decode step with shared prefixes (Section 3.3: requests repeat system prompts and images, so in a decode
 * batch several requests hold the SAME physical pages at the head of their page tables; Section 2.2: the
 * step is bound by reading K/V).  A unit is a run of consecutive requests of the batch together with the
 * number of leading tokens they share; the shared keys and values are then read once per unit instead of
 * once per request, the result is the same attention as emm_decode_attn up to rounding order.
 * Contract for unit u = (first, n, shared_len), all arrays device memory:
 *   - requests first .. first+n-1 each have exactly one new token, n >= 2 and n * (num_q_heads /
 *     num_kv_heads) <= 32;
 *   - shared_len is a multiple of 32, >= 32 and <= prefix_lens[r] of every member, and the members' page
 *     tables agree on entries 0 .. shared_len/page_size - 1;
 *   - req_unit[r] is the unit of request r or -1, req_shared_len[r] the shared_len of that unit or 0; units
 *     do not overlap.
 * emm_shared_prefix_plan_host derives such units from host copies of the batch arrays.
 */
typedef struct {
    int32_t num_units;                 /* U >= 0; with 0 the call is emm_decode_attn with a planning hint    */
    int32_t planned_tiles;             /* hint, host value: sum over units of shared_len / 32 plus sum over  */
                                       /* requests of ceil((tokens the query sees - req_shared_len) / 32);   */
                                       /* 0 = unknown.  Only the way work is cut depends on it, never the    */
                                       /* result: without it every context is planned as the longest one the  */
                                       /* page table can hold, which under-fills the chip on ragged batches.  */
    int32_t max_own_tiles;             /* bound, host value: the largest ceil((tokens the query sees -        */
                                       /* req_shared_len) / 32) over the requests; 0 = not given (the page     */
                                       /* table's width is used).  Unlike the hint it MUST hold when given:    */
                                       /* the grid provides pieces for own parts up to this length only.      */
    int32_t max_unit_tiles;            /* bound, host value: the largest shared_len / 32; 0 = not given        */
    const int32_t *unit_first_req;     /* device [U]                                                         */
    const int32_t *unit_num_reqs;      /* device [U]                                                         */
    const int32_t *unit_shared_len;    /* device [U]                                                         */
    const int32_t *req_unit;           /* device [B]                                                         */
    const int32_t *req_shared_len;     /* device [B]                                                         */
} emm_shared_prefix;

/* Workspace bytes of emm_decode_attn_shared / emm_decode_step for this batch and the four scalar fields of
 * `shared` (the values the call itself will be given; num_units <= num_reqs / 2; the pointers are not looked
 * at; NULL = no units and no hints).
 * EMM_ERR_UNSUPPORTED unless the batch is EMM_BF16, head_dim 128, at most 16 query heads per KV head. */
emm_status emm_decode_attn_shared_workspace_size(const emm_batch *batch, const emm_shared_prefix *shared,
                                                 size_t *bytes);

/* Arguments as for emm_decode_attn, plus the units (`shared` itself is host memory, its arrays device). */
emm_status emm_decode_attn_shared(const emm_batch *batch, const emm_shared_prefix *shared, const void *q,
                                  const void *k_cache, const void *v_cache, void *out, float *lse,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

/* The same for the cross-attention layers of an encoder-decoder model in the decode step (Section 2.1): one
 * text query per request over cached image K/V, unmasked, requests that show the same image sharing its pages.
 * Units as above with "prefix_lens" read as the number of cached image tokens; a request whose tokens are all
 * shared has no part of its own.  emm_shared_prefix_plan_host serves here too (its hint and bounds then
 * overestimate by at most one tile per request, which is harmless). */
emm_status emm_cross_attn_shared(const emm_batch *batch, const emm_shared_prefix *shared, const void *q,
                                 const void *k_cache, const void *v_cache, void *out, float *lse,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One decode step in one call: emm_kv_scatter of the query tokens' K/V rows and emm_decode_attn (or, with
 * units, emm_decode_attn_shared) fused, which saves a kernel launch per layer and step.  k_new / v_new
 * [T][Hkv][d] hold the rows of the new tokens, which need NOT be in the pools beforehand: the attention
 * kernel reads them from here and stores them in their slots (slot prefix_lens[r] of request r), so the pools
 * are written.  `shared` may be NULL (no units, no hints).  Same results as the two separate calls, bit for
 * bit.  Workspace: emm_decode_attn_shared_workspace_size with the same `shared`.  EMM_ERR_UNSUPPORTED unless
 * the batch is EMM_BF16, head_dim 128, at most 16 query heads per KV head (use the two calls then).
 */
emm_status emm_decode_step(const emm_batch *batch, const emm_shared_prefix *shared, const void *q,
                           const void *k_new, const void *v_new, void *k_cache, void *v_cache, void *out,
                           float *lse, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Finds units in a batch given as HOST copies of its arrays: greedily, from each request on, the following
 * requests are added while their page tables share a prefix with the first one's of at least
 * max(32, min_shared_tokens) tokens (whole pages that both requests' cached tokens fill, rounded down to a
 * multiple of 32), the rows still fit, and the number of keys saved, shared_len * (n - 1), does not go down.
 * Requests that share pages must therefore be adjacent in the batch to be found.  Outputs are host arrays:
 * unit_* of length >= num_reqs / 2, req_* of length num_reqs; the four scalar fields of *shared are filled in
 * (its pointers are left alone: set them to the device copies of the arrays).  The hint and the bounds are
 * useful even with no units at all when the contexts are very unequal or much shorter than the page table
 * is wide.  Only the scalar fields of `batch` are read.
 */
emm_status emm_shared_prefix_plan_host(const emm_batch *batch, const int32_t *host_page_table,
                                       const int32_t *host_prefix_lens, const int32_t *host_new_lens,
                                       int32_t min_shared_tokens, int32_t *unit_first_req,
                                       int32_t *unit_num_reqs, int32_t *unit_shared_len, int32_t *req_unit,
                                       int32_t *req_shared_len, emm_shared_prefix *shared);

/*
 * Cross-attention variant (Section 2.1: in encoder-decoder MLLMs text tokens meet vision tokens
 * only in cross-attention layers).  Every query row of request r attends, without mask, to slots
 * 0 .. prefix_lens[r]-1 (the cached image K/V).  new_lens[r] is the number of queries.  A request
 * with prefix_lens[r] == 0 (text-only request in the batch) gets zero rows and lse = -inf.
 * Arguments as for emm_prefill_attn; the pools are only read.
 */
emm_status emm_cross_attn(const emm_batch *batch, const void *q, const void *k_cache,
                          const void *v_cache, void *out, float *lse, void *workspace,
                          size_t workspace_bytes, void *hip_stream);

/*
 * KV page migration primitive (Appendix B.5: when an instance is scaled, a request's KV cache is copied to
 * another GPU exactly and the copy is verified with checksums).  These two calls are the ends of such a
 * move on one GPU each; the transport between them is not part of this library.
 *   emm_kv_pages_pack    gathers pages page_ids[0..n-1] of both pools into `staging`: page i occupies bytes
 *                        [i * 2 * page_bytes, (i+1) * 2 * page_bytes), the K page (all KV heads) first, then
 *                        the V page; checksums[i] (optional) = Adler-32 (RFC 1950) of those bytes.
 *   emm_kv_pages_unpack  scatters such a buffer into pages page_ids[0..n-1] of the destination pools, bit for
 *                        bit, and takes the same checksums of what it received; with `expected` and
 *                        `mismatches` given, *mismatches is incremented once per page whose checksum differs
 *                        from expected[i] (the caller zeroes it beforehand).
 * page_bytes is the size of one page in ONE pool (num_kv_heads * page_size * head_dim * element size), a
 * multiple of 16 up to 1 MiB.  All pointers are device memory, 16-byte aligned (checksums, expected,
 * mismatches: 4); page ids are distinct and inside the pool of num_pages pages.  n == 0 is a no-op.
 */
emm_status emm_kv_pages_pack(const void *k_cache, const void *v_cache, int32_t num_pages, int64_t page_bytes,
                             const int32_t *page_ids, int32_t n, void *staging, uint32_t *checksums,
                             void *hip_stream);
emm_status emm_kv_pages_unpack(const void *staging, const int32_t *page_ids, int32_t n, void *k_cache,
                               void *v_cache, int32_t num_pages, int64_t page_bytes, uint32_t *checksums,
                               const uint32_t *expected, uint32_t *mismatches, void *hip_stream);

/*
 * Host-side consistency check of a batch whose arrays are given as HOST copies (debug / tests).
 * `causal` != 0 checks the prefill contract (pages of prefix+new tokens valid, pages that receive
 * new tokens referenced once), 0 checks the cross-attention contract (pages of the prefix valid).
 * Only the scalar fields of `batch` are read.  Returns EMM_OK or EMM_ERR_INVALID_ARG.
 */
emm_status emm_validate_batch_host(const emm_batch *batch, const int32_t *host_page_table,
                                   const int32_t *host_prefix_lens, const int32_t *host_new_lens,
                                   const int32_t *host_cu_new_lens, int causal);

/*
 * How emm_prefill_attn / emm_cross_attn would lay out an EMM_BF16 batch that is not a decode batch, from the
 * scalar fields and a HOST copy of new_lens (diagnostics, sizing, tests; no GPU work).  The kernels deal the
 * (request, KV head) pairs to the chip's 8 XCDs and cut each pair's query rows into work units of 256 rows
 * (Section 3.3 prefill over cached prefixes; the decomposition is this library's).
 *   fan             each pair is dealt to this many XCDs: 1, or a power of two up to 8 when the batch has fewer than
 *                   8 pairs, or when its requests differ in length and the number of KV heads is no multiple of 8
 *                   (every XCD then gets the same share of every request)
 *   cutting         1: units left over after an XCD's full rounds of 32 may be cut along the keys or halved
 *   slots_per_xcd   workgroups per XCD that may hold a unit; grid = 8 * (slots_per_xcd + 31 if cutting)
 *   units[x]        work units of XCD x
 *   pieces[x]       pieces planned for each of its left-over units (1: none are cut)
 *   uneven_k[x]     > 0: those pieces are a long and a short one, the cut at k / (k + 1) of the keys
 *   rows_only[x]    1: the left-over units are halved along their rows, never cut along the keys
 * with_workspace says whether the call would be given a workspace (without one nothing is cut).
 * EMM_ERR_UNSUPPORTED unless the batch is EMM_BF16 with head_dim 128.
 */
typedef struct {
    int32_t fan, n_row_tiles, pairs_per_xcd, cutting, uneven, slots_per_xcd;
    int64_t grid;
    int32_t units[8], pieces[8], uneven_k[8], rows_only[8];
} emm_prefill_plan;
emm_status emm_prefill_plan_host(const emm_batch *batch, const int32_t *host_new_lens, int with_workspace,
                                 emm_prefill_plan *plan);

const char *emm_status_string(emm_status status);

/* Library version: major * 10000 + minor * 100 + patch. */
int emm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EMM_H */
