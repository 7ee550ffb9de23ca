/*
 * CPU oracle for prefix-cached paged prefill attention.  TEST INFRASTRUCTURE ONLY.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this file.  It
 * shares no code with the HIP library and the library never calls it.
 *
 * What it computes.  The paper's prefix-cache argument (Section 3.3; Appendix B.7, the
 * case analysis ending in g_P^remaining(v, t, k_prefix)) says that prefilling only the
 * un-cached suffix against cached key/value entries gives exactly what prefilling the whole
 * sequence would give.  The method is therefore exact, and the oracle is the plain definition
 * of softmax attention, evaluated one output row at a time in fp64:
 *
 *   - the KV pool is paged (Appendix A: PagedAttention pool): logical token slot i of request
 *     r lives at physical page page_table[r][i / page_size], offset i % page_size;
 *   - scatter: the K/V rows of the new tokens are copied, as bytes, to the slots that follow
 *     the cached prefix (Section 2.2: prefill produces the KV cache of every input token;
 *     Appendix B.5's notion of an exact copy);
 *   - causal row (request r, new token j, query head h): keys 0 .. P_r + j are attended
 *     (the whole cached prefix and the new tokens up to and including j);
 *   - cross row (Section 2.1, encoder-decoder models): every query attends, unmasked, to the
 *     request's L_r cached image tokens;
 *   - grouped-query attention: query head h reads KV head h / (H / Hkv).
 *
 * There is no tiling, no online softmax and no reordering: scores, their maximum, the
 * exponentials, their sum and the weighted sum of V are separate passes over the row.
 * Inputs are fp32 values or bf16 bit patterns, widened exactly to double.
 *
 * Parity pins (tests/test_oracle_*.py): dense recomputation without cache or pages on tiny
 * inputs, closed forms (zero keys -> running mean of V; constant V; single key; dominant key;
 * key-shift invariance), hand-derived fixtures under tests/golden/, scipy's logsumexp/softmax
 * with page size 1, and the invariants cached == recomputed, page-permutation invariance,
 * rows of softmax weights sum to 1, byte-exact scatter.  The paper prints no numeric worked
 * example for this path, so beyond those pins numeric parity is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_CAUSAL = 0, ORACLE_CROSS = 1 };

/* exact widening of one stored element to double */
static double widen(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32) {
        return (double)((const float *)base)[idx];
    } else {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
}

/* element index of (page, kv head, in-page offset, channel 0) in a pool laid out
 * [num_pages][Hkv][page_size][d] */
static int64_t pool_index(int64_t page, int kv_head, int off, int n_kv, int page_size, int d)
{
    return ((page * n_kv + kv_head) * (int64_t)page_size + off) * d;
}

/*
 * KV scatter: for request r, new token j, KV head h, copy the d elements of
 * k_new[cu[r] + j][h][:] to logical slot P_r + j of request r, byte for byte; same for V.
 * Returns 0, or -1 if a page id is out of range.
 */
int oracle_kv_scatter(int n_req, int n_kv, int d, int page_size, int num_pages, int max_pages,
                      int elt_bytes, const int32_t *page_table, const int32_t *prefix_lens,
                      const int32_t *new_lens, const int32_t *cu_new_lens,
                      const void *k_new, const void *v_new, void *k_cache, void *v_cache)
{
    const size_t row_bytes = (size_t)d * (size_t)elt_bytes;
    for (int r = 0; r < n_req; ++r) {
        for (int j = 0; j < new_lens[r]; ++j) {
            const int pos = prefix_lens[r] + j;
            const int32_t page = page_table[(int64_t)r * max_pages + pos / page_size];
            if (page < 0 || page >= num_pages) return -1;
            for (int h = 0; h < n_kv; ++h) {
                const int64_t src = ((int64_t)(cu_new_lens[r] + j) * n_kv + h) * d;
                const int64_t dst = pool_index(page, h, pos % page_size, n_kv, page_size, d);
                memcpy((char *)k_cache + dst * elt_bytes, (const char *)k_new + src * elt_bytes, row_bytes);
                memcpy((char *)v_cache + dst * elt_bytes, (const char *)v_new + src * elt_bytes, row_bytes);
            }
        }
    }
    return 0;
}

/* number of keys the query row (request r, new token j) attends to */
static int attended_len(int kind, int prefix_len, int j)
{
    return kind == ORACLE_CAUSAL ? prefix_len + j + 1 : prefix_len;
}

/*
 * One output row: query = packed token t (request r, in-request index j), query head h.
 * weights (optional, length >= attended_len) receives the normalised softmax weights.
 */
static void attend_row(int kind, int dtype, int n_q, int n_kv, int d, int page_size, int max_pages,
                       double scale, const int32_t *page_table, int r, int j, int prefix_len,
                       int64_t t, int h, const void *q, const void *k_cache, const void *v_cache,
                       double *scores, double *out_row, double *lse, double *weights)
{
    const int group = n_q / n_kv;
    const int kv_head = h / group;
    const int len = attended_len(kind, prefix_len, j);
    const int64_t q_at = (t * n_q + h) * d;

    for (int c = 0; c < d; ++c) out_row[c] = 0.0;
    if (len <= 0) {             /* cross-attention with nothing cached: zero row, lse = -inf */
        *lse = -INFINITY;
        return;
    }
    /* scores s_i = scale * <q, k_i> */
    for (int i = 0; i < len; ++i) {
        const int32_t page = page_table[(int64_t)r * max_pages + i / page_size];
        const int64_t k_at = pool_index(page, kv_head, i % page_size, n_kv, page_size, d);
        double dot = 0.0;
        for (int c = 0; c < d; ++c) dot += widen(q, q_at + c, dtype) * widen(k_cache, k_at + c, dtype);
        scores[i] = scale * dot;
    }
    /* softmax over the row */
    double m = scores[0];
    for (int i = 1; i < len; ++i) if (scores[i] > m) m = scores[i];
    double z = 0.0;
    for (int i = 0; i < len; ++i) { scores[i] = exp(scores[i] - m); z += scores[i]; }
    /* out = sum_i (p_i / Z) v_i */
    for (int i = 0; i < len; ++i) {
        const double w = scores[i] / z;
        if (weights) weights[i] = w;
        const int32_t page = page_table[(int64_t)r * max_pages + i / page_size];
        const int64_t v_at = pool_index(page, kv_head, i % page_size, n_kv, page_size, d);
        for (int c = 0; c < d; ++c) out_row[c] += w * widen(v_cache, v_at + c, dtype);
    }
    *lse = m + log(z);
}

/* request that owns packed token t */
static int find_request(int n_req, const int32_t *cu_new_lens, int64_t t)
{
    int r = 0;
    while (r + 1 < n_req && t >= cu_new_lens[r + 1]) ++r;
    return r;
}

/*
 * Attention for a set of packed query tokens (all query heads of each).
 *   kind      ORACLE_CAUSAL or ORACLE_CROSS
 *   tokens    n_tokens packed token indices in [0, T), or NULL meaning 0 .. n_tokens-1
 *   out       double [n_tokens][H][d]
 *   lse       double [n_tokens][H]   (log of the softmax denominator, natural log, scaled scores)
 * The pool must already contain the new tokens' K/V (call oracle_kv_scatter first).
 * Returns 0, -1 on a page id out of range, -2 on allocation failure.
 */
int oracle_attention(int kind, int dtype, int n_req, int n_q, int n_kv, int d, int page_size,
                     int num_pages, int max_pages, double scale, const int32_t *page_table,
                     const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new_lens,
                     const void *q, const void *k_cache, const void *v_cache,
                     int64_t n_tokens, const int64_t *tokens, double *out, double *lse)
{
    /* validate the pages every selected row will touch, and find the longest row */
    int longest = 1;
    for (int64_t s = 0; s < n_tokens; ++s) {
        const int64_t t = tokens ? tokens[s] : s;
        const int r = find_request(n_req, cu_new_lens, t);
        const int j = (int)(t - cu_new_lens[r]);
        if (j < 0 || j >= new_lens[r]) return -1;
        const int len = attended_len(kind, prefix_lens[r], j);
        if (len > longest) longest = len;
        for (int i = 0; i < len; i += page_size) {
            const int32_t page = page_table[(int64_t)r * max_pages + i / page_size];
            if (page < 0 || page >= num_pages) return -1;
        }
    }
    int failed = 0;
#pragma omp parallel
    {
        double *scores = (double *)malloc(sizeof(double) * (size_t)longest);
        if (!scores) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for collapse(2) schedule(dynamic, 4)
        for (int64_t s = 0; s < n_tokens; ++s) {
            for (int h = 0; h < n_q; ++h) {
                if (!scores) continue;
                const int64_t t = tokens ? tokens[s] : s;
                const int r = find_request(n_req, cu_new_lens, t);
                const int j = (int)(t - cu_new_lens[r]);
                attend_row(kind, dtype, n_q, n_kv, d, page_size, max_pages, scale, page_table, r, j,
                           prefix_lens[r], t, h, q, k_cache, v_cache, scores,
                           out + (s * n_q + h) * d, lse + s * n_q + h, NULL);
            }
        }
        free(scores);
    }
    return failed ? -2 : 0;
}

/*
 * Normalised softmax weights of one row (packed token t, query head h):
 * weights[0 .. attended_len) ; returns the attended length, or -1 on error.
 */
int oracle_row_weights(int kind, int dtype, int n_req, int n_q, int n_kv, int d, int page_size,
                       int num_pages, int max_pages, double scale, const int32_t *page_table,
                       const int32_t *prefix_lens, const int32_t *new_lens, const int32_t *cu_new_lens,
                       const void *q, const void *k_cache, const void *v_cache,
                       int64_t t, int h, double *weights, int weights_cap)
{
    const int r = find_request(n_req, cu_new_lens, t);
    const int j = (int)(t - cu_new_lens[r]);
    if (j < 0 || j >= new_lens[r] || h < 0 || h >= n_q) return -1;
    const int len = attended_len(kind, prefix_lens[r], j);
    if (len > weights_cap) return -1;
    for (int i = 0; i < len; i += page_size) {
        const int32_t page = page_table[(int64_t)r * max_pages + i / page_size];
        if (page < 0 || page >= num_pages) return -1;
    }
    double *scores = (double *)malloc(sizeof(double) * (size_t)(len > 0 ? len : 1));
    double *row = (double *)malloc(sizeof(double) * (size_t)d);
    if (!scores || !row) { free(scores); free(row); return -1; }
    double lse;
    attend_row(kind, dtype, n_q, n_kv, d, page_size, max_pages, scale, page_table, r, j, prefix_lens[r],
               t, h, q, k_cache, v_cache, scores, row, &lse, weights);
    free(scores);
    free(row);
    return len;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
