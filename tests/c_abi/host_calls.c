/* A C99 program that uses the library through its two public headers only: the calls that need no GPU.
 * Built and run by tests/test_c_abi.py; prints "ok" and exits 0 when every check holds. */
#include "emm.h"
#include "emm_prefix_cache.h"

#include <stdio.h>
#include <string.h>

#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            fprintf(stderr, "line %d: %s\n", __LINE__, #cond);           \
            return 1;                                                    \
        }                                                                \
    } while (0)

int main(void)
{
    emm_batch b;
    size_t bytes = 0;
    memset(&b, 0, sizeof b);
    b.num_reqs = 2;
    b.num_q_heads = 28;
    b.num_kv_heads = 4;
    b.head_dim = 128;
    b.page_size = 16;
    b.num_pages = 64;
    b.max_pages_per_req = 8;
    b.total_new_tokens = 40;
    b.max_new_len = 30;
    b.dtype = EMM_BF16;
    b.softmax_scale = 0.088388f;
    CHECK(emm_version() > 0);
    CHECK(emm_prefill_attn_workspace_size(&b, &bytes) == EMM_OK && bytes == 0);   /* contexts of 128 tokens: nothing is cut */
    b.max_pages_per_req = 1024;
    CHECK(emm_prefill_attn_workspace_size(&b, &bytes) == EMM_OK && bytes > 0);
    b.max_pages_per_req = 8;
    b.page_size = 24;
    CHECK(emm_prefill_attn_workspace_size(&b, &bytes) == EMM_ERR_UNSUPPORTED);
    b.page_size = 16;
    CHECK(emm_prefill_attn(&b, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) == EMM_ERR_NULL);
    CHECK(strlen(emm_status_string(EMM_ERR_WORKSPACE)) > 0);

    {
        /* two requests: page table rows as a prefix cache hands them out */
        const int32_t pt[16] = {0, 1, 2, 3, -1, -1, -1, -1, 0, 1, 4, -1, -1, -1, -1, -1};
        const int32_t prefix[2] = {32, 32}, new_lens[2] = {30, 10}, cu[3] = {0, 30, 40};
        CHECK(emm_validate_batch_host(&b, pt, prefix, new_lens, cu, 1) == EMM_OK);
        {
            const int32_t clash[16] = {0, 1, 2, 3, -1, -1, -1, -1, 0, 1, 2, -1, -1, -1, -1, -1};   /* both write page 2 */
            CHECK(emm_validate_batch_host(&b, clash, prefix, new_lens, cu, 1) == EMM_ERR_INVALID_ARG);
        }
    }

    {
        /* two requests with the same four leading pages (64 cached tokens) and few new tokens: one sharing group */
        const int32_t pt[16] = {5, 6, 7, 8, 9, -1, -1, -1, 5, 6, 7, 8, 10, -1, -1, -1};
        const int32_t prefix[2] = {64, 64}, new_lens[2] = {3, 2}, cu[3] = {0, 3, 5};
        int32_t shared_len[2], g_pt[8], g_prefix[1], g_new[1], g_cu[2], own_pt[16], own_prefix[2];
        emm_prefill_shared_plan plan;
        emm_batch small = b;
        small.total_new_tokens = 5;
        small.max_new_len = 3;
        memset(&plan, 0, sizeof plan);
        plan.req_shared_len = shared_len;
        plan.group_page_table = g_pt;
        plan.group_prefix_lens = g_prefix;
        plan.group_new_lens = g_new;
        plan.group_cu_new_lens = g_cu;
        plan.own_page_table = own_pt;
        plan.own_prefix_lens = own_prefix;
        small.num_q_heads = 256;                                /* 64 query heads per KV head: 192 and 128 rows fill two tiles either way */
        CHECK(emm_prefill_shared_plan_host(&small, pt, prefix, new_lens, cu, 64, 0, &plan) == EMM_OK && plan.num_groups == 0);
        small.num_q_heads = 28;                                 /* 21 and 14 rows: two tiles apart, one together */
        CHECK(emm_prefill_shared_plan_host(&small, pt, prefix, new_lens, cu, 64, 0, &plan) == EMM_OK);
        CHECK(plan.num_groups == 1 && shared_len[0] == 64 && shared_len[1] == 64 && g_prefix[0] == 64 && g_new[0] == 5);
        CHECK(own_prefix[0] == 0 && plan.own.max_pages_per_req == 1 && own_pt[0] == 9 && own_pt[1] == 10);   /* packed rows */
        CHECK(plan.groups.max_pages_per_req == 4 && g_pt[0] == 5 && g_pt[3] == 8);
        CHECK(plan.groups.num_reqs == 1 && plan.own.num_reqs == 2 && plan.groups.max_new_len == 5);
        CHECK(emm_prefill_attn_shared_workspace_size(&plan.groups, &plan.own, &bytes) == EMM_OK && bytes > 0);
        CHECK(emm_prefill_attn_shared(&plan.groups, &plan.own, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL) == EMM_ERR_NULL);
        CHECK(emm_prefill_shared_plan_host(&small, pt, prefix, new_lens, cu, 64, -1, &plan) == EMM_OK && plan.num_groups == 0);
    }

    {
        uint8_t digest[32];
        int64_t ids[48], tokens[60];
        int32_t row[8], prefix_len = -1;
        int64_t req = 0, req2 = 0;
        emm_prefix_cache *cache = NULL;
        emm_prefix_cache_stats st;
        int i;
        CHECK(emm_mm_content_hash("abc", 3, digest) == EMM_OK);
        CHECK(digest[0] == 0xba && digest[1] == 0x78 && digest[31] == 0xad);   /* SHA-256("abc") */
        CHECK(emm_mm_token_ids(digest, 48, ids) == EMM_OK && ids[0] < 0 && ids[47] < 0);
        for (i = 0; i < 12; ++i) tokens[i] = 100 + i;          /* text, then the image's placeholders */
        memcpy(tokens + 12, ids, sizeof ids);
        CHECK(emm_prefix_cache_create(64, 16, &cache) == EMM_OK && cache != NULL);
        CHECK(emm_prefix_cache_begin(cache, tokens, 60, 8, row, &prefix_len, &req) == EMM_OK);
        CHECK(prefix_len == 0 && row[3] >= 0 && row[4] == -1);
        CHECK(emm_prefix_cache_commit(cache, req, 60) == EMM_OK);
        CHECK(emm_prefix_cache_begin(cache, tokens, 60, 8, row, &prefix_len, &req2) == EMM_OK);
        CHECK(prefix_len == 48);                                /* three full pages; the last token is always left */
        CHECK(emm_prefix_cache_release(cache, req) == EMM_OK && emm_prefix_cache_release(cache, req2) == EMM_OK);
        CHECK(emm_prefix_cache_release(cache, req) == EMM_ERR_NOT_FOUND);
        CHECK(emm_prefix_cache_get_stats(cache, &st) == EMM_OK && st.hit_tokens == 48 && st.live_requests == 0);
        emm_prefix_cache_destroy(cache);
    }
    puts("ok");
    return 0;
}
