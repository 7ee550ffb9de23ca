// C ABI of the library: host-side validation and dispatch to the kernels.  See include/emm.h for the
// contract of every entry point.  All checks that can fail run before the first HIP call, so the
// error paths work on a machine without a GPU.
#include "../../include/emm.h"
#include "emm_internal.h"

#include <algorithm>
#include <initializer_list>
#include <cmath>
#include <cstdint>
#include <vector>

namespace {

constexpr int kVersion = 100;   // 0.1.0

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

emm_status check_scalars(const emm_batch* b)
{
    if (b == nullptr) return EMM_ERR_NULL;
    if (b->num_reqs < 0 || b->num_q_heads <= 0 || b->num_kv_heads <= 0 || b->head_dim <= 0 ||
        b->page_size <= 0 || b->num_pages < 0 || b->max_pages_per_req < 0 || b->total_new_tokens < 0 ||
        b->max_new_len < 0 || b->max_new_len > b->total_new_tokens || b->reserved != 0)
        return EMM_ERR_INVALID_ARG;
    if (b->num_q_heads % b->num_kv_heads != 0) return EMM_ERR_INVALID_ARG;
    if (b->dtype != EMM_F32 && b->dtype != EMM_BF16) return EMM_ERR_INVALID_ARG;
    if (!(b->softmax_scale > 0.0f) || !std::isfinite(b->softmax_scale)) return EMM_ERR_INVALID_ARG;
    if (b->num_reqs > 0 && b->total_new_tokens > 0 && b->max_new_len == 0) return EMM_ERR_INVALID_ARG;
    return EMM_OK;
}

emm_status check_supported(const emm_batch* b)
{
    if (b->page_size != 16 && b->page_size != 32 && b->page_size != 64 && b->page_size != 128 && b->page_size != 256)
        return EMM_ERR_UNSUPPORTED;
    if (b->dtype == EMM_BF16 && b->head_dim != 128) return EMM_ERR_UNSUPPORTED;
    if (b->dtype == EMM_F32 && b->head_dim != 64 && b->head_dim != 128) return EMM_ERR_UNSUPPORTED;
    return EMM_OK;
}

emm_status check_arrays(const emm_batch* b)
{
    if (b->num_reqs == 0) return EMM_OK;
    if (b->page_table == nullptr || b->prefix_lens == nullptr || b->new_lens == nullptr ||
        b->cu_new_lens == nullptr)
        return EMM_ERR_NULL;
    return EMM_OK;
}

emm::BatchView view_of(const emm_batch* b)
{
    emm::BatchView v;
    v.page_table = b->page_table;
    v.prefix_lens = b->prefix_lens;
    v.new_lens = b->new_lens;
    v.cu_new_lens = b->cu_new_lens;
    v.num_reqs = b->num_reqs;
    v.num_q_heads = b->num_q_heads;
    v.num_kv_heads = b->num_kv_heads;
    v.head_dim = b->head_dim;
    v.page_size = b->page_size;
    v.page_shift = 0;
    while ((16 << v.page_shift) < b->page_size) ++v.page_shift;
    v.num_pages = b->num_pages;
    v.max_pages = b->max_pages_per_req;
    v.total_new_tokens = b->total_new_tokens;
    v.max_new_len = b->max_new_len;
    v.softmax_scale = b->softmax_scale;
    return v;
}

emm::SharedPrefixView shared_view_of(const emm_shared_prefix* sp)
{
    return emm::SharedPrefixView{sp->unit_first_req, sp->unit_num_reqs, sp->unit_shared_len, sp->req_unit,
                                 sp->req_shared_len, sp->num_units, sp->planned_tiles, sp->max_own_tiles,
                                 sp->max_unit_tiles};
}

// sp: shared-prefix units of a decode batch, or nullptr
emm_status attention(const emm_batch* b, const void* q, const void* k_cache, const void* v_cache, void* out,
                     float* lse, void* workspace, size_t workspace_bytes, void* hip_stream, int causal,
                     const emm_shared_prefix* sp = nullptr, const void* k_new = nullptr, const void* v_new = nullptr,
                     bool fused = false, bool static_scratch = false)
{
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    st = check_supported(b);
    if (st != EMM_OK) return st;
    static const emm_shared_prefix no_units = {};
    if (sp != nullptr) {
        if (sp->num_units == 0 && sp->planned_tiles == 0 && sp->max_own_tiles == 0) sp = nullptr;
    }
    if (fused && sp == nullptr) sp = &no_units;              // the fused step goes through the same planner
    size_t need = 0;
    st = sp != nullptr ? emm_decode_attn_shared_workspace_size(b, sp, &need)
                       : emm_prefill_attn_workspace_size(b, &need);
    if (st != EMM_OK) return st;
    if (static_scratch) {
        // the decode kernels with the library's own fixed array in place of a workspace
        if (b->dtype != EMM_BF16 || !emm::attn_bf16_decode_applies(view_of(b))) return EMM_ERR_UNSUPPORTED;
        if (need > emm::attn_bf16_decode_static_scratch_bytes()) return EMM_ERR_WORKSPACE;
        workspace = nullptr;
        workspace_bytes = need;
        need = 0;
    }
    if (sp != nullptr && sp->num_units > 0 && (sp->unit_first_req == nullptr || sp->unit_num_reqs == nullptr || sp->unit_shared_len == nullptr ||
                          sp->req_unit == nullptr || sp->req_shared_len == nullptr))
        return EMM_ERR_NULL;
    if (b->num_reqs == 0 || b->total_new_tokens == 0) return EMM_OK;
    st = check_arrays(b);
    if (st != EMM_OK) return st;
    if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr) return EMM_ERR_NULL;
    if (fused && (k_new == nullptr || v_new == nullptr)) return EMM_ERR_NULL;
    if (fused && (!aligned16(k_new) || !aligned16(v_new))) return EMM_ERR_INVALID_ARG;
    if (need > 0 && workspace == nullptr) return EMM_ERR_NULL;
    if (workspace_bytes < need) return EMM_ERR_WORKSPACE;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) ||
        (lse != nullptr && (reinterpret_cast<uintptr_t>(lse) & 3u) != 0) ||
        (workspace != nullptr && !aligned16(workspace)))
        return EMM_ERR_INVALID_ARG;
    if (b->num_pages == 0 || b->max_pages_per_req == 0) return EMM_ERR_INVALID_ARG;

    emm::AttnArgs args;
    args.b = view_of(b);
    args.q = q;
    args.k_cache = k_cache;
    args.v_cache = v_cache;
    args.out = out;
    args.lse = lse;
    args.causal = causal;
    args.workspace = need > 0 ? workspace : nullptr;
    args.k_new = k_new;
    args.v_new = v_new;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err;
    if (static_scratch) {
        err = emm::launch_attn_bf16_decode_static(args, stream);
    } else if (sp != nullptr) {
        const emm::SharedPrefixView sv = shared_view_of(sp);
        err = fused ? emm::launch_attn_bf16_decode_step(args, sv, stream)
                    : emm::launch_attn_bf16_decode_shared(args, sv, stream);
    } else if (b->dtype != EMM_BF16) err = emm::launch_attn_f32(args, stream);
    else if (emm::attn_bf16_decode_applies(args.b)) err = emm::launch_attn_bf16_decode(args, stream);
    else err = emm::launch_attn_bf16_d128(args, stream);
    return err == hipSuccess ? EMM_OK : EMM_ERR_LAUNCH;
}

}  // namespace

extern "C" {

emm_status emm_kv_scatter(const emm_batch* b, const void* k_new, const void* v_new, void* k_cache,
                          void* v_cache, void* hip_stream)
{
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    st = check_supported(b);
    if (st != EMM_OK) return st;
    if (b->num_reqs == 0 || b->total_new_tokens == 0) return EMM_OK;
    st = check_arrays(b);
    if (st != EMM_OK) return st;
    if (k_new == nullptr || v_new == nullptr || k_cache == nullptr || v_cache == nullptr) return EMM_ERR_NULL;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
        return EMM_ERR_INVALID_ARG;
    if (b->num_pages == 0 || b->max_pages_per_req == 0) return EMM_ERR_INVALID_ARG;
    const int elt = (b->dtype == EMM_BF16) ? 2 : 4;
    const hipError_t err = emm::launch_kv_scatter(view_of(b), k_new, v_new, k_cache, v_cache, elt,
                                                  static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? EMM_OK : EMM_ERR_LAUNCH;
}

emm_status emm_prefill_attn_workspace_size(const emm_batch* b, size_t* bytes)
{
    if (bytes == nullptr) return EMM_ERR_NULL;
    *bytes = 0;
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    st = check_supported(b);
    if (st != EMM_OK) return st;
    if (b->dtype == EMM_BF16) {
        const emm::BatchView v = view_of(b);
        *bytes = emm::attn_bf16_decode_applies(v) ? emm::attn_bf16_decode_workspace_bytes(v)
                                                  : emm::attn_bf16_d128_workspace_bytes(v);
    }
    return EMM_OK;
}

emm_status emm_prefill_attn(const emm_batch* b, const void* q, const void* k_cache, const void* v_cache,
                            void* out, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return attention(b, q, k_cache, v_cache, out, lse, workspace, workspace_bytes, hip_stream, 1);
}

emm_status emm_decode_attn(const emm_batch* b, const void* q, const void* k_cache, const void* v_cache,
                           void* out, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (b != nullptr && b->max_new_len > 1) return EMM_ERR_INVALID_ARG;
    return attention(b, q, k_cache, v_cache, out, lse, workspace, workspace_bytes, hip_stream, 1);
}

emm_status emm_decode_attn_static(const emm_batch* b, const void* q, const void* k_cache, const void* v_cache,
                                  void* out, float* lse, void* hip_stream)
{
    static_assert(EMM_DECODE_STATIC_SCRATCH_BYTES == (16u << 20), "the header states the size of the fixed array");
    if (b != nullptr && b->max_new_len > 1) return EMM_ERR_INVALID_ARG;
    return attention(b, q, k_cache, v_cache, out, lse, nullptr, 0, hip_stream, 1, nullptr, nullptr, nullptr, false, true);
}

emm_status emm_decode_attn_shared_workspace_size(const emm_batch* b, const emm_shared_prefix* sp, size_t* bytes)
{
    if (bytes == nullptr) return EMM_ERR_NULL;
    *bytes = 0;
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    st = check_supported(b);
    if (st != EMM_OK) return st;
    static const emm_shared_prefix no_units = {};
    if (sp == nullptr) sp = &no_units;
    if (sp->num_units < 0 || sp->num_units > b->num_reqs / 2 || sp->planned_tiles < 0 || sp->max_own_tiles < 0 ||
        sp->max_unit_tiles < 0)
        return EMM_ERR_INVALID_ARG;
    if (b->max_new_len > 1) return EMM_ERR_INVALID_ARG;
    const emm::BatchView v = view_of(b);
    if (b->dtype != EMM_BF16 || !emm::attn_bf16_decode_applies(v)) return EMM_ERR_UNSUPPORTED;
    *bytes = emm::attn_bf16_decode_shared_workspace_bytes(v, shared_view_of(sp));
    return EMM_OK;
}

emm_status emm_decode_attn_shared(const emm_batch* b, const emm_shared_prefix* shared, const void* q,
                                  const void* k_cache, const void* v_cache, void* out, float* lse, void* workspace,
                                  size_t workspace_bytes, void* hip_stream)
{
    if (b != nullptr && b->max_new_len > 1) return EMM_ERR_INVALID_ARG;
    return attention(b, q, k_cache, v_cache, out, lse, workspace, workspace_bytes, hip_stream, 1, shared);
}

emm_status emm_cross_attn_shared(const emm_batch* b, const emm_shared_prefix* shared, const void* q,
                                 const void* k_cache, const void* v_cache, void* out, float* lse, void* workspace,
                                 size_t workspace_bytes, void* hip_stream)
{
    if (b != nullptr && b->max_new_len > 1) return EMM_ERR_INVALID_ARG;
    return attention(b, q, k_cache, v_cache, out, lse, workspace, workspace_bytes, hip_stream, 0, shared);
}

emm_status emm_decode_step(const emm_batch* b, const emm_shared_prefix* shared, const void* q, const void* k_new,
                           const void* v_new, void* k_cache, void* v_cache, void* out, float* lse, void* workspace,
                           size_t workspace_bytes, void* hip_stream)
{
    if (b != nullptr && b->max_new_len > 1) return EMM_ERR_INVALID_ARG;
    return attention(b, q, k_cache, v_cache, out, lse, workspace, workspace_bytes, hip_stream, 1, shared, k_new, v_new,
                     true);
}

emm_status emm_shared_prefix_plan_host(const emm_batch* b, const int32_t* pt, const int32_t* prefix,
                                       const int32_t* new_lens, int32_t min_shared_tokens, int32_t* unit_first_req,
                                       int32_t* unit_num_reqs, int32_t* unit_shared_len, int32_t* req_unit,
                                       int32_t* req_shared_len, emm_shared_prefix* shared)
{
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    if (shared == nullptr) return EMM_ERR_NULL;
    shared->num_units = shared->planned_tiles = shared->max_own_tiles = shared->max_unit_tiles = 0;
    if (b->num_reqs == 0) return EMM_OK;
    if (pt == nullptr || prefix == nullptr || new_lens == nullptr || unit_first_req == nullptr ||
        unit_num_reqs == nullptr || unit_shared_len == nullptr || req_unit == nullptr || req_shared_len == nullptr)
        return EMM_ERR_NULL;
    const int B = b->num_reqs, ps = b->page_size;
    const int cap = 32 / (b->num_q_heads / b->num_kv_heads);             // requests whose rows fit one MFMA tile
    const int floor_len = min_shared_tokens < 32 ? 32 : min_shared_tokens;
    for (int r = 0; r < B; ++r) {
        req_unit[r] = -1;
        req_shared_len[r] = 0;
    }
    // tokens that requests i and j share: leading equal page-table entries, counted only as far as both
    // requests' cached tokens fill the page
    auto common = [&](int i, int j) -> int64_t {
        const int64_t full = std::min(prefix[i], prefix[j]) / ps;
        const int32_t* a = pt + static_cast<int64_t>(i) * b->max_pages_per_req;
        const int32_t* c = pt + static_cast<int64_t>(j) * b->max_pages_per_req;
        int64_t p = 0;
        while (p < full && p < b->max_pages_per_req && a[p] == c[p]) ++p;
        return p * ps;
    };
    int U = 0;
    for (int i = 0; i < B;) {
        int n = 1;
        int64_t shared = 0;
        if (new_lens[i] == 1 && cap >= 2) {
            int64_t cur = INT64_MAX;
            for (int j = i + 1; j < B && n < cap && new_lens[j] == 1; ++j) {
                const int64_t cand = std::min(cur, common(i, j)) / 32 * 32;
                // one more request pays if the keys saved, shared * (requests - 1), do not go down
                if (cand < floor_len || (n > 1 && cand * n < shared * (n - 1))) break;
                cur = shared = cand;
                ++n;
            }
        }
        if (n >= 2) {
            unit_first_req[U] = i;
            unit_num_reqs[U] = n;
            unit_shared_len[U] = static_cast<int32_t>(shared);
            for (int r = i; r < i + n; ++r) {
                req_unit[r] = U;
                req_shared_len[r] = static_cast<int32_t>(shared);
            }
            ++U;
        }
        i += n;
    }
    shared->num_units = U;
    int64_t tiles = 0, own_max = 0, unit_max = 0;
    for (int u = 0; u < U; ++u) {
        tiles += unit_shared_len[u] / 32;
        unit_max = std::max<int64_t>(unit_max, unit_shared_len[u] / 32);
    }
    for (int r = 0; r < B; ++r)
        if (new_lens[r] > 0) {
            // a decode query sees its cached tokens and itself; its own part starts behind the unit's
            const int64_t own = (static_cast<int64_t>(prefix[r]) + new_lens[r] + 31) / 32 - req_shared_len[r] / 32;
            tiles += own;
            own_max = std::max(own_max, own);
        }
    shared->planned_tiles = static_cast<int32_t>(std::min<int64_t>(tiles, INT32_MAX));
    shared->max_own_tiles = static_cast<int32_t>(std::max<int64_t>(own_max, 1));
    shared->max_unit_tiles = static_cast<int32_t>(unit_max);
    return EMM_OK;
}

static emm_status check_pages_args(const void* k_cache, const void* v_cache, const void* staging,
                                   const int32_t* page_ids, int32_t n, int32_t num_pages, int64_t page_bytes,
                                   const void* c0, const void* c1, const void* c2)
{
    if (n < 0 || num_pages < 0 || page_bytes < 16 || page_bytes % 16 != 0 || page_bytes > (1 << 20))
        return EMM_ERR_INVALID_ARG;
    if (n == 0) return EMM_OK;
    if (k_cache == nullptr || v_cache == nullptr || staging == nullptr || page_ids == nullptr) return EMM_ERR_NULL;
    if (num_pages == 0) return EMM_ERR_INVALID_ARG;
    if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(staging)) return EMM_ERR_INVALID_ARG;
    for (const void* c : {c0, c1, c2})
        if (c != nullptr && (reinterpret_cast<uintptr_t>(c) & 3u) != 0) return EMM_ERR_INVALID_ARG;
    return EMM_OK;
}

emm_status emm_kv_pages_pack(const void* k_cache, const void* v_cache, int32_t num_pages, int64_t page_bytes,
                             const int32_t* page_ids, int32_t n, void* staging, uint32_t* checksums, void* hip_stream)
{
    const emm_status st = check_pages_args(k_cache, v_cache, staging, page_ids, n, num_pages, page_bytes, checksums,
                                           nullptr, nullptr);
    if (st != EMM_OK || n == 0) return st;
    const hipError_t err = emm::launch_kv_pages(false, const_cast<void*>(k_cache), const_cast<void*>(v_cache), staging,
                                                page_ids, n, num_pages, page_bytes, checksums, nullptr, nullptr,
                                                static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? EMM_OK : EMM_ERR_LAUNCH;
}

emm_status emm_kv_pages_unpack(const void* staging, const int32_t* page_ids, int32_t n, void* k_cache, void* v_cache,
                               int32_t num_pages, int64_t page_bytes, uint32_t* checksums, const uint32_t* expected,
                               uint32_t* mismatches, void* hip_stream)
{
    const emm_status st = check_pages_args(k_cache, v_cache, staging, page_ids, n, num_pages, page_bytes, checksums,
                                           expected, mismatches);
    if (st != EMM_OK || n == 0) return st;
    const hipError_t err = emm::launch_kv_pages(true, k_cache, v_cache, const_cast<void*>(staging), page_ids, n, num_pages,
                                                page_bytes, checksums, expected, mismatches,
                                                static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? EMM_OK : EMM_ERR_LAUNCH;
}

emm_status emm_cross_attn(const emm_batch* b, const void* q, const void* k_cache, const void* v_cache,
                          void* out, float* lse, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return attention(b, q, k_cache, v_cache, out, lse, workspace, workspace_bytes, hip_stream, 0);
}

emm_status emm_validate_batch_host(const emm_batch* b, const int32_t* pt, const int32_t* prefix,
                                   const int32_t* new_lens, const int32_t* cu, int causal)
{
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    if (b->num_reqs == 0) return EMM_OK;
    if (pt == nullptr || prefix == nullptr || new_lens == nullptr || cu == nullptr) return EMM_ERR_NULL;
    if (cu[0] != 0) return EMM_ERR_INVALID_ARG;
    std::vector<int32_t> writers(static_cast<size_t>(b->num_pages), 0);
    int32_t max_new = 0;
    for (int r = 0; r < b->num_reqs; ++r) {
        if (prefix[r] < 0 || new_lens[r] < 0) return EMM_ERR_INVALID_ARG;
        if (cu[r + 1] - cu[r] != new_lens[r]) return EMM_ERR_INVALID_ARG;
        if (new_lens[r] > max_new) max_new = new_lens[r];
        const int64_t ctx = static_cast<int64_t>(prefix[r]) + (causal ? new_lens[r] : 0);
        const int64_t pages = (ctx + b->page_size - 1) / b->page_size;
        if (pages > b->max_pages_per_req) return EMM_ERR_INVALID_ARG;
        for (int64_t lp = 0; lp < pages; ++lp) {
            const int32_t pg = pt[static_cast<int64_t>(r) * b->max_pages_per_req + lp];
            if (pg < 0 || pg >= b->num_pages) return EMM_ERR_INVALID_ARG;
        }
        if (causal && new_lens[r] > 0) {
            // pages that receive new tokens: written by this request, so no one else may reference them
            for (int64_t lp = prefix[r] / b->page_size; lp < pages; ++lp)
                writers[static_cast<size_t>(pt[static_cast<int64_t>(r) * b->max_pages_per_req + lp])] += 1;
        }
    }
    if (cu[b->num_reqs] != b->total_new_tokens || max_new != b->max_new_len) return EMM_ERR_INVALID_ARG;
    if (causal) {
        // a written page may be referenced only by its writer
        std::vector<int32_t> refs(static_cast<size_t>(b->num_pages), 0);
        for (int r = 0; r < b->num_reqs; ++r) {
            const int64_t ctx = static_cast<int64_t>(prefix[r]) + new_lens[r];
            const int64_t pages = (ctx + b->page_size - 1) / b->page_size;
            for (int64_t lp = 0; lp < pages; ++lp)
                refs[static_cast<size_t>(pt[static_cast<int64_t>(r) * b->max_pages_per_req + lp])] += 1;
        }
        for (int32_t pg = 0; pg < b->num_pages; ++pg)
            if (writers[static_cast<size_t>(pg)] > 0 && refs[static_cast<size_t>(pg)] != 1)
                return EMM_ERR_INVALID_ARG;
    }
    return EMM_OK;
}

emm_status emm_prefill_plan_host(const emm_batch* b, const int32_t* new_lens, int with_workspace, emm_prefill_plan* plan)
{
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    st = check_supported(b);
    if (st != EMM_OK) return st;
    if (b->dtype != EMM_BF16) return EMM_ERR_UNSUPPORTED;
    if (plan == nullptr || (b->num_reqs > 0 && new_lens == nullptr)) return EMM_ERR_NULL;
    *plan = emm_prefill_plan{};
    if (b->num_reqs == 0 || b->total_new_tokens == 0) return EMM_OK;
    int32_t shape[6];
    long long grid = 0;
    emm::attn_bf16_d128_plan_host(view_of(b), new_lens, with_workspace != 0, shape, &grid, plan->units, plan->pieces,
                                  plan->uneven_k, plan->rows_only);
    plan->fan = shape[0];
    plan->n_row_tiles = shape[1];
    plan->pairs_per_xcd = shape[2];
    plan->cutting = shape[3];
    plan->uneven = shape[4];
    plan->slots_per_xcd = shape[5];
    plan->grid = grid;
    return EMM_OK;
}

const char* emm_status_string(emm_status s)
{
    switch (s) {
        case EMM_OK: return "ok";
        case EMM_ERR_NULL: return "required pointer is null";
        case EMM_ERR_INVALID_ARG: return "invalid argument";
        case EMM_ERR_UNSUPPORTED: return "unsupported dtype / head_dim / page_size";
        case EMM_ERR_WORKSPACE: return "workspace too small";
        case EMM_ERR_LAUNCH: return "HIP launch failed";
        case EMM_ERR_NO_SPACE: return "no free or evictable page left";
        case EMM_ERR_NOT_FOUND: return "unknown request id";
    }
    return "unknown status";
}

int emm_version(void) { return kVersion; }

}  // extern "C"
