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

// ---- prefill with shared prefixes: the shared keys once per sharing group, each request's own keys, then the merge

namespace {

size_t align256(size_t n) { return (n + 255) & ~static_cast<size_t>(255); }

// do the two descriptors describe the two passes of one batch?
emm_status check_shared_pair(const emm_batch* groups, const emm_batch* own)
{
    emm_status st = check_scalars(groups);
    if (st != EMM_OK) return st;
    st = check_scalars(own);
    if (st != EMM_OK) return st;
    st = check_supported(own);
    if (st != EMM_OK) return st;
    if (own->dtype != EMM_BF16 || groups->dtype != EMM_BF16) return EMM_ERR_UNSUPPORTED;
    if (groups->num_q_heads != own->num_q_heads || groups->num_kv_heads != own->num_kv_heads || groups->head_dim != own->head_dim ||
        groups->page_size != own->page_size || groups->num_pages != own->num_pages || groups->softmax_scale != own->softmax_scale ||
        groups->total_new_tokens != own->total_new_tokens || groups->num_reqs > own->num_reqs)
        return EMM_ERR_INVALID_ARG;
    return EMM_OK;
}

struct SharedWorkspace {
    size_t out_shared, lse_shared, lse_own, inner, inner_bytes, total;
};

emm_status shared_workspace(const emm_batch* groups, const emm_batch* own, SharedWorkspace* w)
{
    const size_t rows = static_cast<size_t>(own->total_new_tokens) * own->num_q_heads;
    size_t a = 0, c = 0;
    emm_status st = emm_prefill_attn_workspace_size(groups, &a);
    if (st != EMM_OK) return st;
    st = emm_prefill_attn_workspace_size(own, &c);
    if (st != EMM_OK) return st;
    w->out_shared = 0;
    w->lse_shared = align256(rows * own->head_dim * 2);
    w->lse_own = w->lse_shared + align256(rows * 4);
    w->inner = w->lse_own + align256(rows * 4);
    w->inner_bytes = std::max(a, c);                         // the two attention passes run one after the other
    w->total = w->inner + align256(w->inner_bytes);
    return EMM_OK;
}

}  // namespace

extern "C" emm_status emm_prefill_attn_shared_workspace_size(const emm_batch* groups, const emm_batch* own, size_t* bytes)
{
    if (bytes == nullptr) return EMM_ERR_NULL;
    *bytes = 0;
    emm_status st = check_shared_pair(groups, own);
    if (st != EMM_OK) return st;
    SharedWorkspace w;
    st = shared_workspace(groups, own, &w);
    if (st != EMM_OK) return st;
    *bytes = w.total;
    return EMM_OK;
}

extern "C" emm_status emm_prefill_attn_shared(const emm_batch* groups, const emm_batch* own, const int32_t* req_shared_len,
                                               const void* q, const void* k_cache, const void* v_cache, void* out, float* lse,
                                               void* workspace, size_t workspace_bytes, void* hip_stream)
{
    emm_status st = check_shared_pair(groups, own);
    if (st != EMM_OK) return st;
    SharedWorkspace w;
    st = shared_workspace(groups, own, &w);
    if (st != EMM_OK) return st;
    if (own->num_reqs == 0 || own->total_new_tokens == 0) return EMM_OK;
    if (req_shared_len == nullptr || workspace == nullptr) return EMM_ERR_NULL;
    if (workspace_bytes < w.total) return EMM_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return EMM_ERR_INVALID_ARG;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    float* lse_own = reinterpret_cast<float*>(ws + w.lse_own);
    void* inner = w.inner_bytes > 0 ? ws + w.inner : nullptr;
    // 1. every group's rows over the group's shared keys: no mask (all of them precede every new token), rows of all
    //    members packed into common row tiles
    if (groups->num_reqs > 0) {
        st = attention(groups, q, k_cache, v_cache, ws + w.out_shared, reinterpret_cast<float*>(ws + w.lse_shared), inner,
                       w.inner_bytes, hip_stream, 0);
        if (st != EMM_OK) return st;
    }
    // 2. every request over its own keys (what its page table holds behind the shared part), causal
    st = attention(own, q, k_cache, v_cache, out, lse_own, inner, w.inner_bytes, hip_stream, 1);
    if (st != EMM_OK) return st;
    // 3. the members' rows: both parts into one
    const hipError_t err = emm::launch_attn_merge_parts(view_of(own), req_shared_len, ws + w.out_shared,
                                                        reinterpret_cast<const float*>(ws + w.lse_shared), lse_own, out, lse,
                                                        static_cast<hipStream_t>(hip_stream));
    return err == hipSuccess ? EMM_OK : EMM_ERR_LAUNCH;
}

extern "C" emm_status emm_prefill_shared_plan_host(const emm_batch* b, const int32_t* pt, const int32_t* prefix,
                                                    const int32_t* new_lens, const int32_t* cu, int32_t min_shared_tokens,
                                                    int64_t min_saved_key_tiles, emm_prefill_shared_plan* plan)
{
    emm_status st = check_scalars(b);
    if (st != EMM_OK) return st;
    st = check_supported(b);                                  // page sizes that divide, or are divided by, a key tile
    if (st != EMM_OK) return st;
    if (plan == nullptr) return EMM_ERR_NULL;
    plan->num_groups = 0;
    plan->rows_tiles_plain = plan->rows_tiles_shared = 0;
    plan->key_tiles_plain = plan->key_tiles_shared = 0;
    plan->groups = *b;
    plan->own = *b;
    plan->groups.page_table = plan->groups.prefix_lens = plan->groups.new_lens = plan->groups.cu_new_lens = nullptr;
    plan->own.page_table = plan->own.prefix_lens = plan->own.new_lens = plan->own.cu_new_lens = nullptr;
    plan->groups.num_reqs = 0;
    plan->groups.max_new_len = 0;
    if (b->num_reqs == 0) return EMM_OK;
    if (pt == nullptr || prefix == nullptr || new_lens == nullptr || cu == nullptr || plan->req_shared_len == nullptr ||
        plan->group_page_table == nullptr || plan->group_prefix_lens == nullptr || plan->group_new_lens == nullptr ||
        plan->group_cu_new_lens == nullptr || plan->own_page_table == nullptr || plan->own_prefix_lens == nullptr)
        return EMM_ERR_NULL;
    const int B = b->num_reqs, ps = b->page_size, G = b->num_q_heads / b->num_kv_heads;
    const int64_t mp = b->max_pages_per_req;
    const int64_t floor_len = std::max<int64_t>(min_shared_tokens, 64);
    auto tiles = [&](int64_t n_new) { return (n_new * G + 255) / 256; };       // row tiles of 256 rows per KV head
    // tokens that requests i and j share: leading equal page-table entries, as far as both requests' cached tokens
    // fill the page
    auto common = [&](int i, int j) -> int64_t {
        const int64_t full = std::min(prefix[i], prefix[j]) / ps;
        const int32_t* x = pt + static_cast<int64_t>(i) * mp;
        const int32_t* y = pt + static_cast<int64_t>(j) * mp;
        int64_t p = 0;
        while (p < full && p < mp && x[p] == y[p]) ++p;
        return p * ps;
    };
    int NG = 0;
    int64_t plain = 0, shared_tiles = 0;
    std::vector<int> group_first(static_cast<size_t>(B) / 2 + 1);
    for (int r = 0; r < B; ++r) plan->req_shared_len[r] = 0;
    for (int i = 0; i < B;) {
        int n = 1;
        int64_t S = 0, sum_new = new_lens[i], before = tiles(new_lens[i]);
        if (new_lens[i] > 0) {
            int64_t cur = INT64_MAX;
            for (int j = i + 1; j < B && new_lens[j] > 0; ++j) {
                const int64_t cand = std::min(cur, common(i, j)) / 64 * 64;     // whole key tiles
                if (cand < floor_len) break;
                // what a group saves: row tiles (the packed rows need fewer than the members' own) times the keys they
                // no longer stream; one more member must not lower that
                const int64_t saved_now = (before - tiles(sum_new)) * S;
                const int64_t saved_then = (before + tiles(new_lens[j]) - tiles(sum_new + new_lens[j])) * cand;
                if (n > 1 && saved_then < saved_now) break;
                cur = S = cand;
                sum_new += new_lens[j];
                before += tiles(new_lens[j]);
                ++n;
            }
        }
        const bool pays = n >= 2 && tiles(sum_new) < before;
        if (pays) {
            for (int r = i; r < i + n; ++r) plan->req_shared_len[r] = static_cast<int32_t>(S);
            group_first[NG] = i;
            plan->group_prefix_lens[NG] = static_cast<int32_t>(S);
            plan->group_new_lens[NG] = static_cast<int32_t>(sum_new);
            plan->group_cu_new_lens[NG] = cu[i];
            plan->groups.max_new_len = std::max<int32_t>(plan->groups.max_new_len, static_cast<int32_t>(sum_new));
            shared_tiles += tiles(sum_new);
            ++NG;
        } else {
            n = 1;
        }
        for (int r = i; r < i + n; ++r) plain += tiles(new_lens[r]);
        i += n;
    }
    // 64-key tiles that the batch's work units stream (per KV head a request has tiles(new) units, each over the
    // request's whole context, taken as prefix + new for all of them), without the groups and with them
    int64_t keys_plain = 0, keys_shared = 0;
    for (int r = 0; r < B; ++r) {
        const int64_t ctx = static_cast<int64_t>(prefix[r]) + new_lens[r], S = plan->req_shared_len[r];
        keys_plain += tiles(new_lens[r]) * ((ctx + 63) / 64);
        keys_shared += tiles(new_lens[r]) * ((ctx - S + 63) / 64);
    }
    for (int g = 0; g < NG; ++g) keys_shared += tiles(plan->group_new_lens[g]) * (plan->group_prefix_lens[g] / 64);
    plan->key_tiles_plain = keys_plain * b->num_kv_heads;
    plan->key_tiles_shared = keys_shared * b->num_kv_heads;
    if (min_saved_key_tiles < 0) min_saved_key_tiles = EMM_PREFILL_SHARED_MIN_SAVED_KEY_TILES;
    if (NG > 0 && plan->key_tiles_plain - plan->key_tiles_shared < min_saved_key_tiles) {
        // not worth two more launches and a second pass over the outputs
        NG = 0;
        plan->groups.max_new_len = 0;
        for (int r = 0; r < B; ++r) plan->req_shared_len[r] = 0;
    }
    plan->group_cu_new_lens[NG] = b->total_new_tokens;
    // The two page tables are packed as narrow as what they hold allows (the descriptors' max_pages_per_req is their
    // row stride): the launches size their grids and decide about cutting along the keys from that width.
    //   groups: the shared pages of the longest shared part
    int64_t wg = 1;
    for (int g = 0; g < NG; ++g) wg = std::max<int64_t>(wg, plan->group_prefix_lens[g] / ps);
    wg = std::min(wg, std::max<int64_t>(mp, 1));
    for (int g = 0; g < NG; ++g) {
        const int32_t* src = pt + static_cast<int64_t>(group_first[g]) * mp;
        for (int64_t p = 0; p < wg; ++p) plan->group_page_table[g * wg + p] = p < mp ? src[p] : -1;
    }
    plan->groups.max_pages_per_req = static_cast<int32_t>(wg);
    //   own: every request's row moved left by the pages of its shared part, as wide as the longest own part
    int64_t wo = 1;
    for (int r = 0; r < B; ++r)
        wo = std::max<int64_t>(wo, (static_cast<int64_t>(prefix[r]) - plan->req_shared_len[r] + new_lens[r] + ps - 1) / ps);
    wo = std::min(wo, std::max<int64_t>(mp, 1));
    for (int r = 0; r < B; ++r) {
        const int64_t skip = plan->req_shared_len[r] / ps;
        int32_t* row = plan->own_page_table + static_cast<int64_t>(r) * wo;
        const int32_t* src = pt + static_cast<int64_t>(r) * mp;
        for (int64_t p = 0; p < wo; ++p) row[p] = p + skip < mp ? src[p + skip] : -1;
        plan->own_prefix_lens[r] = prefix[r] - plan->req_shared_len[r];
    }
    plan->own.max_pages_per_req = static_cast<int32_t>(wo);
    plan->num_groups = NG;
    plan->groups.num_reqs = NG;
    plan->rows_tiles_plain = plain;
    plan->rows_tiles_shared = shared_tiles;
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
