// Internal declarations shared by the translation units of the HIP library.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace emm {

// Everything a device kernel needs to know about a batch (a by-value copy of the public
// descriptor plus tensor pointers).
struct BatchView {
    const int32_t* page_table;   // [B][max_pages]
    const int32_t* prefix_lens;  // [B]
    const int32_t* new_lens;     // [B]
    const int32_t* cu_new_lens;  // [B+1]
    int32_t num_reqs, num_q_heads, num_kv_heads, head_dim;
    int32_t page_size, num_pages, max_pages, total_new_tokens, max_new_len;
    int32_t page_shift;          // page_size == 16 << page_shift: a page is 2^page_shift blocks of 16 tokens
    float softmax_scale;
};

// The batch's lengths as the kernels use them.  The arrays live in device memory, where the host cannot check
// them; whatever they hold (a caller's bug, freed memory), the values below keep every address the kernels form
// inside the caller's buffers.  A consistent batch passes through unchanged.
//   new tokens of request r: 0 .. max_new_len, at most T, and (causal: they have slots) at most what a row of
//   the page table can hold
__device__ inline int safe_new_len(const BatchView& b, int r, bool causal)
{
    int n = min(max(b.new_lens[r], 0), min(b.max_new_len, b.total_new_tokens));
    if (causal) n = (int)min((long long)n, (long long)b.max_pages * b.page_size);
    return n;
}
//   cached tokens: what fits the page-table row next to n_slots more tokens (the new ones if causal, else 0)
__device__ inline int safe_prefix_len(const BatchView& b, int r, int n_slots)
{
    const long long room = (long long)b.max_pages * b.page_size - n_slots;
    return (int)min((long long)max(b.prefix_lens[r], 0), max(room, 0ll));
}
//   first packed row: such that n_new rows from it on lie inside [0, T)
__device__ inline int safe_first_row(const BatchView& b, int r, int n_new)
{
    return min(max(b.cu_new_lens[r], 0), max(b.total_new_tokens - n_new, 0));
}

struct AttnArgs {
    BatchView b;
    const void* q;        // [T][H][d]
    const void* k_cache;  // [num_pages][Hkv][page_size][d]
    const void* v_cache;
    void* out;            // [T][H][d]
    float* lse;           // [T][H] or nullptr
    int32_t causal;       // 1: keys 0..P+j ; 0: keys 0..P-1
    void* workspace;      // scratch for the bf16 kernel's cut units, or nullptr
    const void* k_new = nullptr;   // fused decode step only: the query tokens' own K/V rows [T][Hkv][d], which
    const void* v_new = nullptr;   // the kernel reads from here and stores in the (then writable) pools
};

// Shared-prefix units of a decode batch (device arrays; see emm_shared_prefix in emm.h)
struct SharedPrefixView {
    const int32_t* unit_first_req;   // [U]
    const int32_t* unit_num_reqs;    // [U]
    const int32_t* unit_shared_len;  // [U] multiple of 32
    const int32_t* req_unit;         // [B] or -1
    const int32_t* req_shared_len;   // [B] or 0
    int32_t num_units;
    int32_t planned_tiles;           // host hint: 32-key tiles per KV head over the whole batch, 0 = unknown
    int32_t max_own_tiles;           // bound on a request's own part in tiles, 0 = the page table's width
    int32_t max_unit_tiles;          // bound on a unit's shared part in tiles, 0 = the page table's width
};

// Each launcher enqueues on `stream` and returns the launch status.
hipError_t launch_kv_scatter(const BatchView& b, const void* k_new, const void* v_new, void* k_cache,
                             void* v_cache, int elt_bytes, hipStream_t stream);
hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t stream);
hipError_t launch_attn_bf16_d128(const AttnArgs& a, hipStream_t stream);
size_t attn_bf16_d128_workspace_bytes(const BatchView& b);   // what launch_attn_bf16_d128 wants behind AttnArgs::workspace
// host only: how launch_attn_bf16_d128 would lay the batch out (new_lens: host copy); arrays of 8 are per XCD
void attn_bf16_d128_plan_host(const BatchView& b, const int32_t* new_lens, bool has_workspace, int32_t* shape6, long long* grid,
                              int32_t* units, int32_t* pieces, int32_t* uneven_k, int32_t* rows_only);
// decode step (every request has at most one query token, at most 16 query heads per KV head)
bool attn_bf16_decode_applies(const BatchView& b);
size_t attn_bf16_decode_workspace_bytes(const BatchView& b);
hipError_t launch_attn_bf16_decode(const AttnArgs& a, hipStream_t stream);
// the same with the piece records in the library's own fixed device array (no workspace of the caller's); fails with
// hipErrorInvalidValue when the batch needs more than attn_bf16_decode_static_scratch_bytes()
size_t attn_bf16_decode_static_scratch_bytes();
hipError_t launch_attn_bf16_decode_static(AttnArgs a, hipStream_t stream);
// the same with shared-prefix units (sv.num_units >= 1)
size_t attn_bf16_decode_shared_workspace_bytes(const BatchView& b, const SharedPrefixView& sv);
hipError_t launch_attn_bf16_decode_shared(const AttnArgs& a, const SharedPrefixView& sv, hipStream_t stream);
// the same, fused with the scatter of the query tokens' own K/V rows (a.k_new, a.v_new; pools writable; causal)
hipError_t launch_attn_bf16_decode_step(const AttnArgs& a, const SharedPrefixView& sv, hipStream_t stream);

// merge of two attention results of the same rows over disjoint key sets (prefill with shared prefixes): out and lse
// hold the second part on entry and the merged result on return; rows of requests with req_shared_len <= 0 stay
hipError_t launch_attn_merge_parts(const BatchView& b, const int32_t* req_shared_len, const void* out_shared,
                                   const float* lse_shared, const float* lse_own, void* out, float* lse, hipStream_t stream);

// KV page migration: pack (pools -> staging) or unpack (staging -> pools) n pages with a checksum per page
hipError_t launch_kv_pages(bool unpack, void* k_cache, void* v_cache, void* staging, const int32_t* page_ids, int n,
                           int num_pages, long long page_bytes, uint32_t* checksums, const uint32_t* expected,
                           uint32_t* mismatches, hipStream_t stream);

}  // namespace emm
