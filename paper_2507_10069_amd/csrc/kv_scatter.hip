// KV scatter: the new tokens' K/V rows go to the pool slots that follow each request's cached
// prefix (Section 2.2 of the paper: prefill yields the KV cache of every input token; the copy
// must be exact in the sense of Appendix B.5).
//
// Pure data movement, HBM bound: 4 * T * Hkv * d * elt bytes (read K,V + write K,V).  One wave moves one
// token: finding its request (a search over the batch's offsets) and its page is wave-uniform work done once
// on the scalar unit, and the lanes move the token's K row and V row (all KV heads, Hkv * d * elt bytes each)
// in 16-byte chunks.  The packed source [T][Hkv][d] is read fully coalesced; a (token, head) row of d*elt
// bytes lands contiguously in its page.
#include "emm_internal.h"

namespace emm {

namespace {

constexpr int WAVES = 4;                                 // tokens per workgroup

// row_shift: a (token, head) row is 1 << row_shift chunks of 16 bytes (head_dim * element size / 16)
__global__ __launch_bounds__(64 * WAVES) void kv_scatter_kernel(BatchView b, const uint4* __restrict__ k_new,
                                                                const uint4* __restrict__ v_new,
                                                                uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                                int row_shift)
{
    const int t = blockIdx.x * WAVES + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // packed token, wave-uniform
    if (t >= b.total_new_tokens) return;
    const int lane = threadIdx.x & 63;

    // request that owns packed token t: last r with cu[r] <= t
    int lo = 0, hi = b.num_reqs;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (b.cu_new_lens[mid] <= t) lo = mid; else hi = mid;
    }
    const int r = lo;
    const long long pos64 = (long long)b.prefix_lens[r] + (t - b.cu_new_lens[r]);
    // inconsistent lengths or a corrupt table: drop the write, never stray
    if (pos64 < 0 || pos64 >= (long long)b.max_pages * b.page_size) return;
    const int pos = (int)pos64;
    const int page = b.page_table[(long long)r * b.max_pages + (pos >> (4 + b.page_shift))];
    if (page < 0 || page >= b.num_pages) return;

    const int token_chunks = b.num_kv_heads << row_shift;                 // chunks of the token's K (or V) row, all heads
    const long long src = (long long)t * token_chunks;
    // chunk c of the token is chunk c % row of head c / row; heads are page_size rows apart in the pool
    const long long dst = ((long long)page * b.num_kv_heads * b.page_size + (pos & (b.page_size - 1))) << row_shift;
    const int head_stride = (b.page_size - 1) << row_shift;               // extra chunks between consecutive heads
    for (int c = lane; c < token_chunks; c += 64) {
        const long long d = dst + c + (long long)(c >> row_shift) * head_stride;
        k_cache[d] = k_new[src + c];
        v_cache[d] = v_new[src + c];
    }
}

}  // namespace

hipError_t launch_kv_scatter(const BatchView& b, const void* k_new, const void* v_new, void* k_cache,
                             void* v_cache, int elt_bytes, hipStream_t stream)
{
    if (b.total_new_tokens == 0 || b.num_reqs == 0) return hipSuccess;
    const int chunks_per_row = b.head_dim * elt_bytes / 16;              // 8, 16 or 32: a power of two
    int row_shift = 0;
    while ((1 << row_shift) < chunks_per_row) ++row_shift;
    if ((1 << row_shift) != chunks_per_row) return hipErrorInvalidValue;
    const long long blocks = ((long long)b.total_new_tokens + WAVES - 1) / WAVES;
    hipLaunchKernelGGL(kv_scatter_kernel, dim3((unsigned)blocks), dim3(64 * WAVES), 0, stream, b,
                       (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache, (uint4*)v_cache, row_shift);
    return hipGetLastError();
}

}  // namespace emm
