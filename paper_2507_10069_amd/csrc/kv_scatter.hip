// KV scatter: the new tokens' K/V rows go to the pool slots that follow each request's cached
// prefix (Section 2.2 of the paper: prefill yields the KV cache of every input token; the copy
// must be exact in the sense of Appendix B.5).
//
// Pure data movement, HBM bound: 4 * T * Hkv * d * elt bytes (read K,V + write K,V).  One lane
// moves one 16-byte chunk of a K row and the matching chunk of the V row.  The packed source
// [T][Hkv][d] is read fully coalesced; a (token, head) row of d*elt bytes lands contiguously in
// its page, so each group of row_bytes/16 lanes writes one contiguous run.
#include "emm_internal.h"

namespace emm {

namespace {

__global__ __launch_bounds__(256) void kv_scatter_kernel(BatchView b, const uint4* __restrict__ k_new,
                                                         const uint4* __restrict__ v_new,
                                                         uint4* __restrict__ k_cache, uint4* __restrict__ v_cache,
                                                         int chunks_per_row, long long total_chunks)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= total_chunks) return;
    const long long row = idx / chunks_per_row;          // (token, kv head)
    const int chunk = (int)(idx - row * chunks_per_row);
    const int t = (int)(row / b.num_kv_heads);
    const int h = (int)(row - (long long)t * b.num_kv_heads);

    // request that owns packed token t: last r with cu[r] <= t
    int lo = 0, hi = b.num_reqs;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (b.cu_new_lens[mid] <= t) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int pos = b.prefix_lens[r] + (t - b.cu_new_lens[r]);
    const int page = b.page_table[(long long)r * b.max_pages + (pos >> (4 + b.page_shift))];
    if (page < 0 || page >= b.num_pages) return;         // corrupt table: drop the write, never stray

    const long long dst = (((long long)page * b.num_kv_heads + h) * b.page_size + (pos & (b.page_size - 1))) * chunks_per_row + chunk;
    k_cache[dst] = k_new[idx];
    v_cache[dst] = v_new[idx];
}

}  // namespace

hipError_t launch_kv_scatter(const BatchView& b, const void* k_new, const void* v_new, void* k_cache,
                             void* v_cache, int elt_bytes, hipStream_t stream)
{
    const int chunks_per_row = b.head_dim * elt_bytes / 16;
    const long long total = (long long)b.total_new_tokens * b.num_kv_heads * chunks_per_row;
    if (total == 0) return hipSuccess;
    const long long blocks = (total + 255) / 256;
    hipLaunchKernelGGL(kv_scatter_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, b,
                       (const uint4*)k_new, (const uint4*)v_new, (uint4*)k_cache, (uint4*)v_cache,
                       chunks_per_row, total);
    return hipGetLastError();
}

}  // namespace emm
