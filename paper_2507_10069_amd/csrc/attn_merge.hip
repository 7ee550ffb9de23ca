// Merging two attention results of the same query rows over DISJOINT key sets (bf16, head_dim 128), for gfx950.
//
// Prefill with shared prefixes (Section 3.3 of the paper: requests repeat system prompts, images and videos, so
// several requests of a prefill batch hold the same physical pages at the head of their page tables) is done
// in two attention passes: one over the shared keys, with the query rows of all the requests of a sharing group
// packed into common row tiles, and one over each request's own remaining keys.  Softmax attention over a union
// of key sets is the convex combination of the parts' results with weights exp(lse_part - lse_all), which this
// kernel forms, row by row:
//     out = (e^{lse_a} out_a + e^{lse_b} out_b) / (e^{lse_a} + e^{lse_b}),   lse = log(e^{lse_a} + e^{lse_b}).
// Rows of requests that are in no sharing group have no first part and stay as they are.
//
// Pure data movement, HBM bound: per row two 256-byte reads, one 256-byte write and three floats.  A row is done
// by 16 lanes (8 channels, 16 bytes each), a workgroup does 16 rows.
#include "emm_internal.h"

namespace emm {

namespace {

constexpr int THREADS = 256;
constexpr int D = 128;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// the request that packed token t belongs to: the last r with cu_new_lens[r] <= t among requests that have tokens
// (binary search; what the array holds is forced into range wherever an index depends on it)
__device__ inline int request_of_token(const BatchView& b, int t)
{
    int lo = 0, hi = b.num_reqs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (b.cu_new_lens[mid] <= t) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

__global__ __launch_bounds__(THREADS) void attn_merge_parts_kernel(BatchView b, const int32_t* __restrict__ req_shared_len,
                                                                   const __bf16* __restrict__ out_shared,
                                                                   const float* __restrict__ lse_shared,
                                                                   const float* __restrict__ lse_own, __bf16* __restrict__ out,
                                                                   float* __restrict__ lse)
{
    const long long n_rows = (long long)b.total_new_tokens * b.num_q_heads;
    const long long row = (long long)blockIdx.x * (THREADS / 16) + (threadIdx.x >> 4);
    if (row >= n_rows) return;
    const int t = (int)(row / b.num_q_heads);
    const int r = request_of_token(b, t);
    const float lo = lse_own[row];
    const bool member = req_shared_len[r] > 0;
    float merged = lo;
    if (member) {
        const float ls = lse_shared[row];
        const float m = fmaxf(ls, lo);
        if (m > -INFINITY) {
            const float ws = __expf(ls - m), wo = __expf(lo - m);
            const float inv = 1.f / (ws + wo);
            const long long at = row * D + (threadIdx.x & 15) * 8;
            const bf16x8 a = *(const bf16x8*)(out_shared + at);
            const bf16x8 c = *(const bf16x8*)(out + at);
            bf16x8 o;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[i] = (__bf16)(((float)a[i] * ws + (float)c[i] * wo) * inv);
            *(bf16x8*)(out + at) = o;
            merged = m + __logf(ws + wo);
        }
    }
    if (lse != nullptr && (threadIdx.x & 15) == 0) lse[row] = merged;
}

}  // namespace

hipError_t launch_attn_merge_parts(const BatchView& b, const int32_t* req_shared_len, const void* out_shared,
                                   const float* lse_shared, const float* lse_own, void* out, float* lse, hipStream_t stream)
{
    const long long n_rows = (long long)b.total_new_tokens * b.num_q_heads;
    if (n_rows == 0 || b.num_reqs == 0) return hipSuccess;
    const long long grid = (n_rows + THREADS / 16 - 1) / (THREADS / 16);
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attn_merge_parts_kernel, dim3((unsigned)grid), dim3(THREADS), 0, stream, b, req_shared_len,
                       (const __bf16*)out_shared, lse_shared, lse_own, (__bf16*)out, lse);
    return hipGetLastError();
}

}  // namespace emm
