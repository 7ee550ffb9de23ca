// Plain fp32 attention over the paged pool: one 64-lane wave per (query token, query head) row.
//
// This is the fp32 path of the library (small correctness configurations, head_dim 64 or 128).
// It follows the same definition as the MFMA kernel -- causal over absolute positions for the
// prefix-cached prefill (Section 3.3 / Appendix B.7 of the paper), unmasked for cross-attention
// (Section 2.1) -- with an online softmax over chunks of 64 keys: lanes own keys for the score
// phase and channels for the value phase.  It is latency bound and makes no roofline claim.
#include "emm_internal.h"

namespace emm {

namespace {

__device__ inline float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

__device__ inline float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

template <int D>
__global__ __launch_bounds__(256) void attn_f32_kernel(AttnArgs a)
{
    constexpr int CPL = D / 64;                       // channels per lane in the value phase
    const BatchView& b = a.b;
    const int lane = threadIdx.x & 63;
    const long long row = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (long long)b.total_new_tokens * b.num_q_heads) return;   // no block barrier below
    const int t = (int)(row / b.num_q_heads);
    const int h = (int)(row - (long long)t * b.num_q_heads);
    const int kvh = h / (b.num_q_heads / b.num_kv_heads);

    int lo = 0, hi = b.num_reqs;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (b.cu_new_lens[mid] <= t) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int j = t - b.cu_new_lens[r];
    const int P = b.prefix_lens[r];
    // (forced into what the page-table row can hold, whatever the arrays say: no access leaves the caller's buffers)
    const int len = (int)min(max(a.causal ? (long long)P + j + 1 : (long long)P, 0ll), (long long)b.max_pages * b.page_size);

    const float* __restrict__ q = (const float*)a.q + ((long long)t * b.num_q_heads + h) * D;
    const float* __restrict__ kc = (const float*)a.k_cache;
    const float* __restrict__ vc = (const float*)a.v_cache;
    const int32_t* __restrict__ pt = b.page_table + (long long)r * b.max_pages;

    const int pg_log2 = 4 + b.page_shift, ps = b.page_size;
    float m = -INFINITY, l = 0.f;
    float acc[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) acc[c] = 0.f;

    for (int base = 0; base < len; base += 64) {
        const int i = base + lane;
        float s = -INFINITY;
        int my_page = 0;                                 // page of key base + lane; the value phase gets it by shuffle
        if (i < len) {
            const long long page = my_page = min(max(pt[i >> pg_log2], 0), b.num_pages - 1);
            const float4* k4 = (const float4*)(kc + ((page * b.num_kv_heads + kvh) * ps + (i & (ps - 1))) * D);
            const float4* q4 = (const float4*)q;
            float dot = 0.f;
#pragma unroll 16
            for (int c = 0; c < D / 4; ++c) {
                const float4 kv = k4[c], qv = q4[c];
                dot = fmaf(qv.x, kv.x, dot);
                dot = fmaf(qv.y, kv.y, dot);
                dot = fmaf(qv.z, kv.z, dot);
                dot = fmaf(qv.w, kv.w, dot);
            }
            s = dot * b.softmax_scale;
        }
        const float m_new = fmaxf(m, wave_max(s));       // finite: key `base` is always attended
        const float p = (i < len) ? expf(s - m_new) : 0.f;
        const float alpha = expf(m - m_new);              // 0 on the first chunk (m = -inf)
        l = l * alpha + wave_sum(p);
#pragma unroll
        for (int c = 0; c < CPL; ++c) acc[c] *= alpha;
        const int n_here = min(64, len - base);
        // sixteen keys at a time: their V rows are all requested before the first is used (the page of key
        // base + kk comes from lane kk by shuffle, so no load sits in the chain that leads to a row's address);
        // keys past the chunk's end repeat its last key with weight 0
        constexpr int GROUP = 16;
        for (int kk0 = 0; kk0 < n_here; kk0 += GROUP) {
            float pk[GROUP], vv[GROUP][CPL];
#pragma unroll
            for (int u = 0; u < GROUP; ++u) {
                const int kk = min(kk0 + u, n_here - 1);
                pk[u] = kk0 + u < n_here ? __shfl(p, kk) : 0.f;
                const long long page = __shfl(my_page, kk);
                const float* v = vc + ((page * b.num_kv_heads + kvh) * ps + ((base + kk) & (ps - 1))) * D;
#pragma unroll
                for (int c = 0; c < CPL; ++c) vv[u][c] = v[lane + 64 * c];
            }
#pragma unroll
            for (int u = 0; u < GROUP; ++u)
#pragma unroll
                for (int c = 0; c < CPL; ++c) acc[c] = fmaf(pk[u], vv[u][c], acc[c]);
        }
        m = m_new;
    }

    float* __restrict__ o = (float*)a.out + ((long long)t * b.num_q_heads + h) * D;
    const float inv = (l > 0.f) ? 1.f / l : 0.f;          // no keys (cross, empty cache): zero row
#pragma unroll
    for (int c = 0; c < CPL; ++c) o[lane + 64 * c] = acc[c] * inv;
    if (a.lse != nullptr && lane == 0)
        a.lse[(long long)t * b.num_q_heads + h] = (l > 0.f) ? m + logf(l) : -INFINITY;
}

}  // namespace

hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t stream)
{
    const long long rows = (long long)a.b.total_new_tokens * a.b.num_q_heads;
    if (rows == 0) return hipSuccess;
    const unsigned blocks = (unsigned)((rows + 3) / 4);
    if (a.b.head_dim == 64)
        hipLaunchKernelGGL(attn_f32_kernel<64>, dim3(blocks), dim3(256), 0, stream, a);
    else
        hipLaunchKernelGGL(attn_f32_kernel<128>, dim3(blocks), dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace emm
