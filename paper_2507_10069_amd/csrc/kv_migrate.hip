// KV page migration primitive, the part one GPU can show (Appendix B.5 of the paper: on scaling, a request's
// KV cache moves to another instance by exact copy, verified with checksums).  pack gathers a request's pages
// from the two pools into a contiguous staging buffer -- what would be handed to the transport -- and unpack
// scatters a received staging buffer into whatever free pages the destination pool has; both take the
// Adler-32 (RFC 1950) of every page as it passes, so the two sides can be compared.
//
// Pure data movement, HBM bound: 2 * page_bytes read and written per page.  One workgroup per page; a lane
// moves 16 bytes at a time, fully coalesced on both sides (a page is contiguous in its pool and in the
// staging buffer).  The checksum rides along on the integer dot-product instruction: for the four bytes of a
// word at offset i of the n-byte page, sum(d) and sum(k * d[k]) (v_dot4_u32_u8 with constants), from which
//   A = 1 + sum over the page of d            B = n + sum over the page of (n - position) * d,  both mod 65521.
#include "emm_internal.h"

namespace emm {

namespace {

constexpr int THREADS = 256;
constexpr unsigned ADLER_MOD = 65521;

// wave sum of a 64-bit value
__device__ inline unsigned long long wave_sum_u64(unsigned long long x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const unsigned lo = __shfl_xor((unsigned)x, o, 64), hi = __shfl_xor((unsigned)(x >> 32), o, 64);
        x += ((unsigned long long)hi << 32) | lo;
    }
    return x;
}

// UNPACK = false: pools -> staging; true: staging -> pools.  page_bytes: one page of ONE pool.
template <bool UNPACK>
__global__ __launch_bounds__(THREADS) void kv_pages_kernel(unsigned char* __restrict__ k_cache,
                                                           unsigned char* __restrict__ v_cache,
                                                           unsigned char* __restrict__ staging,
                                                           const int32_t* __restrict__ page_ids, int num_pages,
                                                           long long page_bytes, uint32_t* __restrict__ checksums,
                                                           const uint32_t* __restrict__ expected,
                                                           uint32_t* __restrict__ mismatches)
{
    __shared__ unsigned long long part[2][THREADS / 64];
    const int p = blockIdx.x;
    const int page = min(max(page_ids[p], 0), num_pages - 1);             // never leaves the pool
    const long long n = 2 * page_bytes;                                   // bytes of the page in the staging buffer
    unsigned char* kp = k_cache + (long long)page * page_bytes;
    unsigned char* vp = v_cache + (long long)page * page_bytes;
    unsigned char* sp = staging + (long long)p * n;
    unsigned long long sum_d = 0, sum_w = 0;                              // sum of bytes, sum of (n - position) * byte
    constexpr int BATCH = 8;                                              // loads in flight per lane
    for (long long off0 = (long long)threadIdx.x * 16; off0 < n; off0 += (long long)BATCH * THREADS * 16) {
        uint4 w[BATCH];
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const long long off = off0 + (long long)u * THREADS * 16;
            if (off < n) {
                const unsigned char* pool = off < page_bytes ? kp + off : vp + (off - page_bytes);
                w[u] = UNPACK ? *(const uint4*)(sp + off) : *(const uint4*)pool;
            }
        }
#pragma unroll
        for (int u = 0; u < BATCH; ++u) {
            const long long off = off0 + (long long)u * THREADS * 16;
            if (off < n) {
                unsigned char* pool = off < page_bytes ? kp + off : vp + (off - page_bytes);
                *(uint4*)(UNPACK ? pool : sp + off) = w[u];
                const unsigned words[4] = {w[u].x, w[u].y, w[u].z, w[u].w};
                unsigned s_all = 0;                                       // of the 16 bytes: at most 4080
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const unsigned s = __builtin_amdgcn_udot4(words[j], 0x01010101u, 0u, false);   // d0 + d1 + d2 + d3
                    const unsigned t = __builtin_amdgcn_udot4(words[j], 0x03020100u, 0u, false);   // d1 + 2 d2 + 3 d3
                    s_all += s;
                    // one word's term fits 32 bits ((n - position) <= 2^21, s <= 1020: below 2^31.1), the four of a
                    // chunk together need not (pages above 512 KiB), so each goes into the 64-bit sum by itself
                    sum_w += (unsigned)(n - off - 4 * j) * s - t;
                }
                sum_d += s_all;
            }
        }
    }
    sum_d = wave_sum_u64(sum_d);
    sum_w = wave_sum_u64(sum_w);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        part[0][wave] = sum_d;
        part[1][wave] = sum_w;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long d = 0, w = 0;
        for (int i = 0; i < THREADS / 64; ++i) {
            d += part[0][i];
            w += part[1][i];
        }
        const unsigned a = (unsigned)((1 + d) % ADLER_MOD), b = (unsigned)(((unsigned long long)n + w) % ADLER_MOD);
        const uint32_t sum = (b << 16) | a;
        if (checksums != nullptr) checksums[p] = sum;
        if (UNPACK && expected != nullptr && mismatches != nullptr && expected[p] != sum) atomicAdd(mismatches, 1u);
    }
}

}  // namespace

hipError_t launch_kv_pages(bool unpack, void* k_cache, void* v_cache, void* staging, const int32_t* page_ids, int n,
                           int num_pages, long long page_bytes, uint32_t* checksums, const uint32_t* expected,
                           uint32_t* mismatches, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    if (unpack)
        hipLaunchKernelGGL(kv_pages_kernel<true>, dim3((unsigned)n), dim3(THREADS), 0, stream, (unsigned char*)k_cache,
                           (unsigned char*)v_cache, (unsigned char*)staging, page_ids, num_pages, page_bytes, checksums,
                           expected, mismatches);
    else
        hipLaunchKernelGGL(kv_pages_kernel<false>, dim3((unsigned)n), dim3(THREADS), 0, stream, (unsigned char*)k_cache,
                           (unsigned char*)v_cache, (unsigned char*)staging, page_ids, num_pages, page_bytes, checksums,
                           expected, mismatches);
    return hipGetLastError();
}

}  // namespace emm
