// bf16 MFMA flash-style attention over the paged KV pool, head_dim 128, page size 16, for gfx950.
//
// Computes, for every new token of every request, softmax(scale * q K^T) V over the request's
// logical key range read through the page table: cached prefix plus the new tokens up to the
// query itself (prefix-cached prefill, Section 3.3 and Appendix B.7 of the paper) or the whole
// cached image K/V without mask (cross-attention of encoder-decoder models, Section 2.1).
//
// Work decomposition
//   workgroup = 4 waves = 128 consecutive query rows of one (request, query head);
//   wave      = 32 query rows, all 128 channels;
//   KV loop   = tiles of 64 keys (4 pages), in logical order.
// Per tile: the 4 pages of K and of V for the KV head are read from HBM/L2 as whole 4 KB page
// slabs (16 B per lane, fully coalesced), staged in LDS (K row-major and padded, V transposed and
// XOR-swizzled), and consumed by v_mfma_f32_32x32x16_bf16.
//
// Orientation.  Scores are produced transposed, S^T = K Q^T, so that an accumulator lane owns ONE
// query row (column l%32 of the 32x32 result) and 16 of the 32 keys of a block; the other 16 sit
// in lane l^32.  Row max and row sum therefore need in-lane work plus a single exchange with the
// partner lane.  The output is accumulated transposed as well, O^T = V^T P^T, so the same lane
// owns the same query row there and the online-softmax rescale is a per-lane scalar multiply.
// K rows are stored in LDS with bits 2 and 3 of the in-block key index swapped; with that
// placement the 8 probabilities a lane holds in accumulator registers 8s..8s+7 are exactly the 8
// consecutive keys the B operand of the value product expects from that lane, so P never leaves
// registers.
#include "emm_internal.h"

namespace emm {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;            // head dim
constexpr int BR = 128;           // query rows per workgroup
constexpr int BC = 64;            // keys per tile
constexpr int K_STRIDE = 272;     // bytes per K row in LDS (256 + 16 pad: conflict-free 16 B reads)
constexpr int K_BYTES = BC * K_STRIDE;
constexpr int V_STRIDE = 128;     // bytes per V^T row (64 keys), 16 B chunks XOR-swizzled
constexpr int V_BYTES = D * V_STRIDE;
constexpr int NUM_XCD = 8;

__device__ inline uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ inline uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// in-block LDS row of a key: swap bits 2 and 3 of its index within the 16-key page
__device__ inline int swap23(int x) { return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1); }

template <bool CAUSAL>
__global__ __launch_bounds__(256, 2) void attn_bf16_d128_kernel(AttnArgs a, int n_row_tiles, int n_units,
                                                                int units_per_xcd)
{
    __shared__ __attribute__((aligned(16))) unsigned char smem[K_BYTES + V_BYTES];
    unsigned char* const k_sm = smem;
    unsigned char* const v_sm = smem + K_BYTES;

    const BatchView& b = a.b;
    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of units so
    // that the query heads and row tiles that stream the same KV pages share that XCD's L2.
    const int unit = (blockIdx.x % NUM_XCD) * units_per_xcd + blockIdx.x / NUM_XCD;
    if (unit >= n_units) return;
    const int G = b.num_q_heads / b.num_kv_heads;
    int rest = unit;
    const int g = rest % G;             rest /= G;
    const int tile = n_row_tiles - 1 - rest % n_row_tiles;   rest /= n_row_tiles;   // long tiles first
    const int kvh = rest % b.num_kv_heads;
    const int r = rest / b.num_kv_heads;
    const int hq = kvh * G + g;

    const int N = b.new_lens[r];
    const int row0 = tile * BR;
    if (row0 >= N) return;                                   // uniform over the workgroup
    const int P = b.prefix_lens[r];
    const int ctx_len = CAUSAL ? P + N : P;                  // slots of this request that hold tokens
    const int last_row = min(row0 + BR - 1, N - 1);
    const int kv_len = CAUSAL ? P + last_row + 1 : P;        // keys this row tile can see
    const int n_tiles = (kv_len + BC - 1) / BC;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31, h32 = lane >> 5;

    const int wrow0 = row0 + wave * 32;
    const bool wave_active = wrow0 < N;                      // wave-uniform
    const int my_row = wrow0 + l32;
    const int row_c = min(my_row, N - 1);
    const int limit = CAUSAL ? P + row_c : P - 1;            // last visible key of this lane's row
    const int wave_min_limit = CAUSAL ? P + min(wrow0, N - 1) : P - 1;
    const int wave_max_limit = CAUSAL ? P + min(wrow0 + 31, N - 1) : P - 1;

    const long long q_row = (long long)b.cu_new_lens[r] + row_c;
    const __bf16* __restrict__ qp = (const __bf16*)a.q + (q_row * b.num_q_heads + hq) * D + 8 * h32;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qp + 16 * s);

    const int32_t* __restrict__ pt = b.page_table + (long long)r * b.max_pages;
    const uint4* __restrict__ kc = (const uint4*)a.k_cache;
    const uint4* __restrict__ vc = (const uint4*)a.v_cache;
    const long long page_chunks = (long long)b.num_kv_heads * 256;   // 16 B chunks per page (all heads)
    const long long head_chunks = (long long)kvh * 256;

    // staging registers: K, 4 pages x one 16 B chunk per thread; V, the wave's page, 4 keys x 8 channels
    uint4 k_st[4], v_st[4];
    const int v_kg = lane >> 4, v_dc = lane & 15;

    auto load_tile = [&](int kt) {
        const int n_pages_valid = (ctx_len + 15) >> 4;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int lp = kt * 4 + p;
            if (lp < n_pages_valid) {
                const long long page = min(max(pt[lp], 0), b.num_pages - 1);   // never leave the pool
                k_st[p] = kc[page * page_chunks + head_chunks + tid];
            } else {
                k_st[p] = make_uint4(0, 0, 0, 0);
            }
        }
        const int lp = kt * 4 + wave;
        if (lp < n_pages_valid) {
            const long long page = min(max(pt[lp], 0), b.num_pages - 1);
            const uint4* src = vc + page * page_chunks + head_chunks + v_dc;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int key = lp * 16 + 4 * v_kg + i;
                // slots past the request's tokens may hold anything (even NaN patterns): zero them so
                // that a zero probability times the slot is zero
                v_st[i] = (key < ctx_len) ? src[(4 * v_kg + i) * 16] : make_uint4(0, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v_st[i] = make_uint4(0, 0, 0, 0);
        }
    };

    auto store_tile = [&]() {
        // K: page p, key tid/16, chunk tid%16 -> row 16p + swap23(key), padded stride
        const int krow = swap23(tid >> 4);
#pragma unroll
        for (int p = 0; p < 4; ++p)
            *(uint4*)(k_sm + (16 * p + krow) * K_STRIDE + (tid & 15) * 16) = k_st[p];
        // V: transpose the 4 keys x 8 channels block: for channel d = 8*dc + dd write keys 4kg..4kg+3
        const uint32_t* v0 = (const uint32_t*)&v_st[0];
        const uint32_t* v1 = (const uint32_t*)&v_st[1];
        const uint32_t* v2 = (const uint32_t*)&v_st[2];
        const uint32_t* v3 = (const uint32_t*)&v_st[3];
        const int chunk = 2 * wave + (v_kg >> 1);
        const int half = v_kg & 1;
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
            const int d = 8 * v_dc + dd;
            uint2 w;
            if (dd & 1) {
                w.x = pack_hi(v0[dd >> 1], v1[dd >> 1]);
                w.y = pack_hi(v2[dd >> 1], v3[dd >> 1]);
            } else {
                w.x = pack_lo(v0[dd >> 1], v1[dd >> 1]);
                w.y = pack_lo(v2[dd >> 1], v3[dd >> 1]);
            }
            const int phys = chunk ^ ((dd ^ v_dc) & 7);      // == chunk ^ ((d ^ (d >> 3)) & 7)
            *(uint2*)(v_sm + d * V_STRIDE + phys * 16 + half * 8) = w;
        }
    };

    f32x16 o_acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[nb][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c_log2 = b.softmax_scale * 1.44269504088896340736f;

    if (n_tiles > 0) load_tile(0);
    for (int kt = 0; kt < n_tiles; ++kt) {
        store_tile();
        __syncthreads();
        if (kt + 1 < n_tiles) load_tile(kt + 1);             // in flight while this tile is computed

        const int key0 = kt * BC;
        if (wave_active && key0 <= wave_max_limit) {
            // S^T = K Q^T : two 32-key blocks
            f32x16 s_acc[2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) s_acc[kb][v] = 0.f;
                const unsigned char* krow = k_sm + (32 * kb + l32) * K_STRIDE + h32 * 16;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const bf16x8 kf = *(const bf16x8*)(krow + s * 32);
                    s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s_acc[kb], 0, 0, 0);
                }
            }
            // mask: register v of block kb holds key key0 + 32kb + 16(v/8) + 8*h32 + v%8
            if (key0 + BC - 1 > wave_min_limit) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = key0 + 32 * kb + 16 * (v >> 3) + 8 * h32 + (v & 7);
                        s_acc[kb][v] = (key > limit) ? -INFINITY : s_acc[kb][v];
                    }
            }
            float mx = s_acc[0][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_acc[kb][v]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);            // finite from the first tile on
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
            const float mc = m_new * c_log2;
            float psum = 0.f;
            bf16x8 pf[2][2];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(s_acc[kb][v], c_log2, -mc));
                    psum += p;
                    pf[kb][v >> 3][v & 7] = (__bf16)p;
                }
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) o_acc[nb][v] *= alpha;
            // O^T += V^T P^T
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const int d = 32 * nb + l32;
                const unsigned char* vrow = v_sm + d * V_STRIDE;
                const int swz = (d ^ (d >> 3)) & 7;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        const int chunk = 4 * kb + 2 * s + h32;
                        const bf16x8 vf = *(const bf16x8*)(vrow + ((chunk ^ swz) << 4));
                        o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][s], o_acc[nb], 0, 0, 0);
                    }
            }
        }
        __syncthreads();
    }

    if (!wave_active || my_row >= N) return;
    const float l_tot = l_run + __shfl_xor(l_run, 32);       // partner lane is in the same state
    const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
    __bf16* __restrict__ op = (__bf16*)a.out + (q_row * b.num_q_heads + hq) * D;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            // registers 4*v4 .. 4*v4+3 are channels 32nb + 8*v4 + 4*h32 + 0..3
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            bf16x4 w;
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o_acc[nb][4 * v4 + e] * inv);
            *(bf16x4*)(op + 32 * nb + 8 * v4 + 4 * h32) = w;
        }
    if (a.lse != nullptr && h32 == 0)
        a.lse[q_row * b.num_q_heads + hq] =
            (l_tot > 0.f) ? m_run * b.softmax_scale + logf(l_tot) : -INFINITY;
}

}  // namespace

hipError_t launch_attn_bf16_d128(const AttnArgs& a, hipStream_t stream)
{
    const BatchView& b = a.b;
    if (b.total_new_tokens == 0 || b.num_reqs == 0) return hipSuccess;
    const int n_row_tiles = (b.max_new_len + BR - 1) / BR;
    const long long n_units = (long long)n_row_tiles * b.num_reqs * b.num_q_heads;
    if (n_units > 0x3fffffff) return hipErrorInvalidValue;
    const int units_per_xcd = (int)((n_units + NUM_XCD - 1) / NUM_XCD);
    const unsigned grid = (unsigned)units_per_xcd * NUM_XCD;
    if (a.causal)
        hipLaunchKernelGGL(attn_bf16_d128_kernel<true>, dim3(grid), dim3(256), 0, stream, a, n_row_tiles,
                           (int)n_units, units_per_xcd);
    else
        hipLaunchKernelGGL(attn_bf16_d128_kernel<false>, dim3(grid), dim3(256), 0, stream, a, n_row_tiles,
                           (int)n_units, units_per_xcd);
    return hipGetLastError();
}

}  // namespace emm
