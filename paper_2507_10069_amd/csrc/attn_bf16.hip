// bf16 MFMA flash-style attention over the paged KV pool, head_dim 128, page size 16, for gfx950.
//
// Computes, for every new token of every request, softmax(scale * q K^T) V over the request's
// logical key range read through the page table: cached prefix plus the new tokens up to the
// query itself (prefix-cached prefill, Section 3.3 and Appendix B.7 of the paper) or the whole
// cached image K/V without mask (cross-attention of encoder-decoder models, Section 2.1).
//
// Work decomposition
//   row       = one (new token j, query head g of a KV group): index j * G + g, G = H / Hkv, so the
//               G query heads that share a KV head are neighbours and consume the same K/V tile;
//   workgroup = 8 waves = 256 consecutive rows of one (request, KV head); 2 waves per SIMD;
//   wave      = 32 rows, all 128 channels;
//   KV loop   = tiles of 64 keys (4 pages), in logical order.
// Per tile the 4 pages of K and of V for the KV head are read from L2/HBM as whole 4 KB slabs
// (coalesced), register-staged one iteration ahead and written to LDS (K row-major with padded
// rows, V transposed in registers and XOR-swizzled); v_mfma_f32_32x32x16_bf16 consumes them.
//
// Orientation.  Scores are produced transposed, S^T = K Q^T, so that an accumulator lane owns ONE
// query row (column l%32 of the 32x32 result) and 16 of the 32 keys of a block; the other 16 sit
// in lane l^32.  Row max and row sum need in-lane work plus one exchange with the partner lane.
// The output is accumulated transposed as well, O^T = V^T P^T, so the same lane owns the same row
// there and the online-softmax rescale is a per-lane scalar.  K rows are stored in LDS with bits 2
// and 3 of the in-page key index swapped; with that placement accumulator registers 8s..8s+7 of a
// lane are exactly the 8 consecutive keys the B operand of the value product expects from it, so
// P goes from the score accumulators to the PV operand without leaving registers.
//
// Software pipeline.  A single wave issues a plain VALU instruction only about every 8 cycles and
// an MFMA occupies the matrix pipe for 32, so the softmax arithmetic is placed inside the MFMA
// stream of the same wave: iteration i computes S(i+1) = K(i+1) Q^T (16 MFMA) while the VALU turns
// S(i) into P(i) = exp2(S(i) - m), then O += V(i)^T P(i) (16 MFMA) while the VALU stages the next
// tiles into LDS and takes the row maximum of S(i+1).  The running maximum m may lag the true
// maximum by up to 2^8 (it only has to keep exp2 in range); O and l are rescaled only when a row
// exceeds that.  K and V tiles are double buffered in LDS with one workgroup barrier per tile; the
// loop body exists in two copies (tile parity) so buffer offsets and register roles are static.
#include "emm_internal.h"

#include <type_traits>

namespace emm {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;            // head dim
constexpr int BR = 256;           // rows per workgroup
constexpr int NTHREADS = 512;
constexpr int BC = 64;            // keys per tile
constexpr int KV_BYTES = BC * D * 2;   // one K or V tile in LDS: 64 rows of 256 bytes
constexpr int NUM_XCD = 8;
constexpr float RESCALE_LOG2 = 8.0f;   // slack of the lagging maximum, in powers of two

__device__ inline uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ inline uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// A query row lives in lanes l and l^32 (16 of a block's 32 keys each).  v_permlane32_swap with the
// same register as both operands leaves the low half's value in every lane of the first result and
// the high half's in the second, so one instruction gives both lanes both values.
__device__ inline float pair_max(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float pair_sum(float x)
{
    const uint32_t u = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Asynchronous copy of 16 bytes per lane from global memory straight into LDS: lane i of the wave
// writes at lds_byte_offset + 16 i.  Written as inline assembly because the compiler, which cannot
// tell which LDS bytes such a load will write, would otherwise make every later LDS read wait for
// it; here the tile being filled is never the tile being read, and completion is awaited
// explicitly (s_waitcnt vmcnt(0)) before the workgroup barrier that publishes the tile.
__device__ inline void lds_dma16(const void* gptr, uint32_t lds_byte_offset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :: "s"(lds_byte_offset), "v"(gptr) : "memory");
}

// in-page LDS row of a key: swap bits 2 and 3 of its index within the 16-key page
__device__ inline int swap23(int x) { return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1); }

template <bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, 2) void attn_bf16_d128_kernel(AttnArgs a, int n_row_tiles, int n_units,
                                                                     int units_per_xcd)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[4 * KV_BYTES];   // K0 K1 V0 V1
    constexpr int V_SM = 2 * KV_BYTES;                       // byte offset of the V buffers

    const BatchView& b = a.b;
    // Workgroups are dealt to the 8 XCDs round-robin; give each XCD a contiguous range of units so
    // that the row tiles that stream the same (request, KV head) pages share that XCD's L2.
    const int unit = (blockIdx.x % NUM_XCD) * units_per_xcd + blockIdx.x / NUM_XCD;
    if (unit >= n_units) return;
    const int G = b.num_q_heads / b.num_kv_heads;
    int rest = unit;
    const int tile = n_row_tiles - 1 - rest % n_row_tiles;   rest /= n_row_tiles;   // long tiles first
    const int kvh = rest % b.num_kv_heads;
    const int r = rest / b.num_kv_heads;

    const int N = b.new_lens[r];
    const int n_rows = N * G;                                // rows of this (request, KV head)
    const int row0 = tile * BR;
    if (row0 >= n_rows) return;                              // uniform over the workgroup
    const int P = b.prefix_lens[r];
    const int ctx_len = CAUSAL ? P + N : P;                  // slots of this request that hold tokens
    const int last_row = min(row0 + BR - 1, n_rows - 1);
    const int kv_len = CAUSAL ? P + last_row / G + 1 : P;    // keys this row tile can see
    const int n_tiles = (kv_len + BC - 1) / BC;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31, h32 = lane >> 5;

    const int wrow0 = row0 + wave * 32;
    const int my_row = wrow0 + l32;
    const int row_c = min(my_row, n_rows - 1);
    const int tok = row_c / G;                               // new-token index of this lane's row
    const int hq = kvh * G + (row_c - tok * G);              // its query head
    const int limit = CAUSAL ? P + tok : P - 1;              // last visible key of this lane's row
    const int wave_min_limit = CAUSAL ? P + min(wrow0, n_rows - 1) / G : P - 1;
    // tiles 0 .. n_clear-1 lie entirely below every row's limit in this wave: no mask needed
    const int n_clear = (wave_min_limit + 1) / BC;

    const long long q_row = (long long)b.cu_new_lens[r] + tok;
    const __bf16* __restrict__ qp = (const __bf16*)a.q + (q_row * b.num_q_heads + hq) * D + 8 * h32;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qp + 16 * s);

    const int32_t* __restrict__ pt = b.page_table + (long long)r * b.max_pages;
    // ---- global -> LDS.  Tiles go straight from global memory into LDS (global_load_lds_dwordx4: lane i
    //      of a wave writes 16 bytes at base + 16 i), 4 rows of 256 bytes per instruction.  Wave w brings
    //      rows 8w .. 8w+7 of the K tile and of the V tile (two instructions each), all from logical
    //      page 4 kt + w/2.  Placement is row-major with 16-byte chunks XOR-swizzled; since the hardware
    //      fixes where a lane's bytes land, the swizzle (and for K the row permutation) is applied on
    //      the source side: the lane that lands on (row, physical chunk p) fetches logical chunk
    //      p ^ f(row) of the key that belongs in that row.
    //        K: row = 16 page + swap23(key in page), f(row) = row & 15   (read with ds_read_b128)
    //        V: row = key,                           f(row) = (row & 3) << 2   (read with ds_read_tr16_b64)
    //      Page indices past the request's last page are clamped to it (branch-free): K rows fetched
    //      that way give scores the mask removes; V rows past the request's tokens are zeroed in LDS by
    //      the wave that fetched them (zero_v_tail), because 0 * NaN would poison the output.
    const int ld_row = lane >> 4, ld_p = lane & 15;          // row within the 4-row group, physical chunk
    int k_goff[2], v_goff[2];                                // byte offsets inside a (page, head) slab
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int r16 = 8 * (wave & 1) + 4 * j + ld_row;     // LDS row within the page
        k_goff[j] = swap23(r16) * 256 + ((ld_p ^ r16) << 4);
        v_goff[j] = r16 * 256 + ((ld_p ^ ((r16 & 3) << 2)) << 4);
    }
    const unsigned char* __restrict__ kcb = (const unsigned char*)a.k_cache;
    const unsigned char* __restrict__ vcb = (const unsigned char*)a.v_cache;
    const long long slab_bytes = (long long)b.num_kv_heads * 4096;   // one page, all heads
    const long long head_bytes = (long long)kvh * 4096;
    const int n_pages_valid = (ctx_len + 15) >> 4;
    const int ld_lds = wave * 8 * 256;                       // LDS byte offset of this wave's rows in a tile
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

    // Page ids: lane k of a wave holds the physical page this wave fetches for tile pg_base + k (logical
    // page 4 (pg_base + k) + wave/2), refilled every 63 tiles; a tile's id is moved to an SGPR with
    // v_readlane.  (A scalar load per tile would sit behind the LDS-DMA loads in program order.)
    int pg_vec = 0, pg_base = 0;
    auto refill_pages = [&](int kt0) {
        const int lp = min((kt0 + lane) * 4 + (wave >> 1), n_pages_valid - 1);
        pg_vec = min(max(pt[lp], 0), b.num_pages - 1);       // never leave the pool
        pg_base = kt0;
    };
    auto slab_of = [&](int kt) -> long long {                // byte offset of (page of tile kt, this KV head)
        const int page = __builtin_amdgcn_readlane(pg_vec, kt - pg_base);
        return (long long)page * slab_bytes + head_bytes;
    };
    auto load_k = [&](int kt, int kbuf) {
        const unsigned char* src = kcb + slab_of(kt);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            lds_dma16(src + k_goff[j], smem_base + kbuf * KV_BYTES + ld_lds + j * 1024);
    };
    auto load_v = [&](int kt, int vbuf) {
        const unsigned char* src = vcb + slab_of(kt);
#pragma unroll
        for (int j = 0; j < 2; ++j)
            lds_dma16(src + v_goff[j], smem_base + V_SM + vbuf * KV_BYTES + ld_lds + j * 1024);
    };
    // after this wave's loads of V tile kt have landed: zero the rows (keys) it fetched that lie past
    // the request's tokens.  Only the request's last tile can have such rows.
    auto zero_v_tail = [&](int kt, int vbuf) {
        if ((kt + 1) * BC > ctx_len) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int key = kt * BC + wave * 8 + 4 * j + ld_row;
                if (key >= ctx_len)
                    *(uint4*)(smem + V_SM + vbuf * KV_BYTES + ld_lds + j * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
            }
        }
    };

    // ---- per-wave LDS read addresses (loop invariant per lane; buffer and block offsets are immediates)
    // K operand: row 32kb + l32, logical chunk 2st + h32 -> physical (2st + h32) ^ (l32 & 15)
    int k_rd[8];
#pragma unroll
    for (int st = 0; st < 8; ++st) k_rd[st] = l32 * 256 + (((2 * st + h32) ^ (l32 & 15)) << 4);
    // V operand through the transposing read: within each 16-lane group, lane j supplies the address of
    // 4 channels of key k0 + j/4 and receives keys k0 .. k0+3 of channel d0 + j (d0 = first channel of
    // the group), so two reads give the 8 consecutive keys of one channel that the MFMA A operand wants.
    int v_rd[4];
    {
        const int j = lane & 15, g1 = (lane >> 4) & 1;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
            v_rd[nb] = V_SM + (8 * h32 + (j >> 2)) * 256 + ((4 * (nb ^ (j >> 2)) + 2 * g1 + ((j & 3) >> 1)) << 4) + (j & 1) * 8;
    }

    auto qk_tile = [&](int kbuf, f32x16 (&s)[2]) {          // S^T = K Q^T for the 64 keys of a tile
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {                 // two independent accumulation chains
                const bf16x8 kf = *(const bf16x8*)(smem + kbuf * KV_BYTES + kb * 32 * 256 + k_rd[st]);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kb], 0, 0, 0);
            }
    };

    f32x16 o_acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[nb][v] = 0.f;

    auto pv_tile = [&](int vbuf, const bf16x8 (&p)[2][2]) {  // O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {             // four independent accumulation chains
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const unsigned char* src = smem + vbuf * KV_BYTES + (32 * kb + 16 * s) * 256 + v_rd[nb];
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(src));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(src + 4 * 256));
                    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
                    o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[kb][s], o_acc[nb], 0, 0, 0);
                }
    };

    float m_run = -INFINITY, l_run = 0.f;
    const float c_log2 = b.softmax_scale * 1.44269504088896340736f;

    // P = exp2(S c - m c) rounded to bf16; l accumulates the rounded values (the same numbers the value
    // product uses) with one dot-product instruction per pair
    auto exp_tile = [&](const f32x16 (&s)[2], bf16x8 (&p)[2][2]) {
        const float mc = m_run * c_log2;
        bf16x2 ones;
        ones[0] = (__bf16)1.f;
        ones[1] = (__bf16)1.f;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                bf16x2 pr;
                pr[0] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][v], c_log2, -mc));
                pr[1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][v + 1], c_log2, -mc));
#ifdef EMM_NO_DOT2
                psum += (float)pr[0] + (float)pr[1];
#else
                psum = __builtin_amdgcn_fdot2_f32_bf16(pr, ones, psum, false);
#endif
                p[kb][v >> 3][v & 7] = pr[0];
                p[kb][v >> 3][(v & 7) + 1] = pr[1];
            }
        l_run += psum;
    };

    // scores of keys a row must not see become -inf (register v of block kb holds key
    // key0 + 32kb + 16(v/8) + 8*h32 + v%8)
    auto mask_tile = [&](int kt, f32x16 (&s)[2]) {
        const int key0 = kt * BC;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = key0 + 32 * kb + 16 * (v >> 3) + 8 * h32 + (v & 7);
                s[kb][v] = (key > limit) ? -INFINITY : s[kb][v];
            }
    };
    // row maximum of a tile (both lanes of a row get the same value)
    auto row_max = [&](const f32x16 (&s)[2]) -> float {
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
        return pair_max(mx);
    };

    if (n_tiles > 0) {
        // ---- prologue: K(0), V(0), K(1) on their way to LDS
        refill_pages(0);
        load_k(0, 0);
        load_v(0, 0);
        load_k(1, 1);
        __builtin_amdgcn_s_waitcnt(0x0f70);                  // vmcnt(0): this wave's rows have landed
        zero_v_tail(0, 0);
        __syncthreads();

        f32x16 sc[2][2];                                     // scores of tile i live in sc[i & 1]
        bf16x8 pf[2][2];

        qk_tile(0, sc[0]);
        if (n_clear < 1) mask_tile(0, sc[0]);
        m_run = row_max(sc[0]);                              // finite: key 0 is visible to every row
        __syncthreads();                                     // K buffer 0 is refilled in iteration 0

        // Iteration i (parity PAR = i & 1 fixed at compile time so that buffer offsets and register roles
        // are static): S(i+1) and P(i) in the first half, O += V(i)^T P(i), staging and the row maximum
        // of S(i+1) in the second.  K(i+1) is in K buffer PAR^1, V(i) in V buffer PAR.
        auto iteration = [&](int i, auto par, auto masked) {
            constexpr int PAR = decltype(par)::value;
            load_k(i + 2, PAR);                              // K(i+2) replaces K(i), read last iteration
            load_v(i + 1, PAR ^ 1);                          // V(i+1) replaces V(i-1)
            qk_tile(PAR ^ 1, sc[PAR ^ 1]);
            exp_tile(sc[PAR], pf);
            __builtin_amdgcn_sched_barrier(0);               // keep the two halves apart (register pressure)
            pv_tile(PAR, pf);
            if (decltype(masked)::value) mask_tile(i + 1, sc[PAR ^ 1]);
            // The running maximum only has to keep exp2 in range, so it is raised (and O, l rescaled)
            // only when a row's new maximum exceeds it by more than 2^RESCALE_LOG2.  Both lanes of a row
            // hold the same m_run and the same maximum, so they decide alike.
            const float m_cand = fmaxf(m_run, row_max(sc[PAR ^ 1]));
            const bool raise = (m_cand - m_run) * c_log2 > RESCALE_LOG2;
            if (__builtin_amdgcn_ballot_w64(raise) != 0) {
                const float m_new = raise ? m_cand : m_run;
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
                l_run *= alpha;
                m_run = m_new;
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o_acc[nb][v] *= alpha;
            }
            __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0): K(i+2), V(i+1) rows of this wave landed
            zero_v_tail(i + 1, PAR ^ 1);
            __syncthreads();
        };
        // iteration i takes the maximum of tile i+1: unmasked while i+1 < n_clear.  Every wave runs
        // n_tiles-1 iterations in total (one barrier each), split differently between the two loops.
        const int n_plain = max(0, min(n_clear - 1, n_tiles - 1));
        int i = 0;
        // hot loop: two tiles per trip, straight-line (tile parity is the position in the body)
        for (; i + 2 <= n_plain; i += 2) {
            if (i + 3 - pg_base >= 64) refill_pages(i + 1);  // tiles i+1 .. i+3 are fetched in this trip
            iteration(i, std::integral_constant<int, 0>{}, std::false_type{});
            iteration(i + 1, std::integral_constant<int, 1>{}, std::false_type{});
        }
        // remaining tiles (the ones that touch the diagonal or the end of the key range)
        for (; i + 1 < n_tiles; ++i) {
            if (i + 2 - pg_base >= 64) refill_pages(i + 1);
            if (i & 1) iteration(i, std::integral_constant<int, 1>{}, std::true_type{});
            else       iteration(i, std::integral_constant<int, 0>{}, std::true_type{});
        }
        // ---- tail: tile n-1
        if ((n_tiles - 1) & 1) { exp_tile(sc[1], pf); pv_tile(1, pf); }
        else                   { exp_tile(sc[0], pf); pv_tile(0, pf); }
    }

    if (my_row >= n_rows) return;
    const float l_tot = pair_sum(l_run);                     // partner lane is in the same state
    const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
    __bf16* __restrict__ op = (__bf16*)a.out + (q_row * b.num_q_heads + hq) * D;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            // registers 4*v4 .. 4*v4+3 are channels 32nb + 8*v4 + 4*h32 + 0..3
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
    const int G = b.num_q_heads / b.num_kv_heads;
    const long long max_rows = (long long)b.max_new_len * G;
    const long long n_row_tiles = (max_rows + BR - 1) / BR;
    const long long n_units = n_row_tiles * b.num_reqs * b.num_kv_heads;
    if (n_units > 0x3fffffff) return hipErrorInvalidValue;
    const int units_per_xcd = (int)((n_units + NUM_XCD - 1) / NUM_XCD);
    const unsigned grid = (unsigned)units_per_xcd * NUM_XCD;
    if (a.causal)
        hipLaunchKernelGGL(attn_bf16_d128_kernel<true>, dim3(grid), dim3(NTHREADS), 0, stream, a,
                           (int)n_row_tiles, (int)n_units, units_per_xcd);
    else
        hipLaunchKernelGGL(attn_bf16_d128_kernel<false>, dim3(grid), dim3(NTHREADS), 0, stream, a,
                           (int)n_row_tiles, (int)n_units, units_per_xcd);
    return hipGetLastError();
}

}  // namespace emm
