// Decode-step attention over the paged KV pool (bf16, head_dim 128, page size 16) for gfx950: every
// request has at most ONE query token, which attends to its whole context -- the stage that follows
// prefill and produces one token per iteration (Section 2.2 of the paper; memory bound, as it says).
// Same operation as the prefill kernel restricted to one row tile of G = H / Hkv rows per (request,
// KV head) pair; what differs is where the parallelism comes from: the K/V bytes of a pair are read
// exactly once, so the work is cut along the KEY axis, first into pieces of `tiles_per_piece` 64-key
// tiles (one workgroup each, enough of them to fill the chip), then, inside a workgroup, tile by tile
// over its 8 waves.
//
//   workgroup = one piece of one pair.  All 8 waves stream the piece's tiles through the same LDS rings
//               as the prefill kernel (LDS-DMA, same swizzled layout, one barrier per tile); wave w
//               COMPUTES tiles w, w+8, ... of the piece, all waves holding the same G query rows (padded
//               to the 32 columns of the MFMA).  The matrix pipe is mostly idle; the kernel is bound by
//               the rate at which tiles arrive.
//   merge 1   = the 8 waves' (maximum, row sum, accumulator) are combined through LDS;
//   merge 2   = a pair with several pieces leaves one record per piece in the workspace and
//               attn_bf16_decode_merge_kernel combines them; a pair with one piece writes its output
//               directly.  Both kernels derive the piece count from the lengths, nothing is exchanged.
#include "attn_bf16_common.h"

namespace emm {

namespace {

using namespace bf16attn;

constexpr int MAX_G = 16;                        // query heads per KV head this kernel takes
constexpr int REC_FLOATS = D + 2;                // per row of a record: 128 accumulator values, m, l
static_assert(8 * MAX_G * REC_FLOATS * 4 <= 2 * NBUF * KV_BYTES, "the merge across waves reuses the tile rings");

struct DecodeShape {
    int n_pairs;            // (request, KV head) pairs
    int tiles_per_piece;    // 64-key tiles per workgroup
    int pieces_max;         // workgroups per pair in the grid (a pair uses as many as its context needs)
};

__device__ inline int pieces_of(int kv_len, int tiles_per_piece)
{
    const int n_tiles = (kv_len + BC - 1) / BC;
    return n_tiles == 0 ? 1 : (n_tiles + tiles_per_piece - 1) / tiles_per_piece;
}

__device__ inline void lds_dma16(const void* base, uint32_t byte_offset, uint32_t lds_byte_offset)
{
    // 16 bytes per lane from global memory straight into LDS: lane i writes at lds_byte_offset + 16 i
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_byte_offset), "v"(byte_offset), "s"(base) : "memory");
}

template <bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, 2) void attn_bf16_decode_kernel(AttnArgs a, DecodeShape S)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * NBUF * KV_BYTES];   // K ring, then V ring
    constexpr int V_SM = NBUF * KV_BYTES;

    const BatchView& b = a.b;
    const int G = b.num_q_heads / b.num_kv_heads;
    const int pair = blockIdx.x / S.pieces_max, piece = blockIdx.x % S.pieces_max;
    const int kvh = pair % b.num_kv_heads;
    const int r = pair / b.num_kv_heads;
    if (b.new_lens[r] <= 0) return;                          // no query token
    const int P = b.prefix_lens[r];
    const int kv_len = CAUSAL ? P + 1 : P;                   // keys the query sees = slots that hold tokens
    const int n_pieces = pieces_of(kv_len, S.tiles_per_piece);
    if (piece >= n_pieces) return;
    const int n_tiles_all = (kv_len + BC - 1) / BC;
    const int t_begin = piece * S.tiles_per_piece;
    const int n_tiles = min(S.tiles_per_piece, n_tiles_all - t_begin);     // 0 only for an empty context

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31, h32 = lane >> 5;
    const int limit = kv_len - 1;                            // last visible key (the query's own slot if causal)
    const int n_clear = kv_len / BC;                         // tiles 0 .. n_clear-1 need no mask
    const long long q_row = b.cu_new_lens[r];

    // every wave holds the same G query rows; columns G..31 of the MFMA repeat row G-1 and are discarded
    const int hq = kvh * G + min(l32, G - 1);
    const __bf16* __restrict__ qp = (const __bf16*)a.q + (q_row * b.num_q_heads + hq) * D + 8 * h32;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qp + 16 * s);

    // ---- global -> LDS, exactly the prefill kernel's scheme: wave w brings rows 8w .. 8w+7 of the K tile
    //      and of the V tile (logical page 4 kt + w/2), K rows permuted by swap23 and both with their
    //      16-byte chunks XOR-swizzled on the source side.
    const int32_t* __restrict__ pt = b.page_table + (long long)r * b.max_pages;
    const int ld_row = lane >> 4, ld_p = lane & 15;
    const int r16 = 8 * (wave & 1) + ld_row;
    const int k_goff0 = swap23(r16) * 256 + ((ld_p ^ r16) << 4);
    const int v_goff0 = r16 * 256 + ((ld_p ^ ((r16 & 3) << 2)) << 4);
    const unsigned char* __restrict__ kcb = (const unsigned char*)a.k_cache;
    const unsigned char* __restrict__ vcb = (const unsigned char*)a.v_cache;
    const long long slab_bytes = (long long)b.num_kv_heads * 4096;
    const long long head_bytes = (long long)kvh * 4096;
    const int n_pages_valid = max((kv_len + 15) >> 4, 1);
    const int ld_lds = wave * 8 * 256;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
    // lane k of a wave holds the physical page this wave fetches for tile t_begin + k (a piece has at most
    // 56 tiles and fetches run two tiles ahead, so 64 lanes cover it); never leaves the pool
    const int pg_vec = min(max(pt[min((t_begin + lane) * 4 + (wave >> 1), n_pages_valid - 1)], 0), b.num_pages - 1);
    auto load_tile = [&](int i, int slot) {                  // tile t_begin + i into ring slot `slot`
        const int page = __builtin_amdgcn_readlane(pg_vec, i);
        const long long off = (long long)page * slab_bytes + head_bytes;
        lds_dma16(kcb + off, k_goff0, smem_base + slot * KV_BYTES + ld_lds);
        lds_dma16(kcb + off, (k_goff0 ^ 64) + 2048, smem_base + slot * KV_BYTES + ld_lds + 1024);
        lds_dma16(vcb + off, v_goff0, smem_base + V_SM + slot * KV_BYTES + ld_lds);
        lds_dma16(vcb + off, v_goff0 + 1024, smem_base + V_SM + slot * KV_BYTES + ld_lds + 1024);
    };
    // V rows (keys) past the context are zeroed in LDS by the wave that fetched them: 0 * NaN would poison
    // the output; K rows past it only give scores that the mask removes
    auto zero_v_tail = [&](int i, int slot) {
        if ((t_begin + i + 1) * BC > kv_len) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int key = (t_begin + i) * BC + wave * 8 + 4 * j + ld_row;
                if (key >= kv_len)
                    *(uint4*)(smem + V_SM + slot * KV_BYTES + ld_lds + j * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
            }
        }
    };

    const int k_rd0 = l32 * 256 + ((h32 ^ (l32 & 15)) << 4);
    const int v_rd0 = V_SM + (8 * h32 + ((lane & 15) >> 2)) * 256 +
                      ((4 * ((lane & 15) >> 2) + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) << 4) + (lane & 1) * 8;

    f32x16 o_acc[4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[nb][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const float c_log2 = b.softmax_scale * 1.44269504088896340736f;
    const float slack = RESCALE_LOG2 / c_log2;

    // one tile, start to finish, by one wave: S^T = K Q^T, mask, online softmax, O^T += V^T P^T
    auto compute_tile = [&](int i, int slot) {
        f32x16 s[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 kf = *(const bf16x8*)(smem + slot * KV_BYTES + kb * 32 * 256 + (k_rd0 ^ (st << 5)));
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kb], 0, 0, 0);
            }
        const int kt = t_begin + i;
        if (kt >= n_clear) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = kt * BC + 32 * kb + 16 * (v >> 3) + 8 * h32 + (v & 7);
                    s[kb][v] = (key > limit) ? -INFINITY : s[kb][v];
                }
        }
        float mx = s[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][v]);
        mx = pair_max(mx);                                   // finite: a tile below kv_len has a visible key
        if (mx > m_run + slack || m_run == -INFINITY) {      // per row; both lanes of a row decide alike
            const float alpha = __builtin_amdgcn_exp2f((m_run - mx) * c_log2);   // 0 the first time
            l_run *= alpha;
            m_run = mx;
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) o_acc[nb][v] *= alpha;
        }
        const float mc = m_run * c_log2;
        bf16x8 p[2][2];
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const __bf16 pr = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][v], c_log2, -mc));
                p[kb][v >> 3][v & 7] = pr;
                psum += (float)pr;                           // the rounded value, as in the numerator
            }
        l_run += psum;
        typedef short s16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int sb = 0; sb < 2; ++sb)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {
                    const unsigned char* src = smem + slot * KV_BYTES + (32 * kb + 16 * sb) * 256 + (v_rd0 ^ (nb << 6));
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 4 * 256));
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[kb][sb], o_acc[nb], 0, 0, 0);
                }
    };

    if (n_tiles > 0) {
        load_tile(0, 0);
        load_tile(1, 1);                                     // past the piece's end: a clamped page, never read
        __builtin_amdgcn_s_waitcnt(0x0f70);                  // vmcnt(0)
        zero_v_tail(0, 0);
        __syncthreads();
        for (int i = 0; i < n_tiles; ++i) {
            load_tile(i + 2, (i + 2) & 3);                   // slot last read in iteration i-2
            if ((i & 7) == wave) compute_tile(i, i & 3);
            __builtin_amdgcn_s_waitcnt(0x0f74);              // vmcnt(4): tile i+1 has landed
            zero_v_tail(i + 1, (i + 1) & 3);
            __syncthreads();
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);                  // the last two fetches too, before LDS is reused
    }
    __syncthreads();                                         // every wave's fetches have landed, every read is done

    // ---- merge 1: the 8 waves' partial results for the G rows, through LDS (the rings are free now)
    float* __restrict__ red = (float*)smem;                  // [8 waves][G rows][130]
    const float l_pair = pair_sum(l_run);
    if (l32 < G) {
        float* dst = red + (wave * G + l32) * REC_FLOATS;
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) dst[32 * nb + 8 * (v >> 2) + 4 * h32 + (v & 3)] = o_acc[nb][v];
        if (h32 == 0) {
            dst[D] = m_run;
            dst[D + 1] = l_pair;
        }
    }
    __syncthreads();
    float* __restrict__ rec = (float*)a.workspace + (size_t)(pair * S.pieces_max + piece) * MAX_G * REC_FLOATS;
    for (int idx = tid; idx < G * D; idx += NTHREADS) {
        const int row = idx / D, ch = idx % D;
        float m_all = -INFINITY;
        for (int w = 0; w < 8; ++w) m_all = fmaxf(m_all, red[(w * G + row) * REC_FLOATS + D]);
        float acc = 0.f, l_tot = 0.f;
        for (int w = 0; w < 8; ++w) {
            const float* src = red + (w * G + row) * REC_FLOATS;
            const float wgt = (src[D] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((src[D] - m_all) * c_log2);
            acc += wgt * src[ch];
            l_tot += wgt * src[D + 1];
        }
        if (n_pieces == 1) {
            const int head = kvh * G + row;
            ((__bf16*)a.out)[(q_row * b.num_q_heads + head) * D + ch] = (__bf16)(l_tot > 0.f ? acc / l_tot : 0.f);
            if (ch == 0 && a.lse != nullptr)
                a.lse[q_row * b.num_q_heads + head] = (l_tot > 0.f) ? m_all * b.softmax_scale + logf(l_tot) : -INFINITY;
        } else {
            rec[row * REC_FLOATS + ch] = acc;
            if (ch == 0) {
                rec[row * REC_FLOATS + D] = m_all;
                rec[row * REC_FLOATS + D + 1] = l_tot;
            }
        }
    }
}

// merge 2: one workgroup per pair, thread = channel; pairs with a single piece were finished by the main kernel
template <bool CAUSAL>
__global__ __launch_bounds__(D) void attn_bf16_decode_merge_kernel(AttnArgs a, DecodeShape S)
{
    const BatchView& b = a.b;
    const int G = b.num_q_heads / b.num_kv_heads;
    const int pair = blockIdx.x;
    const int kvh = pair % b.num_kv_heads;
    const int r = pair / b.num_kv_heads;
    if (b.new_lens[r] <= 0) return;
    const int P = b.prefix_lens[r];
    const int n_pieces = pieces_of(CAUSAL ? P + 1 : P, S.tiles_per_piece);
    if (n_pieces == 1) return;
    const float c_log2 = b.softmax_scale * 1.44269504088896340736f;
    const long long q_row = b.cu_new_lens[r];
    const int ch = threadIdx.x;
    const float* __restrict__ rec0 = (const float*)a.workspace + (size_t)pair * S.pieces_max * MAX_G * REC_FLOATS;
    for (int row = 0; row < G; ++row) {
        float m_all = -INFINITY;
        for (int j = 0; j < n_pieces; ++j) m_all = fmaxf(m_all, rec0[((size_t)j * MAX_G + row) * REC_FLOATS + D]);
        float acc = 0.f, l_tot = 0.f;
        for (int j = 0; j < n_pieces; ++j) {
            const float* src = rec0 + ((size_t)j * MAX_G + row) * REC_FLOATS;
            const float wgt = __builtin_amdgcn_exp2f((src[D] - m_all) * c_log2);
            acc += wgt * src[ch];
            l_tot += wgt * src[D + 1];
        }
        const int head = kvh * G + row;
        ((__bf16*)a.out)[(q_row * b.num_q_heads + head) * D + ch] = (__bf16)(l_tot > 0.f ? acc / l_tot : 0.f);
        if (ch == 0 && a.lse != nullptr)
            a.lse[q_row * b.num_q_heads + head] = (l_tot > 0.f) ? m_all * b.softmax_scale + logf(l_tot) : -INFINITY;
    }
}

// how a decode batch is cut: enough workgroups to fill the chip, every wave of a workgroup with a tile to do
DecodeShape decode_shape(const BatchView& b)
{
    DecodeShape S;
    S.n_pairs = b.num_reqs * b.num_kv_heads;
    const long long max_tiles = ((long long)b.max_pages * 16 + BC - 1) / BC;          // longest possible context
    long long tpp = (S.n_pairs * max_tiles + 1023) / 1024;                            // aim at ~1024 workgroups
    tpp = ((tpp + 7) / 8) * 8;
    if (tpp < 8) tpp = 8;
    if (tpp > 56) tpp = 56;
    S.tiles_per_piece = (int)tpp;
    S.pieces_max = (int)((max_tiles + tpp - 1) / tpp);
    if (S.pieces_max < 1) S.pieces_max = 1;
    return S;
}

}  // namespace

bool attn_bf16_decode_applies(const BatchView& b)
{
    return b.max_new_len == 1 && b.num_q_heads / b.num_kv_heads <= MAX_G;
}

size_t attn_bf16_decode_workspace_bytes(const BatchView& b)
{
    const DecodeShape S = decode_shape(b);
    return (size_t)S.n_pairs * S.pieces_max * MAX_G * REC_FLOATS * sizeof(float);
}

hipError_t launch_attn_bf16_decode(const AttnArgs& a, hipStream_t stream)
{
    const BatchView& b = a.b;
    if (b.total_new_tokens == 0 || b.num_reqs == 0) return hipSuccess;
    const DecodeShape S = decode_shape(b);
    const long long grid = (long long)S.n_pairs * S.pieces_max;
    if (grid > 0x3fffffff) return hipErrorInvalidValue;
    if (a.causal)
        hipLaunchKernelGGL(attn_bf16_decode_kernel<true>, dim3((unsigned)grid), dim3(NTHREADS), 0, stream, a, S);
    else
        hipLaunchKernelGGL(attn_bf16_decode_kernel<false>, dim3((unsigned)grid), dim3(NTHREADS), 0, stream, a, S);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || S.pieces_max == 1) return err;
    if (a.causal)
        hipLaunchKernelGGL(attn_bf16_decode_merge_kernel<true>, dim3((unsigned)S.n_pairs), dim3(D), 0, stream, a, S);
    else
        hipLaunchKernelGGL(attn_bf16_decode_merge_kernel<false>, dim3((unsigned)S.n_pairs), dim3(D), 0, stream, a, S);
    return hipGetLastError();
}

}  // namespace emm
