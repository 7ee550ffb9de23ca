// Decode-step attention over the paged KV pool (bf16, head_dim 128, pages of 16 to 256 tokens) for gfx950: every
// request has at most ONE query token, which attends to its whole context -- the stage that follows
// prefill and produces one token per iteration (Section 2.2 of the paper; memory bound, as it says).
// Same operation as the prefill kernel restricted to one row tile of G = H / Hkv rows per (request,
// KV head) pair; what differs is where the parallelism comes from: the K/V bytes of a pair are read
// exactly once, so the work is cut along the KEY axis, first into pieces of `tiles_per_piece` 32-key
// tiles (one workgroup each, several times more of them than the chip holds), then, inside a
// workgroup, tile by tile over its 4 waves.
//
//   workgroup = one piece of one pair, 4 waves, 48 KB of LDS: three workgroups share a CU, so that two
//               stream while the third starts up or writes its result.  All waves fetch the piece's
//               tiles into LDS rings of 3 tiles (LDS-DMA, the prefill kernel's swizzled layout, a tile
//               asked for two iterations before it is computed, every fetch landed at the iteration's
//               one barrier: see the loop); wave w COMPUTES tiles w, w+4, ... of the piece, all
//               waves holding the same G query rows (padded to the 32 columns of the MFMA).  The matrix
//               pipe is mostly idle; the kernel is bound by the rate at which tiles arrive from HBM.
//   merge 1   = the 4 waves' (maximum, row sum, accumulator) are combined through LDS;
//   merge 2   = a pair with several pieces leaves one record per piece in the workspace and
//               attn_bf16_decode_merge_kernel combines them; a pair with one piece writes its output
//               directly.  Both kernels derive the piece count from the lengths, nothing is exchanged.
//
// Shared prefixes (Section 3.3: requests repeat system prompts and images).  Requests whose leading pages
// are the same physical pages can be given as a UNIT: up to 32 / G consecutive requests and the length they
// share.  The shared keys are then read once per unit instead of once per request: extra workgroups at the
// end of the grid take the shared part, with the query rows of all the unit's requests side by side in the
// 32 columns of the MFMA, while the requests' own workgroups start behind the shared part; the merge
// kernel adds the records of both.  Built as a second instantiation (SHARED) so that the plain path pays
// nothing for it.
//
// Fused step (FUSED instantiation, emm_decode_step): the query token's own K/V row need not be in the pool
// beforehand.  The workgroup whose piece holds the token's slot copies the row from k_new / v_new into the
// LDS tile once the tile has landed (into the swizzled places the loads would have put it) and stores it in
// the pool when it is done, so a decode step is one launch less than scatter + attention.
#include "attn_bf16_common.h"

#include <mutex>

namespace emm {

namespace {

using namespace bf16attn;

constexpr int MAX_G = 16;                        // query heads per KV head this kernel takes
constexpr int REC_FLOATS = D + 2;                // per row of a record: 128 accumulator values, m, l
constexpr int NW = 4;                            // waves per workgroup
constexpr int NT = NW * 64;
constexpr int BK = 32;                           // keys per tile: two 16-key blocks (a page holds 1 to 16 blocks)
constexpr int TILE_BYTES = BK * D * 2;           // one K or V tile in LDS: 32 rows of 256 bytes
constexpr int NSLOT = 3;                         // ring depth; tile i of a piece lives in slot i % NSLOT
constexpr int AHEAD = 2;                         // a tile is asked for this many iterations before it is computed
constexpr int MIN_TILES_PER_PIECE = 4, MAX_TILES_PER_PIECE = 124;  // 124 + AHEAD page ids fit two registers of 64 lanes
constexpr int WORKGROUPS_PER_ROUND = 3 * 256;     // three workgroups on each of 256 CUs
constexpr int WORKGROUPS_PER_ROUND_ONE_REQUEST = 384;    // see decode_shape
constexpr int OVERHEAD_TILES = 4;                // start and finish of a workgroup, in tile times
constexpr int MAX_ROWS = 32;                     // query rows of a shared-prefix unit: the MFMA's columns
static_assert(NW * MAX_G * REC_FLOATS * 4 <= 2 * NSLOT * TILE_BYTES, "the merge across waves reuses the tile rings");
static_assert(AHEAD == NSLOT - 1, "the slot refilled in iteration i is the one read in iteration i-1");

struct DecodeShape {
    int n_pairs;            // (request, KV head) pairs
    int n_unit_pairs;       // (shared-prefix unit, KV head) pairs
    int tiles_per_piece;    // 32-key tiles per workgroup
    int pieces_max;         // workgroups per pair in the grid (a pair uses as many as its context needs)
    int pieces_unit;        // workgroups per (unit, KV head) pair in the grid
};

__device__ inline int pieces_of(int kv_len, int tiles_per_piece)
{
    const int n_tiles = (kv_len + BK - 1) / BK;
    return n_tiles == 0 ? 1 : (n_tiles + tiles_per_piece - 1) / tiles_per_piece;
}
// pieces of a request's own part when its first t_off tiles belong to a unit's shared part: possibly none
__device__ inline int own_pieces_of(int kv_len, int t_off, int tiles_per_piece, bool in_unit)
{
    if (!in_unit) return pieces_of(kv_len, tiles_per_piece);
    const int n_tiles = (kv_len + BK - 1) / BK - t_off;
    return n_tiles <= 0 ? 0 : (n_tiles + tiles_per_piece - 1) / tiles_per_piece;
}
// workspace: the requests' own records first, [pair][piece][MAX_G rows], then the units', [unit][KV head][piece][MAX_ROWS]
__device__ __host__ inline size_t unit_records_offset(const DecodeShape& S)
{
    return (size_t)S.n_pairs * S.pieces_max * MAX_G * REC_FLOATS;
}

template <bool CAUSAL, bool SHARED, bool FUSED>
__global__ __launch_bounds__(NT, 3) void attn_bf16_decode_kernel(AttnArgs a, DecodeShape S, SharedPrefixView sv)
{
    static_assert(CAUSAL || !FUSED, "only a causal step has a new token to store");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * NSLOT * TILE_BYTES];   // K ring, then V ring
    constexpr int V_SM = NSLOT * TILE_BYTES;

    const BatchView& b = a.b;
    const int G = b.num_q_heads / b.num_kv_heads;
    const int n_own_blocks = S.n_pairs * S.pieces_max;
    const bool unit_mode = SHARED && (int)blockIdx.x >= n_own_blocks;     // this workgroup: a unit's shared part
    const int blk = unit_mode ? blockIdx.x - n_own_blocks : blockIdx.x;
    // piece-major: the first pieces of all contexts come first in the grid, the workgroups that find their
    // context too short for their piece number (they exit at once) gather at its end
    const int n_items = unit_mode ? S.n_unit_pairs : S.n_pairs;
    const int pair = blk % n_items, piece = blk / n_items;                // unit mode: pair = (unit, KV head)
    const int kvh = pair % b.num_kv_heads;
    const int unit = pair / b.num_kv_heads;                               // own part: this is the request itself
    // (what the device arrays hold is forced into range wherever an address depends on it: see safe_new_len)
    const int r = unit_mode ? min(max(sv.unit_first_req[unit], 0), b.num_reqs - 1) : unit;   // the request whose page table is read
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int t_off = (SHARED && !unit_mode) ? max(sv.req_shared_len[r], 0) / BK : 0;   // tiles a unit computes for this request
    const int t_begin = t_off + piece * S.tiles_per_piece;
    // lane k of a wave holds where in the pool the 16-key block lies that this wave fetches for tile t_begin + k
    // and in a second register for tile t_begin + 64 + k (a piece has at most 124 tiles and fetches run two tiles
    // ahead, so two registers cover it).  Asked for before the lengths are
    // known, so that the two loads overlap: entries past the request's pages are read (the row has
    // max_pages of them) and whatever they hold is forced into the pool; those keys are masked.
    const int32_t* __restrict__ pt = b.page_table + (long long)r * b.max_pages;
    const int blk16 = (t_begin + lane) * 2 + (wave >> 1);                 // logical 16-key block of the request
    const int pg_raw = b.max_pages > 0 ? pt[min(blk16 >> b.page_shift, b.max_pages - 1)] : 0;
    const bool long_piece = S.tiles_per_piece + AHEAD > 64;  // the same for the whole grid
    const int blk16_hi = blk16 + 128;
    const int pg_raw_hi = (long_piece && b.max_pages > 0) ? pt[min(blk16_hi >> b.page_shift, b.max_pages - 1)] : 0;
    int kv_len, n_pieces, n_rows;
    bool direct;                                             // one piece and no unit: this workgroup writes the output
    if (!unit_mode) {
        if (b.new_lens[r] <= 0) return;                      // no query token
        const int P = safe_prefix_len(b, r, CAUSAL ? 1 : 0);
        kv_len = CAUSAL ? P + 1 : P;                         // keys the query sees = slots that hold tokens
        const bool in_unit = SHARED && sv.req_unit[r] >= 0;
        n_pieces = own_pieces_of(kv_len, t_off, S.tiles_per_piece, in_unit);
        n_rows = G;
        direct = n_pieces == 1 && !in_unit;
    } else {
        // a multiple of the tile: no mask, no ragged tail
        kv_len = (int)min((long long)max(sv.unit_shared_len[unit], 0), (long long)b.max_pages * b.page_size) / BK * BK;
        n_pieces = (kv_len / BK + S.tiles_per_piece - 1) / S.tiles_per_piece;
        n_rows = min(max(sv.unit_num_reqs[unit], 1) * G, MAX_ROWS);
        direct = false;
    }
    if (piece >= n_pieces) return;
    const int n_tiles_all = (kv_len + BK - 1) / BK;
    const int n_tiles = min(S.tiles_per_piece, n_tiles_all - t_begin);     // 0 only for an empty context
    // in units of 4096 bytes (one block of one KV head): (page, KV head, block within the page)
    const int pg_vec = ((min(max(pg_raw, 0), b.num_pages - 1) * b.num_kv_heads + kvh) << b.page_shift) +
                       (blk16 & ((1 << b.page_shift) - 1));
    const int pg_vec_hi = ((min(max(pg_raw_hi, 0), b.num_pages - 1) * b.num_kv_heads + kvh) << b.page_shift) +
                          (blk16_hi & ((1 << b.page_shift) - 1));
    const int l32 = lane & 31, h32 = lane >> 5;
    const int limit = kv_len - 1;                            // last visible key (the query's own slot if causal)
    const int n_clear = kv_len / BK;                         // tiles 0 .. n_clear-1 need no mask

    // every wave holds the same query rows: the G heads of the request, or in unit mode the G heads of each
    // of the unit's requests; the remaining columns of the MFMA repeat the last row and are discarded
    const int my_row = min(l32, n_rows - 1);
    const int my_req = unit_mode ? min(r + my_row / G, b.num_reqs - 1) : r;
    const int hq = kvh * G + (unit_mode ? my_row % G : my_row);
    const long long q_row = safe_first_row(b, my_req, 1);
    const __bf16* __restrict__ qp = (const __bf16*)a.q + (q_row * b.num_q_heads + hq) * D + 8 * h32;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qp + 16 * s);

    // ---- global -> LDS, the prefill kernel's scheme at half the tile height: wave w brings rows 8w .. 8w+7
    //      of the K tile and of the V tile (logical 16-key block 2 kt + w/2), K rows permuted by swap23 and both
    //      with their 16-byte chunks XOR-swizzled on the source side.
    const int ld_row = lane >> 4, ld_p = lane & 15;
    const int r16 = 8 * (wave & 1) + ld_row;
    const int k_goff0 = swap23(r16) * 256 + ((ld_p ^ r16) << 4);
    const int v_goff0 = r16 * 256 + ((ld_p ^ ((r16 & 3) << 2)) << 4);
    const unsigned char* __restrict__ kcb = (const unsigned char*)a.k_cache;
    const unsigned char* __restrict__ vcb = (const unsigned char*)a.v_cache;
    const int ld_lds = wave * 8 * 256;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
    auto load_tile = [&](int i, int slot) {                  // tile t_begin + i into ring slot `slot`
        const long long off = (long long)__builtin_amdgcn_readlane(i < 64 ? pg_vec : pg_vec_hi, i & 63) * 4096;
        lds_dma16(kcb + off, k_goff0, smem_base + slot * TILE_BYTES + ld_lds);
        lds_dma16(kcb + off, (k_goff0 ^ 64) + 2048, smem_base + slot * TILE_BYTES + ld_lds + 1024);
        lds_dma16(vcb + off, v_goff0, smem_base + V_SM + slot * TILE_BYTES + ld_lds);
        lds_dma16(vcb + off, v_goff0 + 1024, smem_base + V_SM + slot * TILE_BYTES + ld_lds + 1024);
    };
    // V rows (keys) past the context are zeroed in LDS by the wave that fetched them: 0 * NaN would poison
    // the output; K rows past it only give scores that the mask removes
    auto zero_v_tail = [&](int i, int slot) {
        if ((t_begin + i + 1) * BK > kv_len) {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int key = (t_begin + i) * BK + wave * 8 + 4 * j + ld_row;
                if (key >= kv_len)
                    *(uint4*)(smem + V_SM + slot * TILE_BYTES + ld_lds + j * 1024 + lane * 16) = make_uint4(0, 0, 0, 0);
            }
        }
    };

    // FUSED: the tile of this piece that holds the query token's own slot (none in most workgroups); its K/V
    // row comes from k_new / v_new, written by the waves that fetched the rows it replaces
    const int new_tile = (FUSED && !unit_mode) ? (kv_len - 1) / BK - t_begin : -1;
    const long long new_row_bytes = ((long long)safe_first_row(b, r, 1) * b.num_kv_heads + kvh) * (D * 2);
    auto patch_new_row = [&](int i, int slot) {
        if (FUSED && i == new_tile) {
            const int kk = (kv_len - 1) % BK;                                  // key within the tile
            const int rho = (kk & 16) + swap23(kk & 15);                       // LDS row of that key in the K tile
            if (wave == (rho >> 3) && lane < 16)
                *(uint4*)(smem + slot * TILE_BYTES + rho * 256 + ((lane ^ (rho & 15)) << 4)) =
                    *(const uint4*)((const unsigned char*)a.k_new + new_row_bytes + lane * 16);
            if (wave == (kk >> 3) && lane < 16)
                *(uint4*)(smem + V_SM + slot * TILE_BYTES + kk * 256 + ((lane ^ ((kk & 3) << 2)) << 4)) =
                    *(const uint4*)((const unsigned char*)a.v_new + new_row_bytes + lane * 16);
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
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bf16x8 kf = *(const bf16x8*)(smem + slot * TILE_BYTES + (k_rd0 ^ (st << 5)));
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s, 0, 0, 0);
        }
        const int kt = t_begin + i;
        if (kt >= n_clear) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = kt * BK + 16 * (v >> 3) + 8 * h32 + (v & 7);
                s[v] = (key > limit) ? -INFINITY : s[v];
            }
        }
        float mx = s[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
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
        bf16x8 p[2];
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const __bf16 pr = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[v], c_log2, -mc));
            p[v >> 3][v & 7] = pr;
            psum += (float)pr;                               // the rounded value, as in the numerator
        }
        l_run += psum;
        typedef short s16x4 __attribute__((ext_vector_type(4)));
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
            for (int nb = 0; nb < 4; ++nb) {
                const unsigned char* src = smem + slot * TILE_BYTES + 16 * sb * 256 + (v_rd0 ^ (nb << 6));
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 4 * 256));
                const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[sb], o_acc[nb], 0, 0, 0);
            }
    };

    if (n_tiles > 0) {
        for (int i = 0; i < AHEAD; ++i) load_tile(i, i);     // past the piece's end: a clamped page, never read
        __builtin_amdgcn_s_waitcnt(0x0f70 | 4 * (AHEAD - 1));    // tile 0 has landed
        // The query rows were asked for before the tiles and have landed with tile 0, but the compiler, which does
        // not count the tile fetches, takes half of them to be still on their way and would wait for them where
        // they are first used: inside the loop, in the middle of every tile this wave computes, with a wait that
        // also covers every tile fetch in flight.  Using them here puts that wait in front of the loop, once, and
        // leaves the waits of the loop to the one written there.
#pragma unroll
        for (int s = 0; s < 8; ++s) asm volatile("" ::"v"(qf[s]));
        zero_v_tail(0, 0);
        patch_new_row(0, 0);
        __syncthreads();
        int slot = 0;                                        // of tile i
        for (int i = 0; i < n_tiles; ++i) {
            const int slot_next = slot == NSLOT - 1 ? 0 : slot + 1, slot_last = slot == 0 ? NSLOT - 1 : slot - 1;
            load_tile(i + AHEAD, slot_last);                 // the slot last read in iteration i-1
            if ((i & (NW - 1)) == wave) compute_tile(i, slot);
            // Every fetch of this wave has landed before the barrier, tile i+2 as well as tile i+1: a workgroup
            // thus has one tile on its way at a time, asked for at the start of an iteration and waited for at its
            // end, three workgroups of a CU 48 KB between them.  Waiting for tile i+1 only (two tiles in flight,
            // 96 KB per CU) is slower on everything that streams from HBM (decode_b64_8k 205 against 193 us; a
            // fetch-only kernel shows the same: the rate falls as more is in flight), and so is waiting earlier,
            // before or inside this wave's tile (decode_mixed_b32 49 and 53 against 44 us).
            __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
            zero_v_tail(i + 1, slot_next);
            patch_new_row(i + 1, slot_next);
            __syncthreads();
            slot = slot_next;
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);                  // the last fetches too, before LDS is reused
    }
    __syncthreads();                                         // every wave's fetches have landed, every read is done

    if (FUSED && new_tile >= 0 && new_tile < n_tiles && wave == 0 && lane < 32) {
        // the token's row goes to its slot in the pool (K by lanes 0..15, V by 16..31), for the steps to come
        const int pos = kv_len - 1;
        const int page = min(max(pt[pos >> (4 + b.page_shift)], 0), b.num_pages - 1);
        const long long dst = (((long long)page * b.num_kv_heads + kvh) * b.page_size + (pos & (b.page_size - 1))) * 256 + (lane & 15) * 16;
        const unsigned char* src = (const unsigned char*)(lane < 16 ? a.k_new : a.v_new) + new_row_bytes + (lane & 15) * 16;
        unsigned char* pool = (unsigned char*)const_cast<void*>(lane < 16 ? a.k_cache : a.v_cache);
        *(uint4*)(pool + dst) = *(const uint4*)src;
    }

    // ---- merge 1: the waves' partial results, 16 rows at a time, through LDS (the rings are free now)
    float* __restrict__ red = (float*)smem;                  // [NW waves][16 rows][130]
    const float l_pair = pair_sum(l_run);
    float* __restrict__ rec =
        unit_mode ? (float*)a.workspace + unit_records_offset(S) + (size_t)(pair * S.pieces_unit + piece) * MAX_ROWS * REC_FLOATS
                  : (float*)a.workspace + (size_t)(pair * S.pieces_max + piece) * MAX_G * REC_FLOATS;
    for (int row0 = 0; row0 < n_rows; row0 += MAX_G) {
        if (row0 > 0) __syncthreads();                       // the pass before has been read
        const int rows_here = min(MAX_G, n_rows - row0);
        if (l32 >= row0 && l32 < row0 + rows_here) {
            float* dst = red + (wave * MAX_G + l32 - row0) * REC_FLOATS;
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
        for (int idx = tid; idx < rows_here * D; idx += NT) {
            const int lrow = idx / D, ch = idx % D, row = row0 + lrow;
            float m_all = -INFINITY;
#pragma unroll
            for (int w = 0; w < NW; ++w) m_all = fmaxf(m_all, red[(w * MAX_G + lrow) * REC_FLOATS + D]);
            float acc = 0.f, l_tot = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
                const float* src = red + (w * MAX_G + lrow) * REC_FLOATS;
                const float wgt = (src[D] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f((src[D] - m_all) * c_log2);
                acc += wgt * src[ch];
                l_tot += wgt * src[D + 1];
            }
            if (direct) {
                const int head = kvh * G + row;
                const long long q_own = safe_first_row(b, r, 1);
                ((__bf16*)a.out)[(q_own * b.num_q_heads + head) * D + ch] = (__bf16)(l_tot > 0.f ? acc / l_tot : 0.f);
                if (ch == 0 && a.lse != nullptr)
                    a.lse[q_own * b.num_q_heads + head] = (l_tot > 0.f) ? m_all * b.softmax_scale + logf(l_tot) : -INFINITY;
            } else {
                rec[row * REC_FLOATS + ch] = acc;
                if (ch == 0) {
                    rec[row * REC_FLOATS + D] = m_all;
                    rec[row * REC_FLOATS + D + 1] = l_tot;
                }
            }
        }
    }
}

// merge 2: one workgroup per (pair, query row), thread = (piece number mod 8, channel); pairs with a single
// piece were finished by the main kernel.  Few workgroups, so what counts is the length of the chain of
// memory round trips: every piece's (m, l) is loaded once, by its own thread, the weights of a chunk of pieces
// go through LDS, and the loop over the records has nothing but independent loads in it.  GROUPS threads share
// a channel: 8 when a row has many pieces (a single long context: 6.8 -> 4.8 us for 129 pieces), 2 when it has
// few (a big batch, where 1024-thread workgroups would only crowd the chip).
constexpr int MANY_PIECES = 48;

__device__ inline float wave_max64(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
    return x;
}
__device__ inline float wave_sum64(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

template <bool CAUSAL, bool SHARED, int MERGE_GROUPS>
__global__ __launch_bounds__(MERGE_GROUPS * D) void attn_bf16_decode_merge_kernel(AttnArgs a, DecodeShape S, SharedPrefixView sv)
{
    constexpr int MERGE_THREADS = MERGE_GROUPS * D;
    __shared__ float w_s[MERGE_THREADS], part_s[MERGE_THREADS / 64], acc_s[MERGE_GROUPS][D];
    const BatchView& b = a.b;
    const int G = b.num_q_heads / b.num_kv_heads;
    const int pair = blockIdx.x / G, row = blockIdx.x % G;
    const int kvh = pair % b.num_kv_heads;
    const int r = pair / b.num_kv_heads;
    if (b.new_lens[r] <= 0) return;
    const int P = safe_prefix_len(b, r, CAUSAL ? 1 : 0);
    // the records of this row: n_own from the request's own workgroups, then n_unit from its unit's
    // (counts and positions forced into what the workspace holds, whatever the device arrays say)
    const int unit = SHARED ? min(max(sv.req_unit[r], -1), sv.num_units - 1) : -1;
    const int n_own = min(own_pieces_of(CAUSAL ? P + 1 : P, SHARED ? max(sv.req_shared_len[r], 0) / BK : 0, S.tiles_per_piece, unit >= 0),
                          S.pieces_max);
    if (unit < 0 && n_own == 1) return;
    int n_unit = 0;
    const float* __restrict__ rec_unit = nullptr;
    if (unit >= 0) {
        const int shared_len = (int)min((long long)max(sv.unit_shared_len[unit], 0), (long long)b.max_pages * b.page_size) / BK * BK;
        n_unit = min((shared_len / BK + S.tiles_per_piece - 1) / S.tiles_per_piece, S.pieces_unit);
        const int member = min(max(r - sv.unit_first_req[unit], 0), MAX_ROWS / G - 1);       // position of the request in its unit
        rec_unit = (const float*)a.workspace + unit_records_offset(S) +
                   ((size_t)(unit * b.num_kv_heads + kvh) * S.pieces_unit * MAX_ROWS + member * G + row) * REC_FLOATS;
    }
    const int n_pieces = n_own + n_unit;
    const float c_log2 = b.softmax_scale * 1.44269504088896340736f;
    const int tid = threadIdx.x, ch = tid % D, grp = tid / D, wave = tid >> 6;
    const float* __restrict__ rec_own =
        (const float*)a.workspace + ((size_t)pair * S.pieces_max * MAX_G + row) * REC_FLOATS;
    auto record = [&](int j) -> const float* {               // this row in record j
        return j < n_own ? rec_own + (size_t)j * (MAX_G * REC_FLOATS) : rec_unit + (size_t)(j - n_own) * (MAX_ROWS * REC_FLOATS);   // consecutive pieces of the unit
    };

    // the maximum over all pieces (every piece of a context that needs several has a visible key); the (m, l)
    // of piece `tid` stay in registers for the weights below
    float m_mine = -INFINITY, l_mine = 0.f;
    if (tid < n_pieces) {
        const float* src = record(tid);
        m_mine = src[D];
        l_mine = src[D + 1];
    }
    float m_all = m_mine;
    for (int j = tid + MERGE_THREADS; j < n_pieces; j += MERGE_THREADS) m_all = fmaxf(m_all, record(j)[D]);
    m_all = wave_max64(m_all);
    if ((tid & 63) == 0) part_s[wave] = m_all;
    __syncthreads();
    m_all = part_s[0];
#pragma unroll
    for (int i = 1; i < MERGE_THREADS / 64; ++i) m_all = fmaxf(m_all, part_s[i]);

    float acc = 0.f, l_tot = 0.f;
    for (int c0 = 0; c0 < n_pieces; c0 += MERGE_THREADS) {
        __syncthreads();                                     // the weights of the chunk before have been used
        if (c0 + tid < n_pieces) {
            float m_j = m_mine, l_j = l_mine;
            if (c0 > 0) {
                const float* src = record(c0 + tid);
                m_j = src[D];
                l_j = src[D + 1];
            }
            const float wgt = __builtin_amdgcn_exp2f((m_j - m_all) * c_log2);
            w_s[tid] = wgt;
            l_tot += wgt * l_j;
        }
        __syncthreads();
        const int n = min(MERGE_THREADS, n_pieces - c0);
#pragma unroll 8
        for (int j = grp; j < n; j += MERGE_GROUPS) acc += w_s[j] * record(c0 + j)[ch];
    }
    l_tot = wave_sum64(l_tot);
    __syncthreads();                                         // part_s is read above
    if ((tid & 63) == 0) part_s[wave] = l_tot;
    acc_s[grp][ch] = acc;
    __syncthreads();
    if (grp == 0) {
        acc = 0.f;
        l_tot = 0.f;
#pragma unroll
        for (int g = 0; g < MERGE_GROUPS; ++g) acc += acc_s[g][ch];
#pragma unroll
        for (int i = 0; i < MERGE_THREADS / 64; ++i) l_tot += part_s[i];
        const long long q_row = safe_first_row(b, r, 1);
        const int head = kvh * G + row;
        ((__bf16*)a.out)[(q_row * b.num_q_heads + head) * D + ch] = (__bf16)(l_tot > 0.f ? acc / l_tot : 0.f);
        if (ch == 0 && a.lse != nullptr)
            a.lse[q_row * b.num_q_heads + head] = (l_tot > 0.f) ? m_all * b.softmax_scale + logf(l_tot) : -INFINITY;
    }
}

// How a decode batch is cut.  Workgroups run in rounds of WORKGROUPS_PER_ROUND, a round lasts as long as its
// longest piece plus the fixed cost of starting and finishing a workgroup (about OVERHEAD_TILES tiles'
// worth), every workgroup of the grid, also one that finds nothing to do, costs the dispatcher about 1/128 of a
// tile time, and the piece length with the least total is taken -- in particular one that makes the last
// round a full one.  (Sweeps of the piece length on uniform batches put the optimum where this model puts it;
// finer models of HBM saturation and of ragged batches were tried and predicted no better.)
// What the host is told (SharedPrefixView) sharpens the plan: `max_own_tiles` / `max_unit_tiles` bound the
// longest own part / shared part and with it the pieces per context that the grid must provide, and when
// units take work away `planned_tiles` is the amount that is left (32-key tiles per KV head, summed over
// contexts).  Without them the host knows only the longest possible context (the width of the page table) and
// plans for every context being that long.
// A batch of ONE request has no short contexts beside long ones: its KV heads are all as long as each other, and
// about as long as the table is wide.  HBM is then kept busy by half as many workgroups of twice the length, which
// start, finish and are merged half as often: measured on a single context of 131072 tokens, 350 to 410
// workgroups take 50.6-51.5 us, 570 take 55.1, 750 take 56.3 (and 256 take 56.0: too few).  Such a batch is
// planned for rounds of 384.  (With several requests the same would help uniform batches by 1-4 % and cost a
// ragged one 20 %, and the host cannot tell them apart.)
DecodeShape decode_shape(const BatchView& b, const SharedPrefixView& sv = SharedPrefixView{})
{
    DecodeShape S;
    S.n_pairs = b.num_reqs * b.num_kv_heads;
    S.n_unit_pairs = sv.num_units * b.num_kv_heads;
    const long long table_tiles = ((long long)b.max_pages * b.page_size + BK - 1) / BK;       // longest possible context
    const long long own_tiles = sv.max_own_tiles > 0 ? std::min<long long>(sv.max_own_tiles, table_tiles) : table_tiles;
    const long long unit_tiles = sv.num_units == 0 ? 0
                                 : sv.max_unit_tiles > 0 ? std::min<long long>(sv.max_unit_tiles, table_tiles) : table_tiles;
    const long long items = (long long)S.n_pairs + S.n_unit_pairs;
    auto pieces = [](long long tiles, int tpp) { return tiles > 0 ? (tiles + tpp - 1) / tpp : 1; };
    const int per_round = (b.num_reqs == 1 && sv.num_units == 0) ? WORKGROUPS_PER_ROUND_ONE_REQUEST : WORKGROUPS_PER_ROUND;
    long long best_cost = -1;
    int best = MIN_TILES_PER_PIECE;
    for (int tpp = MIN_TILES_PER_PIECE; tpp <= MAX_TILES_PER_PIECE; ++tpp) {
        const long long grid = S.n_pairs * pieces(own_tiles, tpp) + S.n_unit_pairs * pieces(unit_tiles, tpp);
        // known total: half a piece lost per context; else every context as long as the longest
        const long long wgs = (sv.planned_tiles > 0 && sv.num_units > 0)
                                  ? std::min(grid, ((long long)sv.planned_tiles * b.num_kv_heads + tpp - 1) / tpp + items / 2)
                                  : grid;
        const long long rounds = (wgs + per_round - 1) / per_round;
        const long long cost = 128 * rounds * (tpp + OVERHEAD_TILES) + grid;         // in 1/128 tile times
        if (best_cost < 0 || cost <= best_cost) {            // ties: the longer piece, fewer records to merge
            best_cost = cost;
            best = tpp;
        }
    }
    S.tiles_per_piece = best;
    S.pieces_max = (int)pieces(own_tiles, best);
    S.pieces_unit = (int)pieces(unit_tiles, best);
    return S;
}

}  // namespace

bool attn_bf16_decode_applies(const BatchView& b)
{
    return b.max_new_len <= 1 && b.num_q_heads / b.num_kv_heads <= MAX_G;
}

size_t attn_bf16_decode_workspace_bytes(const BatchView& b)
{
    const DecodeShape S = decode_shape(b);
    return (size_t)S.n_pairs * S.pieces_max * MAX_G * REC_FLOATS * sizeof(float);
}

size_t attn_bf16_decode_shared_workspace_bytes(const BatchView& b, const SharedPrefixView& sv)
{
    const DecodeShape S = decode_shape(b, sv);
    return (unit_records_offset(S) + (size_t)S.n_unit_pairs * S.pieces_unit * MAX_ROWS * REC_FLOATS) * sizeof(float);
}

namespace {

template <bool SHARED, bool FUSED>
hipError_t launch_decode(const AttnArgs& a, const SharedPrefixView& sv, hipStream_t stream)
{
    const BatchView& b = a.b;
    if (b.total_new_tokens == 0 || b.num_reqs == 0) return hipSuccess;
    const DecodeShape S = decode_shape(b, sv);
    // the requests' own workgroups first, then (SHARED) those of the units' shared parts
    const long long grid = (long long)S.n_pairs * S.pieces_max + (long long)S.n_unit_pairs * S.pieces_unit;
    if (grid > 0x3fffffff) return hipErrorInvalidValue;
    if (a.causal)
        hipLaunchKernelGGL((attn_bf16_decode_kernel<true, SHARED, FUSED>), dim3((unsigned)grid), dim3(NT), 0, stream, a, S, sv);
    else if constexpr (!FUSED)
        hipLaunchKernelGGL((attn_bf16_decode_kernel<false, SHARED, false>), dim3((unsigned)grid), dim3(NT), 0, stream, a, S, sv);
    else
        return hipErrorInvalidValue;
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || (!SHARED && S.pieces_max == 1)) return err;   // one piece each: already written
    const int G = b.num_q_heads / b.num_kv_heads;
    const dim3 mgrid((unsigned)(S.n_pairs * G));
    const bool many = S.pieces_max + (SHARED ? S.pieces_unit : 0) > MANY_PIECES;
    if (a.causal && many)
        hipLaunchKernelGGL((attn_bf16_decode_merge_kernel<true, SHARED, 8>), mgrid, dim3(8 * D), 0, stream, a, S, sv);
    else if (a.causal)
        hipLaunchKernelGGL((attn_bf16_decode_merge_kernel<true, SHARED, 2>), mgrid, dim3(2 * D), 0, stream, a, S, sv);
    else if (many)
        hipLaunchKernelGGL((attn_bf16_decode_merge_kernel<false, SHARED, 8>), mgrid, dim3(8 * D), 0, stream, a, S, sv);
    else
        hipLaunchKernelGGL((attn_bf16_decode_merge_kernel<false, SHARED, 2>), mgrid, dim3(2 * D), 0, stream, a, S, sv);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16_decode(const AttnArgs& a, hipStream_t stream)
{
    return launch_decode<false, false>(a, SharedPrefixView{}, stream);
}

// ---- The same launch for callers that cannot allocate (code under HIP graph capture, serving loops, harnesses
// that forbid hipMalloc): the piece records go to a fixed array in the library's own device image instead of a
// workspace of the caller's.  Every GPU the library runs on holds the array (EMM_DECODE_STATIC_SCRATCH_BYTES) until the
// process ends, at an address of its own, which is looked up once per device with that device current.  In host
// code the array's name is only a handle for that lookup, never a device address: kernels get the looked-up pointer.
namespace {

constexpr size_t STATIC_SCRATCH_BYTES = 16u << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
void* scratch_ptr[MAX_DEVICES];                              // per device; nullptr until first use there
std::mutex scratch_lock;

}  // namespace

size_t attn_bf16_decode_static_scratch_bytes() { return STATIC_SCRATCH_BYTES; }

hipError_t launch_attn_bf16_decode_static(AttnArgs a, hipStream_t stream)
{
    if (attn_bf16_decode_workspace_bytes(a.b) > STATIC_SCRATCH_BYTES) return hipErrorInvalidValue;
    int dev = -1;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> guard(scratch_lock);
        if (scratch_ptr[dev] == nullptr) {
            err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (err != hipSuccess) return err;
            if (ptr == nullptr) return hipErrorInvalidSymbol;
            scratch_ptr[dev] = ptr;
        }
        ptr = scratch_ptr[dev];
    }
    // The kernels write every record they later read (no counters or flags, nothing that must start at zero), so
    // what an earlier call left in the array does not matter.
    a.workspace = ptr;
    return launch_decode<false, false>(a, SharedPrefixView{}, stream);
}

hipError_t launch_attn_bf16_decode_shared(const AttnArgs& a, const SharedPrefixView& sv, hipStream_t stream)
{
    // without units only the bounds matter: the plain kernels, cut by the sharper plan
    return sv.num_units > 0 ? launch_decode<true, false>(a, sv, stream) : launch_decode<false, false>(a, sv, stream);
}

hipError_t launch_attn_bf16_decode_step(const AttnArgs& a, const SharedPrefixView& sv, hipStream_t stream)
{
    return sv.num_units > 0 ? launch_decode<true, true>(a, sv, stream) : launch_decode<false, true>(a, sv, stream);
}

}  // namespace emm
