// bf16 MFMA flash-style attention over the paged KV pool, head_dim 128, pages of 16 to 256 tokens, for gfx950.
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
//   KV loop   = tiles of 64 keys (4 blocks of 16 keys; a page holds 1 to 16 blocks), in logical order.
// Per tile the 4 blocks of K and of V for the KV head go straight from L2/HBM into LDS (LDS-DMA loads,
// 16 bytes per lane, whole 4 KB slabs), row-major with XOR-swizzled 16-byte chunks; K is consumed
// with ds_read_b128, V with the transposing ds_read_b64_tr_b16, both by v_mfma_f32_32x32x16_bf16.
//
// Orientation.  Scores are produced transposed, S^T = K Q^T, so that an accumulator lane owns ONE
// query row (column l%32 of the 32x32 result) and 16 of the 32 keys of a block; the other 16 sit
// in lane l^32.  Row max and row sum need in-lane work plus one exchange with the partner lane.
// The output is accumulated transposed as well, O^T = V^T P^T, so the same lane owns the same row
// there and the online-softmax rescale is a per-lane scalar.  K rows are stored in LDS with bits 2
// and 3 of the in-block key index swapped; with that placement accumulator registers 8s..8s+7 of a
// lane are exactly the 8 consecutive keys the B operand of the value product expects from it, so
// P goes from the score accumulators to the PV operand without leaving registers.
//
// Software pipeline.  The softmax arithmetic is placed inside the MFMA stream of the same wave:
// the iteration for tile i computes S(i+1) = K(i+1) Q^T (16 MFMA) while the VALU turns S(i) into
// P(i) = exp2(S(i) c - mc), then O += V(i)^T P(i) (16 MFMA); the body is written as 32 one-MFMA slices
// fenced by scheduling barriers, so the issue order is the written one.  The row sums of P (of the
// bf16-rounded values, so that the normaliser matches the numerator) are taken on the matrix pipe as
// well, with eight small 4x4x4 MFMAs per tile: dot-product instructions on the VALU do not overlap
// with MFMAs.  mc is a per-row reference exponent, not the running maximum: it starts as the maximum of
// the row's first tile and is raised, by whole powers of two, only when a tile's row sum shows that the
// weights have grown large; the loop takes no row maxima.  A unit whose weights overflowed all the same
// (l infinite at its end: every workgroup votes) is done again by a second, careful instantiation that
// keeps the true running maximum.  K and V tiles live in 4-deep rings in LDS, fetched two iterations
// ahead, with one workgroup barrier per tile placed mid-iteration; the loop body exists in four copies
// (ring slot) so buffer offsets and register roles are compile-time constants.
//
// Work units left over after an XCD's full rounds of 32 are cut along the key axis and merged by
// attn_bf16_merge_kernel or, when too short for that, halved along their rows: two workgroups with four
// working waves each (see "Work units" below).  A wave without rows of its own only fetches.
//
// Cost model (measured on gfx950): per MFMA of 32 cycles the SIMD's VALU issue port is taken ~13 cycles
// by the MFMA itself, ~4.3 by each plain VALU instruction, ~8.6 by v_exp_f32, and ~5.6 per KiB of LDS
// data returned; per score the loop needs an fma, an exp and half a cvt, besides the row sums and address
// arithmetic, and runs at about 44 cycles per MFMA.  What holds it there is power, not issue slots: with
// all compute units busy the chip clocks at about 1.65 GHz, and instructions saved come back as clock.
#include "attn_bf16_common.h"

#include <algorithm>
#include <type_traits>

namespace emm {

namespace {

using namespace bf16attn;

constexpr int BR = 256;           // rows per workgroup
constexpr int PF_DIST = 2;          // MFMA operands are read from LDS this many slices ahead of their use
constexpr int K_STEPS_KEPT = 7;     // the K operand's read addresses of steps 1 .. this many are kept in registers over the main loop
constexpr int SOFTMAX_SLICES = 28;  // of an iteration's 32 one-MFMA slices, the first this many carry the softmax arithmetic
constexpr float LAG_LIMIT = 1048576.f;      // 2^20: a tile's row sum beyond this raises the row's reference exponent
constexpr float OVERFLOW_LIMIT = 1.329228e36f;    // 2^120: a row sum at or beyond this (or NaN) at the end of a unit means
                                            // that weights overflowed on the way; the unit is then done again with true maxima
constexpr int VOTE_OFFSET = 2 * NBUF * KV_BYTES - 64;   // LDS bytes of the 8 waves' overflow votes: the end of the rings,
                                            // clear of the output staging area at their start
constexpr int OUT_STRIDE = 272;     // bytes between output rows staged in LDS: 256 + 16, which spreads the banks

// Addresses derived from a per-lane base by one XOR or add, written as volatile assembly, which the optimiser neither
// hoists nor merges nor makes again where the value is used: what is computed before the main loop stays in a
// register over it (the dozen addresses of the operand reads and tile fetches: the loop has the registers for them
// since its last iterations and the last tile share the loop's code, and keeping them is 1.5 % faster than making
// them again in every iteration), what is computed inside costs the one instruction.  IMM: an inline constant or
// 32-bit literal.
template <int IMM>
__device__ inline int xor_here(int x)
{
    if constexpr (IMM == 0) return x;
    int r;
    asm volatile("v_xor_b32_e32 %0, %1, %2" : "=v"(r) : "i"(IMM), "v"(x));
    return r;
}
template <int IMM>
__device__ inline int add_here(int x)
{
    int r;
    asm volatile("v_add_u32_e32 %0, %1, %2" : "=v"(r) : "i"(IMM), "v"(x));
    return r;
}
__device__ inline int xor_add_here(int x, int x_imm, int add)      // (x ^ x_imm) + add; x_imm an inline constant
{
    int r;
    asm volatile("v_xad_u32 %0, %1, %2, %3" : "=v"(r) : "v"(x), "i"(x_imm), "v"(add));
    return r;
}

// Ties a value to the place in the instruction stream where it is written: without it the optimiser
// gathers the softmax arithmetic of several slices into one clump behind the next branch, and the
// matrix pipe idles while both waves of a SIMD work through it.  Emits no instruction.
__device__ inline void pin(float& x) { asm volatile("" : "+v"(x)); }
__device__ inline void pin(bf16x2& x)
{
    uint32_t u = __builtin_bit_cast(uint32_t, x);
    asm volatile("" : "+v"(u));
    x = __builtin_bit_cast(bf16x2, u);
}

// compile-time loop: f(integral_constant<int, I>) for I = BEGIN .. END-1
template <int BEGIN, int END, class F>
__device__ inline void static_for(F&& f)
{
    if constexpr (BEGIN < END) {
        f(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(f);
    }
}

// ---- Work units, and cutting the last ones along the key axis.
// A unit is one row tile of one (request, KV head) pair.  An XCD works through its units in launch order on
// its 32 compute units, so with U units the last U mod 32 of them run in a final, partly empty round.  When
// a workspace is given, each of those tail units is cut into 2 or 4 pieces of equal key range (1 .. 12 units),
// halved along its rows (13 .. 16) or cut into a long and a short piece (17 .. 30), done by
// separate workgroups, so that the final round fills the XCD; a piece writes its unnormalised accumulator,
// running maximum and row sum to the workspace and a second, small kernel merges the pieces of a unit.
// An XCD with fewer units than compute units -- few requests with few new tokens each, the usual case after
// a long cached prefix -- has nothing but a "final round": its units are cut into up to 32 pieces each, as
// many as fill the XCD, so that the latency of a long context is spread over the chip.
// Which units are cut follows from the batch's lengths alone, so every workgroup of either kernel derives
// the same plan by itself: no flags, counters or descriptors are exchanged.
constexpr int CU_PER_XCD = 32;
constexpr int MAX_PARTS = 32;                            // pieces per unit at most
constexpr int PIECES_PER_XCD = 2 * CU_PER_XCD;           // tail units x pieces of an XCD: at most 32, or 2 x 30 (uneven cuts)
constexpr int EXTRA_PER_XCD = CU_PER_XCD - 1;            // workgroups for pieces 1, 2, ... of an XCD's tail units
constexpr int MERGE_PER_XCD = CU_PER_XCD;                // merge workgroups: tail units x shares never exceed 32
constexpr int MIN_TILES_PER_PART = 16;                   // shorter pieces cost more (prologue, merge) than they gain: measured
constexpr int MIN_TILES_PER_PART_UNDERFILLED = 2;        // ... unless the compute units would stay idle otherwise (swept: 1 .. 12)
constexpr int MIN_UNIT_TILES_UNDERFILLED = 24;           // ... and the unit is long enough to pay for the merge launch (measured)
constexpr int SPLIT_MAX_PAIRS_PER_XCD = 64;              // planning scans an XCD's pairs, one per lane of a wave
constexpr int PART_FLOATS = (64 + 2) * NTHREADS;         // per thread: 64 accumulator values, m, l
// A build with -DEMM_TIMELINE (python -m paper_2507_10069_amd.build --timeline -> libemm_timeline.so) makes every
// workgroup of the prefill kernel leave a 64-byte record of when and where it ran in the first TIMELINE_BYTES of
// the workspace; bench.py --timeline reads them.  The regular build has none of it.
#ifdef EMM_TIMELINE
constexpr int TIMELINE_RECORDS = 16384;
constexpr size_t TIMELINE_BYTES = (size_t)TIMELINE_RECORDS * 64;
#else
constexpr size_t TIMELINE_BYTES = 0;
#endif

// With fewer than 8 (request, KV head) pairs some XCDs would get no work, and with requests of different lengths
// and fewer than 8 KV heads the XCDs would get different amounts of it, so each pair is dealt to `fan` XCDs (see
// launch_shape): sub-pair pair * fan + j owns the row tiles j, j + fan, j + 2 fan, ...  "Pair" below means sub-pair.
struct LaunchShape {
    int n_row_tiles;        // row tiles of the longest request's sub-pairs
    int n_pairs;            // sub-pairs in the batch
    int pairs_per_xcd;      // ceil(n_pairs / 8)
    int split;              // 1: tail units may be cut (workspace present)
    int fan;                // sub-pairs per (request, KV head) pair: 1, 2, 4 or 8
    int uneven;             // 1: 17 .. 30 units in an XCD's last round are cut unevenly (see uneven_of)
    int ws_pieces;          // piece records per XCD that the workspace holds
};

struct UnitPlan {
    int pair, tile;         // pair < 0: this workgroup has nothing to do
    int parts, part;        // the unit's key tiles are cut into `parts` ranges; this workgroup does range `part`
    int slot;               // tail slot of the unit within its XCD (meaningful when parts > 1)
    bool rows_only;         // parts == 2 stands for a halving along the rows only (never a cut along the keys)
    int min_tiles;          // key tiles that a piece must have
    int uneven;             // > 0: parts == 2 and piece 0 gets uneven / (uneven + 1) of the key tiles (see uneven_of)
};

// pieces per tail unit when rem units are left over after full_rounds rounds of 32
__host__ __device__ inline int split_factor_of(int rem, int full_rounds)
{
    if (rem == 0) return 1;
    if (full_rounds == 0) {
        // the whole XCD is under-filled: as many pieces per unit as fill it (1 unit: 32, 2: 16, 3-4: 8, 5-8: 4, 9-16: 2)
        int p = 1;
        while (p < MAX_PARTS && 2 * p * rem <= CU_PER_XCD) p *= 2;
        return p;
    }
    // With more leftover units the compute units that stay idle in the last round are few, and the busy
    // ones run at a higher clock for it (the chip is power limited): cutting then costs more than it gains.
    if (rem > 12) return 1;
    return rem > 8 ? 2 : 4;
}
// 13 .. 16 units left over after full rounds are not cut along the keys (see above) but still halved along their
// rows: the 26 .. 32 halves fill the XCD's last round, cost nothing to merge, and each finishes in about 60 % of
// a unit's time.  (On an XCD without a full round they are cut in two along the keys, which also helps units
// of few rows, where there is nothing to halve.)
__host__ __device__ inline bool rows_only_of(int rem, int full_rounds) { return full_rounds > 0 && rem > 12 && rem <= CU_PER_XCD / 2; }
// 17 .. 30 units in the last round leave 15 .. 2 compute units idle for a whole unit's time.  Each of those units is
// cut in two UNEVEN pieces: the long ones keep rem compute units busy, the short ones are dealt k to each of the
// 32 - rem others, k = ceil(rem / (32 - rem)); with the cut at k / (k + 1) of the keys both kinds finish together,
// after k / (k + 1) of a unit's time instead of 1 (24 units: k = 3, cut at 3/4).  Returns k, or 0 if rem is not in range.
__host__ __device__ inline int uneven_of(int rem)
{
    return (rem > CU_PER_XCD / 2 && rem <= CU_PER_XCD - 2) ? (rem + (CU_PER_XCD - rem) - 1) / (CU_PER_XCD - rem) : 0;
}
__host__ __device__ inline int split_factor(int rem, int full_rounds, int uneven_ok)
{
    return (rows_only_of(rem, full_rounds) || (uneven_ok && uneven_of(rem) > 0)) ? 2 : split_factor_of(rem, full_rounds);
}

// row tiles (units) of sub-pair sp
__host__ __device__ inline int sub_pair_tiles(int new_len, int G, int fan, int sp)
{
    const int cnt = (new_len * G + BR - 1) / BR, j = sp % fan;
    return cnt > j ? (cnt - j + fan - 1) / fan : 0;
}

// May a unit of n_tiles key tiles be cut into `parts` pieces?  Every piece must have min_tiles
// tiles, and the first tile of every piece must lie wholly at or below limit_min, the last key that the
// unit's first row sees: then each row finds a visible key in the first tile of each piece and its
// running maximum starts finite.  (Rows only see more keys further down the tile.)
__device__ inline bool cuttable(int n_tiles, int parts, int limit_min, int min_tiles)
{
    const int last_begin = (parts - 1) * n_tiles / parts;
    return n_tiles >= min_tiles * parts && (last_begin + 1) * BC - 1 <= limit_min;
}
// Into how many pieces a unit planned for `parts` pieces is really cut: the largest power of two up to `parts`
// that it can be cut into (1: not at all).  Every workgroup concerned with the unit finds the same number.
__device__ inline int pieces_cut(int n_tiles, int parts, int limit_min, int min_tiles)
{
    if (n_tiles < MIN_UNIT_TILES_UNDERFILLED) min_tiles = MIN_TILES_PER_PART;
    while (parts > 1 && !cuttable(n_tiles, parts, limit_min, min_tiles)) parts >>= 1;
    // two short pieces are no better than two row halves, which need no merge: pieces shorter than the usual
    // minimum only when there are at least four of them
    if (parts == 2 && !cuttable(n_tiles, 2, limit_min, MIN_TILES_PER_PART)) parts = 1;
    return parts;
}
// first tile of piece 1 of a unit cut unevenly, k short pieces to a compute unit
__device__ inline int uneven_split(int n_tiles, int k) { return n_tiles * k / (k + 1); }
// may it be cut that way?  (the same two conditions as in cuttable, for the short piece)
__device__ inline bool uneven_cuttable(int n_tiles, int k, int limit_min)
{
    const int split = uneven_split(n_tiles, k);
    return n_tiles - split >= MIN_TILES_PER_PART && (split + 1) * BC - 1 <= limit_min;
}

__device__ inline int wave_sum64(int x)                  // sum over the wave's 64 lanes, in every lane
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) x += __shfl_xor(x, d, 64);
    return x;
}

// Plan of workgroup `in_xcd` of XCD `xcd`.
// Without cutting (L.split == 0: no workspace, or more than 64 pairs on an XCD) the grid has as many slots per
// pair as the longest request needs (pair-major, row tiles descending) and a workgroup whose slot holds no
// row tile leaves at once.
// With cutting, the lanes of each wave scan the XCD's pairs (at most 64), which gives every workgroup the number
// of units of its XCD and of every pair before it.  Workgroup j then takes unit j in the same order (pair-major,
// row tiles descending); the workgroups after the last unit do pieces 1, 2, ... of the tail units; what is left
// of the grid (sized for the longest request) has nothing to do.  All empty workgroups thus lie at the end of
// the grid: the dispatcher hands out workgroups in order and waits when the next one does not fit anywhere,
// so empty ones in between real ones (a batch of one long request and many short ones) would hold those up.
// merge_idx >= 0 asks instead, whatever in_xcd is, for the plan of merge workgroup merge_idx of the XCD: the unit
// in tail slot merge_idx / shares, with .part = merge_idx % shares, shares = parts (1 for an uneven cut).
__device__ inline UnitPlan plan_unit(const BatchView& b, int G, const LaunchShape& L, int xcd, int in_xcd, int merge_idx = -1)
{
    UnitPlan u;
    u.pair = -1; u.tile = 0; u.parts = 1; u.part = 0; u.slot = 0; u.rows_only = false; u.min_tiles = MIN_TILES_PER_PART; u.uneven = 0;
    if (!L.split) {
        if (merge_idx >= 0 || in_xcd >= L.pairs_per_xcd * L.n_row_tiles) return u;
        const int sp = xcd + NUM_XCD * (in_xcd / L.n_row_tiles);
        if (sp >= L.n_pairs) return u;
        const int idx = L.n_row_tiles - 1 - in_xcd % L.n_row_tiles;      // position among the sub-pair's tiles
        if (idx >= sub_pair_tiles(safe_new_len(b, sp / L.fan / b.num_kv_heads, false), G, L.fan, sp)) return u;
        u.pair = sp / L.fan;
        u.tile = sp % L.fan + L.fan * idx;
        return u;
    }
    // lane pi looks at pair xcd + 8 pi
    const int pi = threadIdx.x & 63;
    const int lane_sp = xcd + NUM_XCD * pi;
    const int cnt = (pi < L.pairs_per_xcd && lane_sp < L.n_pairs)
                        ? sub_pair_tiles(safe_new_len(b, lane_sp / L.fan / b.num_kv_heads, false), G, L.fan, lane_sp) : 0;
    const int total = __builtin_amdgcn_readfirstlane(wave_sum64(cnt));
    const int rem = total % CU_PER_XCD;
    const int parts = split_factor(rem, total / CU_PER_XCD, L.uneven);
    const int first_tail = total - rem;
    int ordinal, slot = 0, part = 0;
    if (merge_idx < 0 && in_xcd < total) {
        ordinal = in_xcd;                                    // a whole unit, or piece 0 of a tail unit
        slot = ordinal - first_tail;
    } else {
        if (parts == 1) return u;
        const int e = in_xcd - total;
        const int shares = (L.uneven && uneven_of(rem) > 0) ? 1 : parts;     // merge workgroups per unit
        slot = merge_idx >= 0 ? merge_idx / shares : e / (parts - 1);
        part = merge_idx >= 0 ? merge_idx % shares : 1 + e % (parts - 1);
        if (slot >= rem) return u;
        ordinal = first_tail + slot;
    }
    // the pair that holds this ordinal: the first one whose inclusive running count exceeds it
    int incl = cnt;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (pi >= d) incl += up;
    }
    const unsigned long long hit = __builtin_amdgcn_ballot_w64(incl > ordinal);
    if (hit == 0) return u;
    const int hit_pi = __builtin_ctzll(hit);
    const int hit_incl = __builtin_amdgcn_readlane(incl, hit_pi);
    const int hit_sp = xcd + NUM_XCD * hit_pi;
    u.pair = hit_sp / L.fan;
    u.tile = hit_sp % L.fan + L.fan * (hit_incl - 1 - ordinal);   // position = cnt - 1 - (ordinal - exclusive count)
    if (parts > 1 && ordinal >= first_tail) {                // a tail unit
        u.parts = parts;
        u.part = part;
        u.slot = slot;
        u.rows_only = rows_only_of(rem, total / CU_PER_XCD);
        u.min_tiles = total < CU_PER_XCD ? MIN_TILES_PER_PART_UNDERFILLED : MIN_TILES_PER_PART;
        u.uneven = L.uneven ? uneven_of(rem) : 0;
    }
    return u;
}

// Workspace: a timeline build's records, then the piece records, [xcd][tail slot x planned pieces per unit + piece]
// [66][512] floats, ws_pieces of them per XCD.
__device__ inline float* part_base(void* workspace, int ws_pieces, int xcd, int slot, int parts, int part)
{
    return (float*)((unsigned char*)workspace + TIMELINE_BYTES) + (size_t)(xcd * ws_pieces + slot * parts + part) * PART_FLOATS;
}

struct KernArgs {
    AttnArgs a;
    LaunchShape L;
};
typedef __attribute__((address_space(3))) unsigned char* lds_bytes;

// One work item -- a unit, or one piece of a cut unit -- from its plan to its output rows (or its record in the
// workspace), by the whole workgroup.  CAREFUL = false is the fast way described at the top; if some row's weights
// overflowed on the way (see OVERFLOW_LIMIT) it writes nothing and hands the item to the CAREFUL = true
// instantiation, which takes the true running maximum before every tile's exponentials and cannot overflow.  `smem`: the 128 KB of LDS of the workgroup, K ring, then V ring.
template <bool CAUSAL>
__device__ void attend_unit_carefully(unsigned long long kernargs, int xcd, int in_xcd, lds_bytes lds);

template <bool CAUSAL, bool CAREFUL>
__device__ inline void attend_unit(const AttnArgs& a, const LaunchShape& L, const int xcd, const int in_xcd, UnitPlan plan,
                                   unsigned char* smem)
{
    constexpr int V_SM = NBUF * KV_BYTES;                    // byte offset of the V buffers

    const BatchView& b = a.b;
    // Workgroups are dealt to the 8 XCDs round-robin.  The (request, KV head) pairs are dealt to the XCDs
    // round-robin as well -- the KV heads of one request cost the same, so this balances the XCDs whatever
    // the request lengths are -- and an XCD works through its pairs one after the other, row tiles from
    // the last (longest key range) to the first, so that the workgroups running together on an XCD mostly
    // stream the same pages through its L2.  plan_unit() says which unit, and which part of its key range,
    // this workgroup does.
    const int G = b.num_q_heads / b.num_kv_heads;
#ifdef EMM_TIMELINE
    const long long tl_t0 = __builtin_amdgcn_s_memrealtime();            // 100 MHz, the same on every compute unit
    const long long tl_c0 = __builtin_readcyclecounter();                // shader clock of this compute unit
#endif
    const int pair = plan.pair, tile = plan.tile;
    const int kvh = pair % b.num_kv_heads;
    const int r = pair / b.num_kv_heads;

    // The page ids of the unit's first 64 key tiles are asked for right away, before the request's lengths are
    // known (the load needs only the request): one memory latency less between launch and first MFMA.  Lane k
    // will fetch 16-key block 4 k + wave / 2 of tile k; what entries past the context hold is never used.
    const int32_t* __restrict__ pt = b.page_table + (long long)r * b.max_pages;
    const int blk_early = (threadIdx.x & 63) * 4 + (threadIdx.x >> 7);
    const int pg_early = pt[min(blk_early >> b.page_shift, b.max_pages - 1)];

    // (lengths forced into what the page table and the packed tensors can hold: see safe_new_len)
    const int N = safe_new_len(b, r, CAUSAL);
    const int n_rows = N * G;                                // rows of this (request, KV head)
    const int row0 = tile * BR;
    if (row0 >= n_rows) return;                              // uniform over the workgroup
    const int P = safe_prefix_len(b, r, CAUSAL ? N : 0);
    const int first_row = safe_first_row(b, r, N);           // of the request in the packed tensors
    const int ctx_len = CAUSAL ? P + N : P;                  // slots of this request that hold tokens
    const int last_row = min(row0 + BR - 1, n_rows - 1);
    const int kv_len = CAUSAL ? P + last_row / G + 1 : P;    // keys this row tile can see
    const int n_tiles_unit = (kv_len + BC - 1) / BC;
    // A tail unit that cannot be cut along the keys (too short) is halved along its ROWS instead: waves 0-3 of
    // the row tile work in the regular workgroup, waves 4-7 in the workgroup of piece 1, the other four only
    // fetch.  Rows are independent, so nothing has to be merged, and with one working wave per SIMD a tile
    // takes about 60 % of the time.  (With at most half a tile of rows there is nothing to halve.)
    int row_half = -1;                                       // -1: all eight waves work on their rows
    // into how many pieces the unit is really cut along the keys: as planned for its XCD, fewer if it is too
    // short for that, 1 if it cannot be cut at all or is only to be halved
    const int limit_first_row = CAUSAL ? P + row0 / G : P - 1;
    const int cut = (plan.parts == 1 || plan.rows_only) ? 1
                    : plan.uneven > 0 ? (uneven_cuttable(n_tiles_unit, plan.uneven, limit_first_row) ? 2 : 1)
                                      : pieces_cut(n_tiles_unit, plan.parts, limit_first_row, plan.min_tiles);
    if (plan.uneven > 0 && cut == 1) {
        if (plan.part > 0) return;                           // too short to cut: the regular workgroup does it all
    } else if (plan.parts > 1 && cut == 1) {
        const bool halve = n_rows - row0 > BR / 2;
        if (plan.part > (halve ? 1 : 0)) return;
        if (halve) row_half = plan.part;
        plan.part = 0;
    } else if (plan.part >= cut) {
        return;
    }
    // this workgroup's key tiles: t_begin .. t_begin + n_tiles - 1
    const int t_split = uneven_split(n_tiles_unit, plan.uneven);          // meaningful for an uneven cut only
    const int t_begin = (plan.uneven > 0 && cut == 2) ? (plan.part ? t_split : 0) : plan.part * n_tiles_unit / cut;
    const int n_tiles = (plan.uneven > 0 && cut == 2) ? (plan.part ? n_tiles_unit - t_split : t_split)
                                                      : (plan.part + 1) * n_tiles_unit / cut - t_begin;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int l32 = lane & 31, h32 = lane >> 5;

    const int wrow0 = row0 + wave * 32;
    // a wave without rows of its own (past the pair's last row, or the other half of a halved unit) computes nothing
    const bool active = wrow0 < n_rows && (row_half < 0 || (wave >> 2) == row_half);
    const int my_row = wrow0 + l32;
    const int row_c = min(my_row, n_rows - 1);
    const int tok = row_c / G;                               // new-token index of this lane's row
    const int limit = CAUSAL ? P + tok : P - 1;              // last visible key of this lane's row
    const int wave_min_limit = CAUSAL ? P + min(wrow0, n_rows - 1) / G : P - 1;
    // tiles 0 .. n_clear-1 lie entirely below every row's limit in this wave: no mask needed
    const int n_clear = (wave_min_limit + 1) / BC;

    const int hq = kvh * G + (row_c - tok * G);              // its query head
    const long long q_row = (long long)first_row + tok;
    const __bf16* __restrict__ qp = (const __bf16*)a.q + (q_row * b.num_q_heads + hq) * D + 8 * h32;
    bf16x8 qf[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) qf[s] = *(const bf16x8*)(qp + 16 * s);

    // ---- global -> LDS.  Tiles go straight from global memory into LDS (global_load_lds_dwordx4: lane i
    //      of a wave writes 16 bytes at base + 16 i), 4 rows of 256 bytes per instruction.  Wave w brings
    //      rows 8w .. 8w+7 of the K tile and of the V tile (two instructions each), all from logical
    //      16-key block 4 kt + w/2.  Placement is row-major with 16-byte chunks XOR-swizzled; since the hardware
    //      fixes where a lane's bytes land, the swizzle (and for K the row permutation) is applied on
    //      the source side: the lane that lands on (row, physical chunk p) fetches logical chunk
    //      p ^ f(row) of the key that belongs in that row.
    //        K: row = 16 block + swap23(key in block), f(row) = row & 15   (read with ds_read_b128)
    //        V: row = key,                           f(row) = (row & 3) << 2   (read with ds_read_tr16_b64)
    //      Block indices past the request's last block are clamped to it (branch-free): K rows fetched
    //      that way give scores the mask removes; V rows past the request's tokens are zeroed in LDS by
    //      the wave that fetched them (zero_v_tail), because 0 * NaN would poison the output.
    const int ld_row = lane >> 4, ld_p = lane & 15;          // row within the 4-row group, physical chunk
    // byte offsets inside a (block, head) slab of what this lane fetches first (rows 8(w&1) + ld_row); the
    // second fetch (4 rows further down) is derived: for K the key moves by 8 and chunk bit 2 flips, for
    // V the row moves by 4
    const int r16 = 8 * (wave & 1) + ld_row;
    const int k_goff0 = swap23(r16) * 256 + ((ld_p ^ r16) << 4);
    const int v_goff0 = r16 * 256 + ((ld_p ^ ((r16 & 3) << 2)) << 4);
    const unsigned char* __restrict__ kcb = (const unsigned char*)a.k_cache;
    const unsigned char* __restrict__ vcb = (const unsigned char*)a.v_cache;
    const int k_goff1 = xor_add_here(k_goff0, 64, 2048), v_goff1 = add_here<1024>(v_goff0);
    const int n_blocks_valid = (ctx_len + 15) >> 4;          // 16-key blocks (4096 bytes per KV head in the pool)
    const int ld_lds = wave * 8 * 256;                       // LDS byte offset of this wave's rows in a tile
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;

    // Block ids: lane k of a wave holds, in units of 4096 bytes, where in the pool the 16-key block lies that
    // this wave fetches for tile pg_base + k (logical block 4 (pg_base + k) + wave/2 of this KV head; a page
    // is 2^page_shift such blocks); refilled every 63 tiles; a tile's id is moved to an SGPR with
    // v_readlane.  (A scalar load per tile would sit behind the LDS-DMA loads in program order.)
    int pg_vec = 0, pg_base = 0;
    auto refill_pages = [&](int kt0) {
        const int blk = min((kt0 + lane) * 4 + (wave >> 1), n_blocks_valid - 1);
        const int page = min(max(pt[blk >> b.page_shift], 0), b.num_pages - 1);       // never leave the pool
        pg_vec = ((page * b.num_kv_heads + kvh) << b.page_shift) + (blk & ((1 << b.page_shift) - 1));
        pg_base = kt0;
    };
    auto slab_of = [&](int kt) -> long long {                // byte offset of this wave's block of tile kt
        return (long long)__builtin_amdgcn_readlane(pg_vec, kt - pg_base) * 4096;
    };
    auto load_k = [&](int kt, int kbuf) {
        const unsigned char* src = kcb + slab_of(kt);
        lds_dma16(src, k_goff0, smem_base + kbuf * KV_BYTES + ld_lds);
        lds_dma16(src, k_goff1, smem_base + kbuf * KV_BYTES + ld_lds + 1024);
    };
    auto load_v = [&](int kt, int vbuf) {
        const unsigned char* src = vcb + slab_of(kt);
        lds_dma16(src, v_goff0, smem_base + V_SM + vbuf * KV_BYTES + ld_lds);
        lds_dma16(src, v_goff1, smem_base + V_SM + vbuf * KV_BYTES + ld_lds + 1024);
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
    // K operand: row 32kb + l32, logical chunk 2st + h32 -> physical (2st + h32) ^ (l32 & 15).  The step
    // index only touches address bits 5..7, so the address of step st is k_rd0 ^ (st << 5).
    const int k_rd0 = l32 * 256 + ((h32 ^ (l32 & 15)) << 4);
    auto k_rd = [&](int st) { return k_rd0 ^ (st << 5); };

    // V operand through the transposing read: within each 16-lane group, lane j supplies the address of
    // 4 channels of key k0 + j/4 and receives keys k0 .. k0+3 of channel d0 + j (d0 = first channel of
    // the group), so two reads give the 8 consecutive keys of one channel that the MFMA A operand wants.
    // The channel block nb only touches address bits 6..7: v_rd(nb) = v_rd0 ^ (nb << 6).
    const int v_rd0 = V_SM + (8 * h32 + ((lane & 15) >> 2)) * 256 +
                      ((4 * ((lane & 15) >> 2) + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) << 4) + (lane & 1) * 8;
    auto v_rd = [&](int nb) { return v_rd0 ^ (nb << 6); };

    auto qk_tile = [&](int kbuf, f32x16 (&s)[2]) {          // S^T = K Q^T for the 64 keys of a tile
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[kb][v] = 0.f;
#pragma unroll
        for (int st = 0; st < 8; ++st)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {                 // two independent accumulation chains
                const bf16x8 kf = *(const bf16x8*)(smem + kbuf * KV_BYTES + kb * 32 * 256 + k_rd(st));
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[kb], 0, 0, 0);
            }
    };

    f32x16 o_acc[4];

    auto pv_tile = [&](int vbuf, const bf16x8 (&p)[2][2]) {  // O^T += V^T P^T
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int nb = 0; nb < 4; ++nb) {             // four independent accumulation chains
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const unsigned char* src = smem + vbuf * KV_BYTES + (32 * kb + 16 * s) * 256 + v_rd(nb);
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(src));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) s16x4*)(src + 4 * 256));
                    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
                    o_acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[kb][s], o_acc[nb], 0, 0, 0);
                }
    };

    // The weights are P = exp2(S c - mc) for a per-row reference exponent mc (in powers of two; c = log2(e) * scale).
    // mc starts as the true maximum of the row's first tile and is NOT kept at the running maximum afterwards: any
    // reference gives the same normalised result as long as nothing overflows, so the loop takes no row maxima at
    // all.  It watches the row sums instead, which the matrix pipe delivers anyway: when a tile's sum passes
    // 2^LAG_LOG2, mc is raised by a whole number of powers of two and O and l are scaled down by exactly that
    // (see the end of iteration()).  mc never exceeds the row's true maximum, so the largest weight of a row is at
    // least 1 and l cannot vanish.  A tile whose scores exceed everything before by more than about 2^90 would
    // overflow before the sums can tell; l is then infinite at the end of the unit, and the unit is done again the
    // slow, safe way (see `careful` below).
    float mc_run, l_run;
    // log2(e) * scale, wave-uniform: kept in a scalar register
    const float c_log2 = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(
        __builtin_bit_cast(int, b.softmax_scale * 1.44269504088896340736f)));

    // P = exp2(S c - m c) rounded to bf16; l accumulates the rounded values (the same numbers the value
    // product uses), four at a time on the matrix pipe
    auto exp_tile = [&](const f32x16 (&s)[2], bf16x8 (&p)[2][2]) {
        const float mc = mc_run;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; v += 2) {
                p[kb][v >> 3][v & 7] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][v], c_log2, -mc));
                p[kb][v >> 3][(v & 7) + 1] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[kb][v + 1], c_log2, -mc));
            }
        f32x4 psum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < 8; ++u)
        {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 w = __builtin_bit_cast(u32x4, p[u >> 2][(u >> 1) & 1]);
            psum = sum4_bf16(w[2 * (u & 1)], w[2 * (u & 1) + 1], psum);
        }
        l_run += psum[0];
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

    mc_run = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int v = 0; v < 16; ++v) o_acc[nb][v] = 0.f;
    if (n_tiles > 0) {
        // ---- prologue: the first tiles K(0), V(0), K(1), V(1), K(2) of this workgroup's range on their way
        //      to LDS (tile numbers in the comments below are relative to t_begin; ring slots follow them)
        const int last_lane = (n_blocks_valid - 1 - (wave >> 1)) >> 2;      // last lane whose block of tile `lane` holds tokens
        if (t_begin == 0 && last_lane >= 0) {
            // the ids asked for at the start; lanes past the context take the wave's last block that holds tokens
            // (any block inside the context will do there: its keys are masked and its V rows zeroed)
            const int src_lane = min(last_lane, 63);
            const int id = min(max(pg_early, 0), b.num_pages - 1);
            const int page = lane <= src_lane ? id : __builtin_amdgcn_readlane(id, src_lane);
            const int blk = min(blk_early, src_lane * 4 + (wave >> 1));
            pg_vec = ((page * b.num_kv_heads + kvh) << b.page_shift) + (blk & ((1 << b.page_shift) - 1));
            pg_base = 0;
        } else {
            refill_pages(t_begin);
        }
        load_k(t_begin, 0);
        load_v(t_begin, 0);
        load_k(t_begin + 1, 1);
        load_v(t_begin + 1, 1);
        load_k(t_begin + 2, 2);
        __builtin_amdgcn_s_waitcnt(0x0f70);                  // vmcnt(0): this wave's rows have landed
        zero_v_tail(t_begin, 0);
        __syncthreads();
        if (!active) {
            // keep fetching this wave's share of every tile and meet the others at the barriers: the same
            // loads, waits and barriers as an iteration of the main loop below, and nothing else
            for (int i = t_begin; i + 1 < t_begin + n_tiles; ++i) {
                const int R = (i - t_begin) & 3;
                if (i + 3 - pg_base >= 64) refill_pages(i + 2);
                load_k(i + 3, (R + 3) & 3);
                load_v(i + 2, (R + 2) & 3);
                __builtin_amdgcn_s_waitcnt(0x0f74);          // vmcnt(4)
                if (i + 1 >= n_clear) zero_v_tail(i + 1, (R + 1) & 3);
                __syncthreads();
            }
        } else {

        f32x16 sc[2][2];                                     // scores of tile i live in sc[i & 1]

        qk_tile(0, sc[0]);
        if (t_begin >= n_clear) mask_tile(t_begin, sc[0]);
        mc_run = row_max(sc[0]) * c_log2;                    // finite: every row sees a key of the first tile

        // Iteration i (R = i % 4 fixed at compile time so that buffer offsets and register roles are
        // static).  K(i+1) is in K slot (R+1)%4, V(i) in V slot R, S(i) in sc[R & 1].  The tiles fetched
        // here, K(i+3) and V(i+2), are first read two iterations later.
        // The body is written as 32 slices, one MFMA each, fenced by scheduling barriers so that the
        // issue order is the one written here: the matrix pipe gets an instruction every slice and the
        // softmax arithmetic fills the VALU slots in between.
        //   slices  0..15  S(i+1) = K(i+1) Q^T        + exp2 work on S(i), key block 0 then 1; tile fetches
        //   slices 16..23  O += V(i)^T P(i), block 0  + rest of the exp2 work (block 1)
        //   slices 24..31  O += V(i)^T P(i), block 1  + row sums of P(i) (slice 24), row maximum of S(i+1)
        // Operands are read from LDS PF_DIST slices ahead of their MFMA.
        // read addresses of the operands, kept over the loop: the three further channel blocks of V, the K steps
        const int v_rd_kept[4] = {v_rd0, xor_here<(1 << 6)>(v_rd0), xor_here<(2 << 6)>(v_rd0), xor_here<(3 << 6)>(v_rd0)};
        int k_rd_kept[8];
        k_rd_kept[0] = k_rd0;
        static_for<1, 1 + K_STEPS_KEPT>([&](auto sc_) { constexpr int st = decltype(sc_)::value; k_rd_kept[st] = xor_here<(st << 5)>(k_rd0); });
        auto iteration = [&](int i, auto par) {
            constexpr int R = decltype(par)::value;
            // tile i+1 needs masking / may hold keys past the request's tokens (both wave-uniform, both rare)
            const bool needs_mask = i + 1 >= n_clear;
            f32x16 (&s_cur)[2] = sc[R & 1];
            f32x16 (&s_nxt)[2] = sc[(R & 1) ^ 1];
            const float mc = mc_run;
            f32x4 psum = {0.f, 0.f, 0.f, 0.f};
            // Softmax work on S(i): 16 units; unit u = 8 kb + 4 s + j turns scores 8s + 2j, 8s + 2j + 1 of
            // key block kb into one register of the operand P[kb][s], with five instructions: F0 F1 (scale,
            // subtract the maximum), E0 E1 (exp2), C (round the pair to bf16).  They are issued as a
            // software-pipelined stream in which no instruction directly follows the one it depends on:
            // group g is E0(g) E1(g) C(g-1) F0(g+1) F1(g+1), 90 slots in all, dealt evenly to slices 0..23.
            uint32_t pw[2][2][4];
            float fa[16], fb[16], ea[16], eb[16];
            auto softmax_op = [&](auto idx_c) {
                constexpr int idx = decltype(idx_c)::value;
                constexpr int g = idx / 5, slot = idx % 5;
                if constexpr (slot == 0) {
                    if constexpr (g < 16) {
                        ea[g] = __builtin_amdgcn_exp2f(fa[g]);
                        pin(ea[g]);
                    }
                } else if constexpr (slot == 1) {
                    if constexpr (g < 16) {
                        eb[g] = __builtin_amdgcn_exp2f(fb[g]);
                        pin(eb[g]);
                    }
                } else if constexpr (slot == 2) {
                    constexpr int u = g - 1;
                    if constexpr (u >= 0 && u < 16) {
                        bf16x2 pr;
                        pr[0] = (__bf16)ea[u];
                        pr[1] = (__bf16)eb[u];
                        pin(pr);
                        pw[u >> 3][(u >> 2) & 1][u & 3] = __builtin_bit_cast(uint32_t, pr);
                    }
                } else {
                    constexpr int u = g + 1;
                    if constexpr (u < 16) {
                        constexpr int kb = u >> 3, v = 2 * (u & 7) + (slot - 3);
                        if constexpr (slot == 3) {
                            fa[u] = fmaf(s_cur[kb][v], c_log2, -mc);
                            pin(fa[u]);
                        } else {
                            fb[u] = fmaf(s_cur[kb][v], c_log2, -mc);
                            pin(fb[u]);
                        }
                    }
                }
            };
            auto softmax_slice = [&](auto slice_c) {         // slice 0 .. SOFTMAX_SLICES-1 of the iteration
                constexpr int sl = decltype(slice_c)::value;
                static_for<(sl * 90) / SOFTMAX_SLICES, ((sl + 1) * 90) / SOFTMAX_SLICES>(softmax_op);
            };
            auto p_operand = [&](int kb, int sblk) -> bf16x8 {
                typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
                const u32x4 t = {pw[kb][sblk][0], pw[kb][sblk][1], pw[kb][sblk][2], pw[kb][sblk][3]};
                return __builtin_bit_cast(bf16x8, t);
            };
            fa[0] = fmaf(s_cur[0][0], c_log2, -mc);
            fb[0] = fmaf(s_cur[0][1], c_log2, -mc);
            int k_addr = k_rd0;                              // of the step last asked for
            int v_addr[4] = {v_rd0, 0, 0, 0};                // of the four channel blocks: made at first use, then kept
            auto read_k = [&](auto kc) -> bf16x8 {           // operand of QK slice k: step k/2, key block k%2
                constexpr int k = decltype(kc)::value;
                if constexpr ((k & 1) == 0) {
                    if constexpr ((k >> 1) <= K_STEPS_KEPT) k_addr = k_rd_kept[k >> 1];
                    else k_addr = xor_here<((k >> 1) << 5)>(k_rd0);
                }
                return *(const bf16x8*)(smem + ((R + 1) & 3) * KV_BYTES + (k & 1) * 32 * 256 + k_addr);
            };
            auto read_v = [&](auto kc) -> bf16x8 {           // operand of PV slice k: kb = k/8, s = (k/4)%2, nb = k%4
                constexpr int k = decltype(kc)::value;
                typedef short s16x4 __attribute__((ext_vector_type(4)));
                if constexpr (k >= 1 && k < 4) v_addr[k] = v_rd_kept[k];
                const unsigned char* src = smem + R * KV_BYTES + (32 * (k >> 3) + 16 * ((k >> 2) & 1)) * 256 + v_addr[k & 3];
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(src + 4 * 256));
                return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            };

            bf16x8 opnd[32 + PF_DIST];                       // operands in flight (short live ranges)
            static_for<0, PF_DIST>([&](auto kc) { opnd[decltype(kc)::value] = read_k(kc); });
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, 16>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                if constexpr (k + PF_DIST < 16) opnd[k + PF_DIST] = read_k(std::integral_constant<int, k + PF_DIST>{});
                else opnd[k + PF_DIST] = read_v(std::integral_constant<int, k + PF_DIST - 16>{});
                if constexpr (k < 2) {
                    f32x16 zero;
#pragma unroll
                    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                    s_nxt[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[k], qf[k >> 1], zero, 0, 0, 0);
                } else {
                    s_nxt[k & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[k], qf[k >> 1], s_nxt[k & 1], 0, 0, 0);
                }
                softmax_slice(kc);
                // fetch the tiles that are first read two iterations from now (slots last read two
                // iterations ago), once the matrix pipe has work queued
                if constexpr (k == 2) load_k(i + 3, (R + 3) & 3);
                if constexpr (k == 4) load_v(i + 2, (R + 2) & 3);
                __builtin_amdgcn_sched_barrier(0);
            });
            // Mid-iteration publish point.  K(i+2) and V(i+1), fetched one iteration ago, must have landed
            // (the four loads issued above may stay in flight); the barrier makes them visible to all
            // waves well before iteration i+1 needs them, and sits where every wave still has MFMAs in
            // flight and its next operands already on the way.
            __builtin_amdgcn_s_waitcnt(0x0f74);              // vmcnt(4)
            if (needs_mask) zero_v_tail(i + 1, (R + 1) & 3);  // such a tile lies beyond every wave's n_clear
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            static_for<0, 16>([&](auto kc) {
                constexpr int k = decltype(kc)::value;
                if constexpr (k + PF_DIST < 16) opnd[16 + k + PF_DIST] = read_v(std::integral_constant<int, k + PF_DIST>{});
                o_acc[k & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(opnd[16 + k], p_operand(k >> 3, (k >> 2) & 1),
                                                                       o_acc[k & 3], 0, 0, 0);
                if constexpr (k == 8) {
                    if (needs_mask) {
                        __builtin_amdgcn_sched_barrier(0);
                        mask_tile(i + 1, s_nxt);             // before the next iteration turns S(i+1) into weights
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                if constexpr (16 + k < SOFTMAX_SLICES) softmax_slice(std::integral_constant<int, 16 + k>{});
                if constexpr (16 + k == SOFTMAX_SLICES) {
                    // row sums of P(i) on the matrix pipe, all eight back to back: switching between MFMA
                    // shapes costs the pipe about 16 cycles each time (measured), so they are not spread out
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<0, 8>([&](auto uc) {
                        constexpr int u = decltype(uc)::value;
                        psum = sum4_bf16(pw[u >> 2][(u >> 1) & 1][2 * (u & 1)], pw[u >> 2][(u >> 1) & 1][2 * (u & 1) + 1], psum);
                    });
                    __builtin_amdgcn_sched_barrier(0);
                }
                __builtin_amdgcn_sched_barrier(0);
            });
            l_run += psum[0];
            // The reference exponent is raised only when a tile's row sum says that the weights have grown past
            // 2^LAG_LOG2: one compare per tile in the common case.  The lane's sum covers its 32 keys of the tile,
            // so sum / 32 <= largest weight <= sum: raising mc by floor(log2(sum)) - 5 powers of two, taken of the
            // larger of the row's two lanes, leaves it at or below the row's true maximum, and scaling O and l
            // by that power of two is exact.
            if (__builtin_amdgcn_ballot_w64(psum[0] > LAG_LIMIT) != 0) {
                const float big = pair_max(psum[0]);         // both lanes of a row decide alike
                const int e = (int)(__float_as_uint(big) >> 23) - 127;          // big > 0: no sign bit
                const int delta = big > LAG_LIMIT ? e - 5 : 0;                  // 15 .. 123
                const float alpha = __uint_as_float((uint32_t)(127 - delta) << 23);
                l_run *= alpha;
                mc_run += (float)delta;
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o_acc[nb][v] *= alpha;
            }
        };
        // The same iteration the slow, safe way (second pass only): nothing interleaved, and before the
        // exponentials of S(i) the row's reference exponent is raised to the true maximum seen so far, so that no
        // weight exceeds 1.  Same ring slots, fetches, waits and barrier as above.
        auto rescale_to_max = [&](const f32x16 (&s_cur)[2]) {
            const float mxc = row_max(s_cur) * c_log2;       // finite from the first tile on
            if (mxc > mc_run) {
                const float alpha = __builtin_amdgcn_exp2f(mc_run - mxc);
                l_run *= alpha;
                mc_run = mxc;
#pragma unroll
                for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) o_acc[nb][v] *= alpha;
            }
        };
        auto careful_iteration = [&](int i, f32x16 (&s_cur)[2], f32x16 (&s_nxt)[2]) {
            const int R = (i - t_begin) & 3;
            if (i + 3 - pg_base >= 64) refill_pages(i + 2);
            qk_tile((R + 1) & 3, s_nxt);
            load_k(i + 3, (R + 3) & 3);
            load_v(i + 2, (R + 2) & 3);
            __builtin_amdgcn_s_waitcnt(0x0f74);              // vmcnt(4)
            if (i + 1 >= n_clear) zero_v_tail(i + 1, (R + 1) & 3);
            __syncthreads();
            rescale_to_max(s_cur);
            bf16x8 pc[2][2];
            exp_tile(s_cur, pc);
            pv_tile(R, pc);
            if (i + 1 >= n_clear) mask_tile(i + 1, s_nxt);
        };
        // four tiles per trip, straight-line (a tile's ring slot is its position in the body); the loop is left
        // wherever the tiles end (separate copies of the body for the last one to three iterations were 1.7 % slower
        // on the mixed workload: more code, and the register allocator deals worse with seven copies than with
        // four); every wave runs n_tiles-1 iterations, one barrier each
        // (iteration() takes the absolute tile number; the ring slot is the position relative to t_begin)
        int i = t_begin;
        const int t_end = t_begin + n_tiles;
        if constexpr (CAREFUL) {
            for (; i + 2 < t_end; i += 2) {                  // S(i) lives in sc[(i - t_begin) & 1]
                careful_iteration(i, sc[0], sc[1]);
                careful_iteration(i + 1, sc[1], sc[0]);
            }
            if (i + 1 < t_end) careful_iteration(i, sc[0], sc[1]);
            if ((n_tiles - 1) & 1) rescale_to_max(sc[1]);
            else rescale_to_max(sc[0]);
        } else {
        for (;;) {
            if (i + 6 - pg_base >= 64) refill_pages(i + 2);  // tiles i+2 .. i+6 may be fetched in this trip
            if (i + 1 >= t_end) break;
            iteration(i, std::integral_constant<int, 0>{});
            if (i + 2 >= t_end) break;
            iteration(i + 1, std::integral_constant<int, 1>{});
            if (i + 3 >= t_end) break;
            iteration(i + 2, std::integral_constant<int, 2>{});
            if (i + 4 >= t_end) break;
            iteration(i + 3, std::integral_constant<int, 3>{});
            i += 4;
        }
        }
        // ---- tail: tile n-1
        bf16x8 pf[2][2];
        const int last_slot = (n_tiles - 1) & 3;             // of the rings; the scores' place follows its parity
        if (last_slot & 1) exp_tile(sc[1], pf);
        else exp_tile(sc[0], pf);
        pv_tile(last_slot, pf);
        }                                                    // active
    }
    // ---- every wave's fetches have landed and every wave is past its last read of the rings, which are free from
    //      here on; then the vote: did any row of the workgroup overflow?
    __builtin_amdgcn_s_waitcnt(0x0f70);                      // vmcnt(0)
    __syncthreads();
    if constexpr (!CAREFUL) {
        const bool lane_bad = active && n_tiles > 0 && !(l_run < OVERFLOW_LIMIT);
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        __attribute__((address_space(3))) int* vote = (__attribute__((address_space(3))) int*)(smem + VOTE_OFFSET);
        const int wave_bad = __builtin_amdgcn_ballot_w64(lane_bad) != 0 ? 1 : 0;      // taken by all lanes, stored by one
        if (lane == 0) vote[wave] = wave_bad;
        __syncthreads();
        const i32x4 v0 = *(const __attribute__((address_space(3))) i32x4*)vote;
        const i32x4 v1 = *(const __attribute__((address_space(3))) i32x4*)(vote + 4);
        const int any = v0[0] | v0[1] | v0[2] | v0[3] | v1[0] | v1[1] | v1[2] | v1[3];
        if (__builtin_amdgcn_readfirstlane(any) != 0) {
            __syncthreads();                                 // all have read the votes before the second pass refills the rings
            attend_unit_carefully<CAUSAL>((unsigned long long)(uintptr_t)__builtin_amdgcn_kernarg_segment_ptr(), xcd, in_xcd,
                                          (lds_bytes)smem);
            // the wave ends here: said in so many words, because otherwise the accumulators count as live across
            // the call and are kept in private memory from here to the epilogue on the fast path too
            __builtin_amdgcn_endpgm();
        }
    }

#ifdef EMM_TIMELINE
    // one record per workgroup at the head of the workspace (the pieces follow): start, end of the tile loop (100 MHz ticks),
    // shader cycles in between, key tiles done, where it ran (HW_ID: compute unit, shader engine; XCC_ID), which unit
    if (threadIdx.x == 0 && blockIdx.x < TIMELINE_RECORDS) {
        long long* rec = (long long*)a.workspace + 8 * (long long)blockIdx.x;
        rec[0] = tl_t0;
        rec[1] = __builtin_amdgcn_s_memrealtime();
        rec[2] = __builtin_readcyclecounter() - tl_c0;
        rec[3] = n_tiles;
        rec[4] = __builtin_amdgcn_s_getreg(4 | (31 << 11));            // HW_REG_HW_ID, all 32 bits
        rec[5] = __builtin_amdgcn_s_getreg(20 | (3 << 11));            // HW_REG_XCC_ID, bits 3:0
        rec[6] = ((long long)pair << 32) | (unsigned)(tile * 64 + plan.part);
        rec[7] = cut;
    }
#endif
    // ---- epilogue.  The row bookkeeping is recomputed from an opaque copy of the thread index so that
    //      none of it has to stay in registers across the main loop.
    {
        int t2 = threadIdx.x;
        asm volatile("" : "+v"(t2));
        if (cut > 1) {
            // a piece of a cut unit: unnormalised accumulator, running maximum and row sum go to the
            // workspace, one coalesced row of 512 floats per register; attn_bf16_merge_kernel finishes
            if (!active) return;                             // a wave without rows has nothing to hand over
            float* __restrict__ ws = part_base(a.workspace, L.ws_pieces, xcd, plan.slot, plan.parts, plan.part) + t2;
            const float l_part = pair_sum(l_run);
#pragma unroll
            for (int nb = 0; nb < 4; ++nb)
#pragma unroll
                for (int v = 0; v < 16; ++v) ws[(16 * nb + v) * NTHREADS] = o_acc[nb][v];
            ws[64 * NTHREADS] = mc_run;
            ws[65 * NTHREADS] = l_part;
            return;
        }
        // The normalised rows go to global memory through LDS, so that a store instruction writes four whole
        // rows of 256 bytes (16 lanes x 16 bytes each): written straight from the accumulator layout, every
        // lane of an instruction would touch a different row, which costs about 2 us per workgroup.  The rings
        // are free by now (see above).
        if (!active) return;
        const int e_wave = t2 >> 6, e_lane = t2 & 63;
        const int e_l32 = e_lane & 31, e_h32 = e_lane >> 5;
        const float l_tot = pair_sum(l_run);                 // partner lane is in the same state
        const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
        unsigned char* stage = smem + e_wave * (32 * OUT_STRIDE);        // this wave's 32 rows, OUT_STRIDE bytes apart
#pragma unroll
        for (int nb = 0; nb < 4; ++nb)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                // registers 4*v4 .. 4*v4+3 are channels 32nb + 8*v4 + 4*h32 + 0..3
                bf16x4 w;
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = (__bf16)(o_acc[nb][4 * v4 + e] * inv);
                *(bf16x4*)(stage + e_l32 * OUT_STRIDE + 2 * (32 * nb + 8 * v4 + 4 * e_h32)) = w;
            }
        const int e_row = row0 + e_wave * 32 + e_l32;
        if (a.lse != nullptr && e_h32 == 0 && e_row < n_rows) {
            const int e_tok = e_row / G;
            a.lse[((long long)first_row + e_tok) * b.num_q_heads + kvh * G + (e_row - e_tok * G)] =
                (l_tot > 0.f) ? mc_run * 0.69314718055994530942f + logf(l_tot) : -INFINITY;
        }
        // the wave's own LDS writes are visible to its own reads once they have completed
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        const long long q_row0 = first_row;
        const int t_add = 4 / G, g_add = 4 - t_add * G;      // row + 4 is token + t_add, head + g_add (mod G)
        const int first = row0 + e_wave * 32 + (e_lane >> 4);
        int o_tok = first / G, o_g = first - o_tok * G;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int in_wave = (e_lane >> 4) + 4 * j;       // lanes 16k .. 16k+15 take row 4j + k
            if (first + 4 * j < n_rows) {
                const uint4 v = *(const uint4*)(stage + in_wave * OUT_STRIDE + (e_lane & 15) * 16);
                *(uint4*)((__bf16*)a.out + ((q_row0 + o_tok) * b.num_q_heads + kvh * G + o_g) * D + (e_lane & 15) * 8) = v;
            }
            o_tok += t_add;
            o_g += g_add;
            if (o_g >= G) { o_g -= G; o_tok += 1; }
        }
    }
}

// The second, safe pass over a work item whose weights overflowed.  A function of its own, not inlined: its
// registers are allocated apart from the fast path's, which has none to spare, and nothing of the caller has to
// survive the call.  It reads the kernel's arguments from the kernel argument segment, whose address the kernel
// hands over (asked for in here, in a function that is not a kernel, that address comes out as null), rather than
// through a copy in private memory, and works the item's plan out again.
template <bool CAUSAL>
__device__ __attribute__((noinline)) void attend_unit_carefully(unsigned long long kernargs_v, int xcd_v, int in_xcd_v, lds_bytes lds_v)
{
    // arguments arrive in vector registers; everything here is the same in all lanes, and the tile loads want their
    // base addresses in scalar registers
    const int xcd = __builtin_amdgcn_readfirstlane(xcd_v), in_xcd = __builtin_amdgcn_readfirstlane(in_xcd_v);
    const lds_bytes lds = (lds_bytes)(uintptr_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)lds_v);
    const unsigned long long kernargs =
        ((unsigned long long)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(kernargs_v >> 32)) << 32) |
        (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)kernargs_v);
    const KernArgs* __restrict__ ka = (const KernArgs*)(const __attribute__((address_space(4))) KernArgs*)kernargs;
    const AttnArgs& a = ka->a;
    const LaunchShape& L = ka->L;
    const UnitPlan plan = plan_unit(a.b, a.b.num_q_heads / a.b.num_kv_heads, L, xcd, in_xcd);
    if (plan.pair < 0) return;
    attend_unit<CAUSAL, true>(a, L, xcd, in_xcd, plan, (unsigned char*)lds);
}

template <bool CAUSAL>
__global__ __launch_bounds__(NTHREADS, 2) void attn_bf16_d128_kernel(KernArgs ka)
{
    __shared__ __attribute__((aligned(1024))) unsigned char smem[2 * NBUF * KV_BYTES];   // K ring, then V ring
    const AttnArgs& a = ka.a;
    const LaunchShape& L = ka.L;
    const BatchView& b = a.b;
    // Workgroups are dealt to the 8 XCDs round-robin by the dispatcher; plan_unit() says which unit, and which
    // part of its key range, this one does.
    const int xcd = blockIdx.x % NUM_XCD, in_xcd = blockIdx.x / NUM_XCD;
    const UnitPlan plan = plan_unit(b, b.num_q_heads / b.num_kv_heads, L, xcd, in_xcd);
    if (plan.pair < 0) return;
    attend_unit<CAUSAL, false>(a, L, xcd, in_xcd, plan, smem);
}

// One workgroup's share of the merge of a unit planned for PARTS pieces and cut into `cut` of them: REGS = 64 / SHARES
// consecutive ones of each thread's 64 accumulator registers (32 pieces: 32 shares of 2 registers, so that what is
// in flight fits the register file).  Every load is issued whatever `cut` is (pieces past the last repeat it,
// with weight 0), all of them before the first use, so that one memory latency covers them.
template <int PARTS, int SHARES = PARTS>
__device__ inline void merge_share(const float* __restrict__ ws0, unsigned tid, int cut, int sub,
                                   __bf16* __restrict__ op, int h32, float* __restrict__ lse)
{
    // ws0 is the same for the whole workgroup and tid a 32-bit offset: loads with a scalar base, no address registers
    constexpr int REGS = 64 / SHARES;
    float m_part[PARTS], l_part[PARTS], val[PARTS][REGS];
#pragma unroll
    for (int j = 0; j < PARTS; ++j) {
        const float* __restrict__ wsj = ws0 + (size_t)min(j, cut - 1) * PART_FLOATS;
        m_part[j] = (wsj + 64 * NTHREADS)[tid];
        l_part[j] = (wsj + 65 * NTHREADS)[tid];
#pragma unroll
        for (int i = 0; i < REGS; ++i) val[j][i] = (wsj + (size_t)(sub * REGS + i) * NTHREADS)[tid];
    }
    float m_all = -INFINITY;
#pragma unroll
    for (int j = 0; j < PARTS; ++j)
        if (j < cut) m_all = fmaxf(m_all, m_part[j]);
    float l_tot = 0.f, acc[REGS];
#pragma unroll
    for (int i = 0; i < REGS; ++i) acc[i] = 0.f;
#pragma unroll
    for (int j = 0; j < PARTS; ++j) {
        const float w = j < cut ? __builtin_amdgcn_exp2f(m_part[j] - m_all) : 0.f;
        l_tot += w * l_part[j];
#pragma unroll
        for (int i = 0; i < REGS; ++i) acc[i] += w * val[j][i];
    }
    const float inv = (l_tot > 0.f) ? 1.f / l_tot : 0.f;
    // register 4g + e of a thread is channel 32 (g / 4) + 8 (g % 4) + 4 h32 + e
    if constexpr (REGS == 2) {
        const int g = sub >> 1;
        bf16x2 o;
        o[0] = (__bf16)(acc[0] * inv);
        o[1] = (__bf16)(acc[1] * inv);
        *(bf16x2*)(op + 32 * (g >> 2) + 8 * (g & 3) + 4 * h32 + 2 * (sub & 1)) = o;
    } else {
#pragma unroll
        for (int i = 0; i < REGS / 4; ++i) {
            const int g = sub * (REGS / 4) + i;
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (__bf16)(acc[4 * i + e] * inv);
            *(bf16x4*)(op + 32 * (g >> 2) + 8 * (g & 3) + 4 * h32) = o;
        }
    }
    if (lse != nullptr) *lse = (l_tot > 0.f) ? m_all * 0.69314718055994530942f + logf(l_tot) : -INFINITY;
}

// Merges the pieces of the cut units, thread for thread the layout of the main kernel's epilogue.  An XCD
// whose tail units are planned for p pieces each gets 32 workgroups: number k works on tail slot k / p and
// there on share k % p of the 64 accumulator registers, so every workgroup reads the same 64 rows of 2 KB
// whatever p is (one workgroup per unit, 128 rows, for an uneven cut in two).  Workgroups whose slot holds no cut unit leave at once.
__global__ __launch_bounds__(NTHREADS) void attn_bf16_merge_kernel(AttnArgs a, LaunchShape L)
{
    const BatchView& b = a.b;
    const int G = b.num_q_heads / b.num_kv_heads;
    const int xcd = blockIdx.x % NUM_XCD;
    const UnitPlan plan = plan_unit(b, G, L, xcd, 0, blockIdx.x / NUM_XCD);   // .part is this workgroup's share
    if (plan.pair < 0) return;
    const int kvh = plan.pair % b.num_kv_heads;
    const int r = plan.pair / b.num_kv_heads;
    const int N = safe_new_len(b, r, a.causal != 0);         // the same values as in the main kernel
    const int n_rows = N * G;
    const int row0 = plan.tile * BR;
    if (row0 >= n_rows) return;
    const int P = safe_prefix_len(b, r, a.causal ? N : 0);
    const int last_row = min(row0 + BR - 1, n_rows - 1);
    const int kv_len = a.causal ? P + last_row / G + 1 : P;
    const int limit_first_row = a.causal ? P + row0 / G : P - 1;
    const int cut = plan.rows_only ? 1
                    : plan.uneven > 0 ? (uneven_cuttable((kv_len + BC - 1) / BC, plan.uneven, limit_first_row) ? 2 : 1)
                                      : pieces_cut((kv_len + BC - 1) / BC, plan.parts, limit_first_row, plan.min_tiles);
    if (cut == 1) return;                                    // not cut along the keys

    const int tid = threadIdx.x;
    const int l32 = tid & 31, h32 = (tid >> 5) & 1;
    const int row = row0 + (tid >> 6) * 32 + l32;
    if (row >= n_rows) return;
    const int tok = row / G;
    const int hq = kvh * G + (row - tok * G);
    const long long q_row = (long long)safe_first_row(b, r, N) + tok;
    const float* __restrict__ ws0 = part_base(a.workspace, L.ws_pieces, xcd, plan.slot, plan.parts, 0);
    __bf16* __restrict__ op = (__bf16*)a.out + (q_row * b.num_q_heads + hq) * D;
    float* lse = (a.lse != nullptr && h32 == 0 && plan.part == 0) ? a.lse + q_row * b.num_q_heads + hq : nullptr;
    if (plan.uneven > 0) {
        merge_share<2, 1>(ws0, tid, cut, 0, op, h32, lse);
        return;
    }
    switch (plan.parts) {
        case 2: merge_share<2>(ws0, tid, cut, plan.part, op, h32, lse); break;
        case 4: merge_share<4>(ws0, tid, cut, plan.part, op, h32, lse); break;
        case 8: merge_share<8>(ws0, tid, cut, plan.part, op, h32, lse); break;
        case 16: merge_share<16>(ws0, tid, cut, plan.part, op, h32, lse); break;
        default: merge_share<32>(ws0, tid, cut, plan.part, op, h32, lse); break;
    }
}

}  // namespace

static bool long_enough_to_cut(const BatchView& b)
{
    constexpr long long MIN_CUT_TILES = 2 * MIN_TILES_PER_PART < MIN_UNIT_TILES_UNDERFILLED ? 2 * MIN_TILES_PER_PART : MIN_UNIT_TILES_UNDERFILLED;
    static_assert(4 * MIN_TILES_PER_PART_UNDERFILLED <= MIN_UNIT_TILES_UNDERFILLED, "short pieces come four or more at a time");
    return ((long long)b.max_pages * b.page_size + BC - 1) / BC >= MIN_CUT_TILES;
}

// The launch shape of a batch, from what the host knows: the scalar fields and whether there is a workspace.
// `slots` is the number of workgroups per XCD that may hold units (the extra ones for pieces come on top).
static void launch_shape(const BatchView& b, bool has_workspace, LaunchShape& L, long long& slots)
{
    const int G = b.num_q_heads / b.num_kv_heads;
    const long long max_rows = (long long)b.max_new_len * G;
    const long long n_pair_tiles = (max_rows + BR - 1) / BR;
    const long long n_real_pairs = (long long)b.num_reqs * b.num_kv_heads;
    int fan = 1;
    while (fan < NUM_XCD && n_real_pairs * fan * 2 <= NUM_XCD) fan *= 2;
    // A request's KV heads go to consecutive XCDs; with fewer than 8 of them (or a number that 8 is no multiple
    // of) a request reaches only some XCDs, and requests of different lengths then load the XCDs unevenly.
    // Dealing every pair to `fan` XCDs with Hkv fan a multiple of 8 gives every XCD the same share of every
    // request.  (A batch of equal requests is balanced without it.)
    if ((long long)b.num_reqs * b.max_new_len != b.total_new_tokens)
        while (fan < NUM_XCD && (b.num_kv_heads * fan) % NUM_XCD != 0) fan *= 2;
    const long long n_pairs = n_real_pairs * fan;                        // sub-pairs
    const long long n_row_tiles = (n_pair_tiles + fan - 1) / fan;        // per sub-pair
    const long long pairs_per_xcd = (n_pairs + NUM_XCD - 1) / NUM_XCD;
    L.n_row_tiles = (int)n_row_tiles;
    L.n_pairs = (int)n_pairs;
    L.pairs_per_xcd = (int)pairs_per_xcd;
    L.fan = fan;
    L.split = (has_workspace && pairs_per_xcd <= SPLIT_MAX_PAIRS_PER_XCD) ? 1 : 0;
    L.uneven = 1;
    const bool uniform = L.split && (long long)b.num_reqs * b.max_new_len == b.total_new_tokens;
    long long units[NUM_XCD] = {};
    if (uniform) {
        // every request has max_new_len new tokens, so the host knows each XCD's unit count and can tell
        // whether any tail unit would be cut at all; if none, the extra workgroups and the merge launch go
        bool alike = true;
        for (int x = 0; x < NUM_XCD; ++x) {
            units[x] = 0;
            for (long long sp = x; sp < n_pairs; sp += NUM_XCD) units[x] += sub_pair_tiles(b.max_new_len, G, fan, (int)sp);
            alike = alike && units[x] == units[0];
        }
        // Uneven cuts shorten the last round of an XCD.  When every XCD has the same number of units, all of them
        // are in their last round together, and the chip being power limited, the compute units that run then use
        // the budget of those that idle: measured, the cut gains nothing there and the merge costs 2 %.  It pays
        // when XCDs finish at different times (ragged batches: 4 % on the cross-attention workload).
        if (alike) L.uneven = 0;
        bool any = false;
        for (int x = 0; x < NUM_XCD; ++x)
            any = any || split_factor((int)(units[x] % CU_PER_XCD), (int)(units[x] / CU_PER_XCD), L.uneven) > 1;
        if (!any) L.split = 0;
    }
    L.ws_pieces = 0;
    if (L.split && long_enough_to_cut(b)) {
        // Piece records of an XCD: tail slot x planned pieces + piece.  r units left over are planned for p pieces
        // with r p <= 32, or for 2 (an uneven cut of 17 .. 30 units): at most 60, which takes 17 units on the XCD.
        // (A context too short to be cut along the keys -- two pieces of the usual minimum, or four short ones on an
        // under-filled XCD -- leaves no records: left-over units can then only be halved along their rows.)
        long long most = 0;
        if (uniform) {
            for (int x = 0; x < NUM_XCD; ++x) {
                const int rem = (int)(units[x] % CU_PER_XCD), full = (int)(units[x] / CU_PER_XCD);
                const int p = rows_only_of(rem, full) ? 1 : split_factor(rem, full, L.uneven);
                most = std::max<long long>(most, p > 1 ? (long long)rem * p : 0);
            }
        } else {
            most = pairs_per_xcd * n_row_tiles > CU_PER_XCD / 2 ? PIECES_PER_XCD : CU_PER_XCD;
        }
        L.ws_pieces = (int)most;
    }
    slots = pairs_per_xcd * n_row_tiles;                                 // one per row tile of the longest request, per pair
    if (L.split) {
        // With cutting, workgroup j of an XCD takes the XCD's unit j, so the grid only has to cover the units there
        // are.  An XCD holds at most ceil(Hkv / 8) pairs of a request, and the row tiles of all requests number at
        // most T G / 256 + B: a batch of one long request and many short ones gets a grid of about its real size
        // instead of one with the longest request's row tiles for every pair (an empty workgroup still holds a
        // compute unit for about a microsecond).
        const long long bound = (long long)((b.num_kv_heads * fan + NUM_XCD - 1) / NUM_XCD) *
                                ((long long)b.total_new_tokens * G / (BR * fan) + b.num_reqs);
        slots = slots < bound ? slots : bound;
    }
}

// bytes behind AttnArgs::workspace that launch_attn_bf16_d128 wants for this batch
size_t attn_bf16_d128_workspace_bytes(const BatchView& b)
{
    LaunchShape L;
    long long slots = 0;
    launch_shape(b, true, L, slots);
    return TIMELINE_BYTES + (size_t)NUM_XCD * L.ws_pieces * PART_FLOATS * sizeof(float);
}

// What the planner makes of a batch whose new-token counts are given as a host array: the launch shape and, per
// XCD, the units, the pieces planned for each tail unit and the kind of cut (see emm_prefill_plan in emm.h).
void attn_bf16_d128_plan_host(const BatchView& b, const int32_t* new_lens, bool has_workspace, int32_t* shape6, long long* grid,
                              int32_t* units, int32_t* pieces, int32_t* uneven_k, int32_t* rows_only)
{
    LaunchShape L;
    long long slots = 0;
    launch_shape(b, has_workspace, L, slots);
    const int G = b.num_q_heads / b.num_kv_heads;
    shape6[0] = L.fan; shape6[1] = L.n_row_tiles; shape6[2] = L.pairs_per_xcd; shape6[3] = L.split; shape6[4] = L.uneven;
    shape6[5] = (int32_t)slots;
    *grid = NUM_XCD * (slots + (L.split ? EXTRA_PER_XCD : 0));
    for (int x = 0; x < NUM_XCD; ++x) {
        long long total = 0;
        for (long long sp = x; sp < L.n_pairs; sp += NUM_XCD) {
            const int r = (int)(sp / L.fan / b.num_kv_heads);
            const int n = std::min(std::max(new_lens[r], 0), std::min(b.max_new_len, b.total_new_tokens));
            total += sub_pair_tiles(n, G, L.fan, (int)sp);
        }
        const int rem = (int)(total % CU_PER_XCD), full = (int)(total / CU_PER_XCD);
        units[x] = (int32_t)total;
        pieces[x] = L.split ? split_factor(rem, full, L.uneven) : 1;
        uneven_k[x] = (L.split && L.uneven) ? uneven_of(rem) : 0;
        rows_only[x] = (L.split && rows_only_of(rem, full)) ? 1 : 0;
    }
}

hipError_t launch_attn_bf16_d128(const AttnArgs& a, hipStream_t stream)
{
    const BatchView& b = a.b;
    if (b.total_new_tokens == 0 || b.num_reqs == 0) return hipSuccess;
    LaunchShape L;
    long long slots = 0;
    launch_shape(b, true, L, slots);
    if (L.ws_pieces > 0 && a.workspace == nullptr) launch_shape(b, false, L, slots);   // no room for piece records: nothing is cut
    const long long per_xcd = slots + (L.split ? EXTRA_PER_XCD : 0);
    const long long grid = NUM_XCD * per_xcd;
    if (grid > 0x3fffffff) return hipErrorInvalidValue;
    if (a.causal)
        hipLaunchKernelGGL(attn_bf16_d128_kernel<true>, dim3((unsigned)grid), dim3(NTHREADS), 0, stream, KernArgs{a, L});
    else
        hipLaunchKernelGGL(attn_bf16_d128_kernel<false>, dim3((unsigned)grid), dim3(NTHREADS), 0, stream, KernArgs{a, L});
    hipError_t err = hipGetLastError();
    if (err != hipSuccess || L.ws_pieces == 0) return err;              // nothing can have been cut along the keys
    hipLaunchKernelGGL(attn_bf16_merge_kernel, dim3(NUM_XCD * MERGE_PER_XCD), dim3(NTHREADS), 0, stream, a, L);
    return hipGetLastError();
}

}  // namespace emm
