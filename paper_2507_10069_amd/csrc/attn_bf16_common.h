// Pieces shared by the bf16 MFMA attention kernels for gfx950 (prefill and decode): vector types, tile
// geometry in LDS, and the few wave-level primitives both use.  Internal to the library.
#pragma once

#include "emm_internal.h"

namespace emm {
namespace bf16attn {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int D = 128;            // head dim
constexpr int NTHREADS = 512;
constexpr int BC = 64;            // keys per tile
constexpr int KV_BYTES = BC * D * 2;   // one K or V tile in LDS: 64 rows of 256 bytes
constexpr int NBUF = 4;             // depth of the K and of the V tile ring in LDS (tile t lives in slot t % NBUF)
constexpr int NUM_XCD = 8;
constexpr float RESCALE_LOG2 = 8.0f;   // slack of the lagging maximum, in powers of two

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

// Row sums of P on the matrix pipe.  v_mfma_f32_4x4x4_16b_bf16 multiplies, in each group of four lanes, a
// 4x4 A (lane = row) by a 4x4 B (lane = column, four k values per lane) and adds C (lane = column, four
// rows per lane).  With A all ones every row of the result is the column sum of B, i.e. each lane gets
// the sum of the four bf16 values it passed in, in all four result registers.  Eight cycles of the
// matrix pipe per instruction and no VALU slot; the dot-product instructions that would do the same on
// the VALU cannot overlap with MFMAs at all.
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4v __attribute__((ext_vector_type(4)));
__device__ inline f32x4 sum4_bf16(uint32_t pair0, uint32_t pair1, f32x4 acc)   // two packed bf16 pairs
{
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const s16x4v ones = {0x3f80, 0x3f80, 0x3f80, 0x3f80};
    const u32x2 q = {pair0, pair1};
    return __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ones, __builtin_bit_cast(s16x4v, q), acc, 0, 0, 0);
}

// Asynchronous copy of 16 bytes per lane from global memory straight into LDS: lane i of the wave
// writes at lds_byte_offset + 16 i.  Written as inline assembly because the compiler, which cannot
// tell which LDS bytes such a load will write, would otherwise make every later LDS read wait for
// it; here the tile being filled is never the tile being read, and completion is awaited
// explicitly (s_waitcnt vmcnt(0)) before the workgroup barrier that publishes the tile.
__device__ inline void lds_dma16(const void* base, uint32_t byte_offset, uint32_t lds_byte_offset)
{
    // address = base (wave-uniform, SGPR pair) + byte_offset (per lane, 32 bits)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_byte_offset), "v"(byte_offset), "s"(base) : "memory");
}

// in-page LDS row of a key: swap bits 2 and 3 of its index within the 16-key page.  With K rows placed
// that way, accumulator registers 8s..8s+7 of a lane of the transposed score block are exactly the 8
// consecutive keys the B operand of the value product expects from it.
__device__ inline int swap23(int x) { return (x & ~12) | ((x & 4) << 1) | ((x & 8) >> 1); }

}  // namespace bf16attn
}  // namespace emm
