// Standalone microbenchmark (not part of libemm.so): the rate at which a gfx950 chip can READ a large
// buffer from HBM, by the ways the decode-step attention kernel could fetch its K/V bytes.  The kernels
// fetch and discard (nothing is computed), so the numbers are ceilings for a kernel that must also do
// something with the data.
//
//   reg<U>          512 threads, every lane keeps U 16-byte global loads in flight, contiguous chunks
//   ring<S, A>      512 threads, 32 KB tiles fetched with LDS-DMA (global_load_lds_dwordx4) into a ring of
//                   S slots, A tiles ahead of the one being "consumed", one workgroup barrier per tile
//                   (the scheme of the decode kernel)
//   wave<S, A>      8 independent waves, each with a private ring of S 4 KB slots, A ahead, no barriers
// Each in a "linear" variant (a workgroup reads contiguous memory) and a "paged" one (4 KB chunks in a
// scrambled order, as a page table gives them).
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o hbm_read_rates paper_2507_10069_amd/csrc/hbm_read_rates.hip && ./hbm_read_rates
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e = (x);                                                               \
        if (e != hipSuccess) {                                                            \
            printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__);          \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

constexpr int THREADS = 512;
constexpr int TILE = 32768;            // bytes per tile of the ring kernels
constexpr int CHUNK = 4096;            // bytes that stay contiguous in the paged variants

// chunk -> chunk, a bijection on [0, n_chunks) for n_chunks a power of two
__device__ inline uint32_t scramble(uint32_t c, uint32_t n_chunks, bool paged)
{
    return (paged ? c * 0x9E3779B1u + 0x7F4A7C15u : c) & (n_chunks - 1);      // never leaves the buffer
}

template <int N>
__device__ inline void wait_vm()
{
    __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

__device__ inline void lds_dma16(const void* base, uint32_t byte_offset, uint32_t lds_byte_offset)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_byte_offset), "v"(byte_offset), "s"(base) : "memory");
}

// every workgroup takes tiles blockIdx.x, blockIdx.x + gridDim.x, ...; n_tiles a power of two
template <int U>
__global__ __launch_bounds__(THREADS) void reg_kernel(const unsigned char* buf, uint32_t n_tiles, int paged, uint32_t* out)
{
    const uint32_t n_chunks = n_tiles * (TILE / CHUNK);
    uint4 acc = make_uint4(0, 0, 0, 0);
    // a lane's U loads of one step cover U consecutive 8 KB stripes (2 chunks each); a tile is 4 stripes
    constexpr int STRIPES_PER_TILE = TILE / (THREADS * 16);
    const uint32_t n_stripes = n_tiles * STRIPES_PER_TILE;
    for (uint32_t s0 = blockIdx.x * U; s0 < n_stripes; s0 += gridDim.x * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t stripe = s0 + u;
            const uint32_t byte_in = threadIdx.x * 16;
            const uint32_t chunk = scramble(stripe * 2 + byte_in / CHUNK, n_chunks, paged);
            v[u] = *(const uint4*)(buf + (size_t)chunk * CHUNK + byte_in % CHUNK);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w;
        }
    }
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x12345678u) out[0] = 1;      // keeps the loads alive
}

template <int S, int A>
__global__ __launch_bounds__(THREADS) void ring_kernel(const unsigned char* buf, uint32_t n_tiles, int paged, uint32_t* out)
{
    static_assert(A < S, "the slot being consumed is not overwritten");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[S * TILE];
    const uint32_t n_chunks = n_tiles * (TILE / CHUNK);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
    const uint32_t my_tiles = (n_tiles - blockIdx.x + gridDim.x - 1) / gridDim.x;
    // wave w fetches chunk w of the tile: four 1 KB pieces
    auto load_tile = [&](uint32_t i) {
        const uint32_t tile = (blockIdx.x + (i % my_tiles) * gridDim.x) % n_tiles;      // wraps: stays in the buffer
        const uint32_t chunk = scramble(tile * (TILE / CHUNK) + wave, n_chunks, paged);
        const uint32_t src = chunk * CHUNK;                 // the buffer is at most 1 GiB: 32-bit offsets
        const uint32_t dst = smem_base + (i % S) * TILE + wave * CHUNK;
#pragma unroll
        for (int j = 0; j < 4; ++j) lds_dma16(buf, src + j * 1024 + lane * 16, dst + j * 1024);
    };
    for (int i = 0; i < A; ++i) load_tile(i);
    for (uint32_t i = 0; i < my_tiles; ++i) {
        load_tile(i + A);                                   // into the slot consumed in iteration i - (S - A)
        wait_vm<4 * A>();                                   // tile i has landed
        __syncthreads();
    }
    wait_vm<0>();
    __syncthreads();
    if (smem[threadIdx.x * 16] == 0x5a && n_tiles == 1) out[0] = 1;
}

template <int S, int A>
__global__ __launch_bounds__(THREADS) void wave_kernel(const unsigned char* buf, uint32_t n_tiles, int paged, uint32_t* out)
{
    static_assert(A < S, "the slot being consumed is not overwritten");
    __shared__ __attribute__((aligned(1024))) unsigned char smem[8 * S * CHUNK];
    const uint32_t n_chunks = n_tiles * (TILE / CHUNK);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem + wave * S * CHUNK;
    const uint32_t wave_id = blockIdx.x * 8 + wave, n_waves = gridDim.x * 8;
    const uint32_t my_chunks = (n_chunks - wave_id + n_waves - 1) / n_waves;
    auto load_chunk = [&](uint32_t i) {
        const uint32_t chunk = scramble((wave_id + (i % my_chunks) * n_waves) % n_chunks, n_chunks, paged);
        const uint32_t src = chunk * CHUNK;
        const uint32_t dst = smem_base + (i % S) * CHUNK;
#pragma unroll
        for (int j = 0; j < 4; ++j) lds_dma16(buf, src + j * 1024 + lane * 16, dst + j * 1024);
    };
    for (int i = 0; i < A; ++i) load_chunk(i);
    for (uint32_t i = 0; i < my_chunks; ++i) {
        load_chunk(i + A);
        wait_vm<4 * A>();
    }
    wait_vm<0>();
    __syncthreads();
    if (smem[threadIdx.x * 16] == 0x5a && n_tiles == 1) out[0] = 1;
}


// the decode kernel's fetch pattern: 256 threads, 16 KB tiles = 32 keys of K (first half of the buffer) and
// of V (second half); a tile is two 4 KB pages per pool, wave w fetches half a page of each (K as two
// separate 1 KB runs, V as one 2 KB run).  Workgroup g takes the `per_wg` consecutive tiles from g * per_wg on.
template <int S, int A>
__global__ __launch_bounds__(256) void piece_kernel(const unsigned char* buf, uint32_t n_tiles, int paged, uint32_t* out)
{
    static_assert(A < S, "the slot being consumed is not overwritten");
    constexpr int T = 16384;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[S * T];
    const uint32_t n16 = n_tiles * 2;                       // 16 KB tiles in the buffer
    const uint32_t pool_chunks = n16;                       // 4 KB chunks per pool: two per tile
    const uint32_t pool_bytes = pool_chunks * CHUNK;
    const uint32_t per_wg = n16 / gridDim.x;                // the host picks grids that divide it
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const uint32_t smem_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)smem;
    auto load_tile = [&](uint32_t i) {
        const uint32_t tile = blockIdx.x * per_wg + i % per_wg;
        const uint32_t chunk = scramble(tile * 2 + (wave >> 1), pool_chunks, paged);
        const uint32_t src = chunk * CHUNK + (wave & 1) * 1024;
        const uint32_t dst = smem_base + (i % S) * T + wave * 2048;
        lds_dma16(buf, src + lane * 16, dst);
        lds_dma16(buf, src + 2048 + lane * 16, dst + 1024);
        lds_dma16(buf, pool_bytes + chunk * CHUNK + (wave & 1) * 2048 + lane * 16, dst + 8192);
        lds_dma16(buf, pool_bytes + chunk * CHUNK + (wave & 1) * 2048 + 1024 + lane * 16, dst + 8192 + 1024);
    };
    for (int i = 0; i < A; ++i) load_tile(i);
    for (uint32_t i = 0; i < per_wg; ++i) {
        load_tile(i + A);
        wait_vm<4 * A>();
        __syncthreads();
    }
    wait_vm<0>();
    __syncthreads();
    if (smem[threadIdx.x * 16] == 0x5a && n_tiles == 1) out[0] = 1;
}

typedef void (*Kernel)(const unsigned char*, uint32_t, int, uint32_t*);

static void run(const char* name, Kernel k, const unsigned char* buf, size_t bytes, int grid, int paged, uint32_t* out, int threads = THREADS)
{
    const uint32_t n_tiles = (uint32_t)(bytes / TILE);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int reps = 20;
    for (int i = 0; i < 3; ++i) hipLaunchKernelGGL(k, dim3(grid), dim3(threads), 0, 0, buf, n_tiles, paged, out);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) hipLaunchKernelGGL(k, dim3(grid), dim3(threads), 0, 0, buf, n_tiles, paged, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    CHECK(hipGetLastError());
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double us = ms * 1e3 / reps;
    printf("| %-12s | %5zu MiB | %5d | %-6s | %8.1f | %7.0f |\n", name, bytes >> 20, grid, paged ? "paged" : "linear", us,
           bytes / (us * 1e-6) / 1e9);
    fflush(stdout);
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

int main()
{
    const size_t max_bytes = (size_t)1 << 30;
    unsigned char* buf = nullptr;
    uint32_t* out = nullptr;
    CHECK(hipMalloc(&buf, max_bytes));
    CHECK(hipMalloc(&out, 256));
    CHECK(hipMemset(buf, 1, max_bytes));
    CHECK(hipMemset(out, 0, 256));
    printf("| kernel       | bytes     | WGs   | order  | us       | GB/s    |\n");
    printf("|---|---|---|---|---|---|\n");
    const size_t sizes[2] = {(size_t)256 << 20, (size_t)1 << 30};
    for (size_t bytes : sizes)
        for (int paged = 0; paged < 2; ++paged) {
            for (int grid : {1024, 2048}) {
                run("reg<4>", reg_kernel<4>, buf, bytes, grid, paged, out);
                run("reg<8>", reg_kernel<8>, buf, bytes, grid, paged, out);
            }
            for (int grid : {256, 512}) {
                run("ring<4,2>", ring_kernel<4, 2>, buf, bytes, grid, paged, out);
                run("ring<4,3>", ring_kernel<4, 3>, buf, bytes, grid, paged, out);
                run("ring<5,4>", ring_kernel<5, 4>, buf, bytes, grid, paged, out);
                run("wave<4,3>", wave_kernel<4, 3>, buf, bytes, grid, paged, out);
                run("wave<5,4>", wave_kernel<5, 4>, buf, bytes, grid, paged, out);
            }
            run("ring<2,1>x2", ring_kernel<2, 1>, buf, bytes, 512, paged, out);     // two workgroups per CU
            run("wave<2,1>x2", wave_kernel<2, 1>, buf, bytes, 512, paged, out);
            for (int grid : {512, 1024, 2048, 4096}) run("piece<4,3>", piece_kernel<4, 3>, buf, bytes, grid, paged, out, 256);
        }
    CHECK(hipFree(buf));
    CHECK(hipFree(out));
    return 0;
}
