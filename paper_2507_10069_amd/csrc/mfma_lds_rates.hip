// Standalone microbenchmark (not part of libemm.so): sustained v_mfma_f32_32x32x16_bf16 rate on gfx950
// when the matrix pipe is fed like the attention kernel feeds it -- two waves per SIMD, operands with
// realistic bit patterns, a few VALU instructions and LDS operand reads per MFMA.  It answers what the
// attention kernel can at best reach (the ceilings quoted in the header of attn_bf16.hip).
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o mfma_lds_rates paper_2507_10069_amd/csrc/mfma_lds_rates.hip && ./mfma_lds_rates
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                          \
    do {                                                                                  \
        hipError_t e = (x);                                                               \
        if (e != hipSuccess) {                                                            \
            printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__);          \
            exit(1);                                                                      \
        }                                                                                 \
    } while (0)

// THREADS / 256 waves per SIMD.  Per MFMA: RD2 / 2 LDS reads of 1 KiB (operands fetched one loop trip
// ahead into alternating register sets, so latency is hidden and no copies are needed), NVALU VALU
// instructions (fma and exp2 alternating), and a workgroup barrier every 32 MFMAs if BARRIER.
template <int THREADS, int RD2, int NVALU, int BARRIER>
__global__ __launch_bounds__(THREADS) void rate_kernel(const uint4* data, int iters, float* out)
{
    __shared__ __attribute__((aligned(16))) uint4 sm[4096];
    for (int i = threadIdx.x; i < 4096; i += THREADS) sm[i] = data[i];
    __syncthreads();
    bf16x8 a[8], b[4];
    for (int i = 0; i < 8; ++i) a[i] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 8 + i) & 4095]);
    for (int i = 0; i < 4; ++i) b[i] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 8 + 8 + i) & 4095]);
    f32x16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * (threadIdx.x + i);
    const int addr = (threadIdx.x & 63) * 17;
    uint4 buf_a[8], buf_b[8];
    for (int i = 0; i < 8; ++i) buf_a[i] = sm[(addr + i * 512) & 4095];
    auto body = [&](uint4 (&cur)[8], uint4 (&nxt)[8], int it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (RD2 == 2 || (RD2 == 1 && (i & 1) == 0)) nxt[i] = sm[(addr + (it + 1) * 64 + i * 512) & 4095];
            const bf16x8 op = RD2 == 0 ? a[i] : __builtin_bit_cast(bf16x8, cur[RD2 == 2 ? i : (i & ~1)]);
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(op, b[i & 3], acc[i], 0, 0, 0);
#pragma unroll
            for (int j = 0; j < NVALU; ++j) {
                if (j & 1) x[(i + j) & 7] = __builtin_amdgcn_exp2f(x[(i + j) & 7]);
                else x[(i + j) & 7] = fmaf(x[(i + j) & 7], 1.0001f, 0.5f);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    for (int it = 0; it < iters; it += 2) {
        body(buf_a, buf_b, it);
        body(buf_b, buf_a, it + 1);
        if (BARRIER && (it & 2)) __syncthreads();
    }
    float s = 0;
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    for (int i = 0; i < 8; ++i) s += x[i];
    if (s == 12345.678f) out[0] = s;
}

template <int THREADS, int RD2, int NVALU, int BARRIER>
void run(const char* name, const uint4* d, float* out)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int iters = 24000;
    rate_kernel<THREADS, RD2, NVALU, BARRIER><<<256, THREADS>>>(d, iters, out);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    rate_kernel<THREADS, RD2, NVALU, BARRIER><<<256, THREADS>>>(d, iters, out);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double mfma_per_simd = (double)iters * 8 * (THREADS / 256);
    printf("%-58s %7.3f ms  %5.1f cycles/MFMA at 2.4 GHz  %5.0f TFLOP/s\n", name, ms,
           ms * 1e-3 * 2.4e9 / mfma_per_simd, 256.0 * 4 * mfma_per_simd * 32768.0 / (ms * 1e-3) / 1e12);
}

int main()
{
    float* out;
    CHECK(hipMalloc(&out, 64));
    uint4* d;
    CHECK(hipMalloc(&d, 4096 * 16));
    std::vector<unsigned short> h(4096 * 8);
    for (int mode = 0; mode < 2; ++mode) {
        for (size_t i = 0; i < h.size(); ++i) {
            float f = mode == 0 ? 1.0f : ((rand() % 2001) - 1000) / 500.0f;   // all ones, or uniform in [-2, 2]
            unsigned u;
            memcpy(&u, &f, 4);
            h[i] = (unsigned short)(u >> 16);
        }
        CHECK(hipMemcpy(d, h.data(), h.size() * 2, hipMemcpyHostToDevice));
        printf("-- operands: %s\n", mode == 0 ? "all 1.0" : "uniform in [-2, 2]");
        run<512, 0, 0, 0>("2 waves/SIMD: MFMA only", d, out);
        if (mode == 0) continue;
        run<512, 0, 5, 0>("2 waves/SIMD: MFMA + 5 VALU", d, out);
        run<512, 1, 0, 0>("2 waves/SIMD: MFMA + 0.5 LDS read", d, out);
        run<512, 2, 0, 0>("2 waves/SIMD: MFMA + 1 LDS read", d, out);
        run<512, 1, 5, 0>("2 waves/SIMD: MFMA + 0.5 LDS read + 5 VALU", d, out);
        run<512, 2, 5, 0>("2 waves/SIMD: MFMA + 1 LDS read + 5 VALU", d, out);
        run<512, 2, 5, 1>("2 waves/SIMD: MFMA + 1 LDS read + 5 VALU + barrier / 32 MFMA", d, out);
        run<256, 1, 5, 0>("1 wave/SIMD:  MFMA + 0.5 LDS read + 5 VALU", d, out);
        run<256, 2, 5, 0>("1 wave/SIMD:  MFMA + 1 LDS read + 5 VALU", d, out);
        run<512, 2, 4, 0>("2 waves/SIMD: MFMA + 1 LDS read + 4 VALU", d, out);
        run<512, 2, 3, 0>("2 waves/SIMD: MFMA + 1 LDS read + 3 VALU", d, out);
        run<256, 1, 4, 0>("1 wave/SIMD:  MFMA + 0.5 LDS read + 4 VALU", d, out);
        run<256, 1, 3, 0>("1 wave/SIMD:  MFMA + 0.5 LDS read + 3 VALU", d, out);
        run<256, 1, 0, 0>("1 wave/SIMD:  MFMA + 0.5 LDS read", d, out);
        run<256, 0, 0, 0>("1 wave/SIMD:  MFMA only", d, out);
        run<256, 0, 4, 0>("1 wave/SIMD:  MFMA + 4 VALU", d, out);
    }
    return 0;
}
