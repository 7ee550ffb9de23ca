// Standalone microbenchmark (not part of libemm.so): what one more instruction per MFMA costs on gfx950.
// Every wave runs a stream of v_mfma_f32_32x32x16_bf16 (eight independent accumulators) with N
// instructions of one kind after each MFMA, everything written as inline assembly so that the stream is
// exactly the written one.  One workgroup per XCD, so the clock stays at its nominal 2.4 GHz and the
// numbers are cycles, not power.  Two waves per SIMD (512 threads) and one (256 threads).
// Source of the issue-cost model quoted in the header of attn_bf16.hip.
//
//   hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         -o valu_issue_costs paper_2507_10069_amd/csrc/valu_issue_costs.hip && ./valu_issue_costs
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

enum Kind { FMA = 1, EXP, CVT_PK_BF16, DOT2C_BF16, MAX3, NOP, MOV, DOT2C_BURST, PK_FMA_F16, MFMA_4X4X4 };

template <int THREADS, int N, int KIND>
__global__ __launch_bounds__(THREADS) void rate_kernel(const uint4* data, int iters, float* out, float cs)
{
    bf16x8 a[8], b[4];
    for (int i = 0; i < 8; ++i) a[i] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 8 + i) & 4095]);
    for (int i = 0; i < 4; ++i) b[i] = __builtin_bit_cast(bf16x8, data[(threadIdx.x * 8 + 8 + i) & 4095]);
    f32x16 acc[8];
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    float x[16];
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * (threadIdx.x + i);
    float c = 1.0001f;
    float q4[4] = {0.f, 0.f, 0.f, 0.f};
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x4 small = {0.f, 0.f, 0.f, 0.f};
    f32x2 pair = {c, c};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[i]) : "v"(a[i]), "v"(b[i & 3]));
#pragma unroll
            for (int j = 0; j < N; ++j) {
                // sources: results of an MFMA issued four MFMAs earlier (long complete)
                const float s0 = acc[(i + 4) & 7][(4 * j + i) & 15], s1 = acc[(i + 4) & 7][(4 * j + i + 1) & 15];
                float& d = x[(i * N + j) & 15];
                if (KIND == FMA) asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(d) : "v"(s0), "s"(cs), "v"(c));
                if (KIND == EXP) asm volatile("v_exp_f32 %0, %1" : "=v"(d) : "v"(s0));
                if (KIND == CVT_PK_BF16) asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(d) : "v"(s0), "v"(s1));
                if (KIND == DOT2C_BF16) asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(d) : "v"(s0), "v"(c));
                if (KIND == MAX3) asm volatile("v_max3_f32 %0, %1, %2, %0" : "+v"(d) : "v"(s0), "v"(s1));
                if (KIND == NOP) asm volatile("s_nop 0");
                if (KIND == MOV) asm volatile("v_mov_b32 %0, %1" : "=v"(d) : "v"(s0));
                // the same number of dot products per eight MFMAs, but all after the first MFMA
                if (KIND == DOT2C_BURST && i == 0)
                    for (int r = 0; r < 8; ++r) asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(d) : "v"(s0), "v"(c));
                if (KIND == PK_FMA_F16) asm volatile("v_pk_fma_f16 %0, %1, %2, %0" : "+v"(d) : "v"(s0), "v"(c));
                if (KIND == MFMA_4X4X4)
                    asm volatile("v_mfma_f32_4x4x4_16b_bf16 %0, %1, %2, %0" : "+v"(small) : "v"(pair), "v"(pair));
            }
        }
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    float s = q4[0] + small[0];
    for (int i = 0; i < 8; ++i)
        for (int v = 0; v < 16; ++v) s += acc[i][v];
    for (int i = 0; i < 16; ++i) s += x[i];
    if (s == 12345.678f) out[0] = s;
}

template <int THREADS, int N, int KIND>
double run(const uint4* d, float* out)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int iters = 12000;
    rate_kernel<THREADS, N, KIND><<<8, THREADS>>>(d, iters, out, 1.0001f);
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    rate_kernel<THREADS, N, KIND><<<8, THREADS>>>(d, iters, out, 1.0001f);
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double mfma_per_simd = (double)iters * 8 * (THREADS / 256);
    return ms * 1e-3 * 2.4e9 / mfma_per_simd;
}

template <int KIND>
void sweep(const char* name, const uint4* d, float* out)
{
    printf("| %-26s | %5.1f | %5.1f | %5.1f | %5.1f | %5.1f | %5.1f | %5.1f | %5.1f |\n", name,
           run<512, 1, KIND>(d, out), run<512, 2, KIND>(d, out), run<512, 4, KIND>(d, out), run<512, 6, KIND>(d, out),
           run<512, 8, KIND>(d, out), run<512, 12, KIND>(d, out), run<256, 4, KIND>(d, out), run<256, 8, KIND>(d, out));
}

int main()
{
    float* out;
    CHECK(hipMalloc(&out, 64));
    uint4* d;
    CHECK(hipMalloc(&d, 4096 * 16));
    std::vector<unsigned short> h(4096 * 8);
    for (size_t i = 0; i < h.size(); ++i) {
        float f = ((rand() % 2001) - 1000) / 500.0f;   // uniform in [-2, 2]
        unsigned u;
        memcpy(&u, &f, 4);
        h[i] = (unsigned short)(u >> 16);
    }
    CHECK(hipMemcpy(d, h.data(), h.size() * 2, hipMemcpyHostToDevice));
    printf("cycles per MFMA at 2.4 GHz with N instructions of one kind per MFMA and wave (MFMA alone: 32)\n");
    printf("| instruction                | 2 waves/SIMD N=1 | N=2 | N=4 | N=6 | N=8 | N=12 | 1 wave/SIMD N=4 | N=8 |\n");
    printf("|---|---|---|---|---|---|---|---|---|\n");
    sweep<FMA>("v_fma_f32", d, out);
    sweep<MOV>("v_mov_b32", d, out);
    sweep<CVT_PK_BF16>("v_cvt_pk_bf16_f32", d, out);
    sweep<MAX3>("v_max3_f32", d, out);
    sweep<PK_FMA_F16>("v_pk_fma_f16", d, out);
    sweep<EXP>("v_exp_f32", d, out);
    sweep<DOT2C_BF16>("v_dot2c_f32_bf16", d, out);
    sweep<DOT2C_BURST>("v_dot2c, 8N after 1 MFMA in 8", d, out);
    sweep<MFMA_4X4X4>("v_mfma_f32_4x4x4_16b_bf16", d, out);
    sweep<NOP>("s_nop 0", d, out);
    return 0;
}
