/*
 * pq_issuebench.hip -- stand-alone probe of what the kernels' instructions cost a SIMD of this chip:
 *   rates    time per vector instruction and SIMD for the encodings the kernels use, with 1, 2 and 4
 *            wavefronts per SIMD (64 independent instructions per loop trip, register operands only)
 *   overlap  whether vector work runs under matrix instructions: matrix only, vector only and both interleaved,
 *            for the encode kernel's v_mfma_f32_32x32x16_bf16 and for the attention kernel's mix of
 *            v_mfma_f32_4x4x4_16b_f16 and v_mfma_f32_16x16x32_f16
 * One workgroup per CU (256 workgroups of 256, 512 or 1024 threads); nothing but registers is touched inside
 * the loops, every thread stores one word at the end.
 */
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>

#define CK(x) do { hipError_t e__ = (x); if (e__ != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e__), __LINE__); exit(1); } } while (0)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBlocks = 256, kMaxThreads = 1024, kTrips = 20000;

enum Kind { FMAC, MUL, LSHR, CVT, FMA, AND_OR, LSHL_OR, ALIGNBIT, PK_MUL_F16, EXP };

template <int KIND>
__global__ __launch_bounds__(kMaxThreads) void rate_kernel(float *out, int trips, float c1, float c2, uint32_t u1, uint32_t u2)
{
    float x[32];
    uint32_t y[32];
    for (int i = 0; i < 32; ++i) { x[i] = (float)threadIdx.x * 0.001f + i; y[i] = threadIdx.x * 2654435761u + i; }
#pragma unroll 1
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int r = 0; r < 2; ++r)
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                if (KIND == FMAC) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[i]) : "v"(c1), "v"(c2));
                if (KIND == MUL) asm volatile("v_mul_f32 %0, %0, %1" : "+v"(x[i]) : "v"(c1));
                if (KIND == LSHR) asm volatile("v_lshrrev_b32 %0, 3, %0" : "+v"(y[i]));
                if (KIND == CVT) asm volatile("v_cvt_f32_f16 %0, %1" : "=v"(x[i]) : "v"(y[i]));
                if (KIND == FMA) asm volatile("v_fma_f32 %0, %0, %1, %2" : "+v"(x[i]) : "v"(c1), "v"(c2));
                if (KIND == AND_OR) asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(y[i]) : "v"(u1), "v"(u2));
                if (KIND == LSHL_OR) asm volatile("v_lshl_or_b32 %0, %0, 3, %1" : "+v"(y[i]) : "v"(u2));
                if (KIND == ALIGNBIT) asm volatile("v_alignbit_b32 %0, %0, %1, 7" : "+v"(y[i]) : "v"(u1));
                if (KIND == PK_MUL_F16) asm volatile("v_pk_mul_f16 %0, %0, %1" : "+v"(y[i]) : "v"(u1));
                if (KIND == EXP) asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
            }
    }
    float s = 0.f;
    for (int i = 0; i < 32; ++i) s += x[i] + (float)y[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

/* MODE bit 0: matrix instructions, bit 1: vector instructions.  Per trip: four v_mfma_f32_32x32x16_bf16 on four
   accumulators, each followed by eight v_fmac_f32. */
template <int MODE>
__global__ __launch_bounds__(512) void overlap_encode_kernel(float *out, int trips, float c1, float c2)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(float)(threadIdx.x + i); b[i] = (__bf16)(float)(i + 1); }
    f32x16 acc[4];
    for (int m = 0; m < 4; ++m)
        for (int i = 0; i < 16; ++i) acc[m][i] = 0.f;
    float x[32];
    for (int i = 0; i < 32; ++i) x[i] = (float)threadIdx.x * 0.001f + i;
#pragma unroll 1
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            if (MODE & 1) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[m]) : "v"(a), "v"(b));
            if (MODE & 2) {
#pragma unroll
                for (int i = 0; i < 8; ++i) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[8 * m + i]) : "v"(c1), "v"(c2));
            }
        }
    }
    float s = 0.f;
    for (int m = 0; m < 4; ++m)
        for (int i = 0; i < 16; ++i) s += acc[m][i];
    for (int i = 0; i < 32; ++i) s += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

/* Per trip: eight v_mfma_f32_4x4x4_16b_f16 each followed by four v_fmac_f32, then four v_mfma_f32_16x16x32_f16 each
   followed by eight v_fmac_f32 (the proportions of a key-tile / value-tile pass of the attention kernel). */
template <int MODE>
__global__ __launch_bounds__(kMaxThreads) void overlap_attn_kernel(float *out, int trips, float c1, float c2)
{
    f16x4 a4, b4;
    for (int i = 0; i < 4; ++i) { a4[i] = (_Float16)(float)(threadIdx.x + i); b4[i] = (_Float16)(float)(i + 1); }
    f16x8 a8, b8;
    for (int i = 0; i < 8; ++i) { a8[i] = (_Float16)(float)(threadIdx.x + i); b8[i] = (_Float16)(float)(i + 1); }
    f32x4 d[8], o[4];
    for (int m = 0; m < 8; ++m)
        for (int i = 0; i < 4; ++i) d[m][i] = 0.f;
    for (int m = 0; m < 4; ++m)
        for (int i = 0; i < 4; ++i) o[m][i] = 0.f;
    float x[32];
    for (int i = 0; i < 32; ++i) x[i] = (float)threadIdx.x * 0.001f + i;
#pragma unroll 1
    for (int t = 0; t < trips; ++t) {
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            if (MODE & 1) asm volatile("v_mfma_f32_4x4x4_16b_f16 %0, %1, %2, %0" : "+v"(d[m]) : "v"(a4), "v"(b4));
            if (MODE & 2) {
#pragma unroll
                for (int i = 0; i < 4; ++i) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[4 * m + i]) : "v"(c1), "v"(c2));
            }
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            if (MODE & 1) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(o[m]) : "v"(a8), "v"(b8));
            if (MODE & 2) {
#pragma unroll
                for (int i = 0; i < 8; ++i) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(x[8 * m + i]) : "v"(c1), "v"(c2));
            }
        }
    }
    float s = 0.f;
    for (int m = 0; m < 8; ++m)
        for (int i = 0; i < 4; ++i) s += d[m][i];
    for (int m = 0; m < 4; ++m)
        for (int i = 0; i < 4; ++i) s += o[m][i];
    for (int i = 0; i < 32; ++i) s += x[i];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <typename F>
static float time_ms(F launch)
{
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0));
    CK(hipEventCreate(&e1));
    launch();
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    for (int r = 0; r < 5; ++r) launch();
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipEventDestroy(e0));
    CK(hipEventDestroy(e1));
    return ms / 5;
}

template <int KIND>
static void rate(const char *name, float *out)
{
    printf("%-26s", name);
    for (int threads : {256, 512, 1024}) {
        const float ms = time_ms([&] {
            hipLaunchKernelGGL(rate_kernel<KIND>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f, 0x0FF0u, 0x3u);
        });
        printf("  %d wavefront%s: %.3f ns", threads / 256, threads == 256 ? " " : "s", ms * 1e6 / ((double)kTrips * 64 * (threads / 256)));
    }
    printf("\n");
    fflush(stdout);
}

int main()
{
    float *out;
    CK(hipMalloc(&out, (size_t)kBlocks * kMaxThreads * sizeof(float)));
    printf("rates: ns per instruction and SIMD (64 independent instructions per trip), by wavefronts per SIMD\n");
    rate<FMAC>("v_fmac_f32 (VOP2)", out);
    rate<MUL>("v_mul_f32 (VOP2)", out);
    rate<LSHR>("v_lshrrev_b32 (VOP2)", out);
    rate<CVT>("v_cvt_f32_f16 (VOP1)", out);
    rate<FMA>("v_fma_f32 (VOP3)", out);
    rate<AND_OR>("v_and_or_b32 (VOP3)", out);
    rate<LSHL_OR>("v_lshl_or_b32 (VOP3)", out);
    rate<ALIGNBIT>("v_alignbit_b32 (VOP3)", out);
    rate<PK_MUL_F16>("v_pk_mul_f16 (VOP3P)", out);
    rate<EXP>("v_exp_f32 (VOP1)", out);
    printf("overlap, encode: per trip 4 x v_mfma_f32_32x32x16_bf16 and / or 32 x v_fmac_f32; ms per launch of %d trips\n", kTrips);
    for (int threads : {256, 512}) {
        const float m1 = time_ms([&] { hipLaunchKernelGGL(overlap_encode_kernel<1>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f); });
        const float m2 = time_ms([&] { hipLaunchKernelGGL(overlap_encode_kernel<2>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f); });
        const float m3 = time_ms([&] { hipLaunchKernelGGL(overlap_encode_kernel<3>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f); });
        printf("  %d wavefronts per SIMD: matrix only %.3f, vector only %.3f, both %.3f (sum %.3f, larger %.3f)\n", threads / 256,
               m1, m2, m3, m1 + m2, m1 > m2 ? m1 : m2);
        fflush(stdout);
    }
    printf("overlap, attention: per trip 8 x v_mfma_f32_4x4x4_16b_f16 + 4 x v_mfma_f32_16x16x32_f16 and / or 64 x v_fmac_f32\n");
    for (int threads : {256, 512, 1024}) {
        const float m1 = time_ms([&] { hipLaunchKernelGGL(overlap_attn_kernel<1>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f); });
        const float m2 = time_ms([&] { hipLaunchKernelGGL(overlap_attn_kernel<2>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f); });
        const float m3 = time_ms([&] { hipLaunchKernelGGL(overlap_attn_kernel<3>, dim3(kBlocks), dim3(threads), 0, 0, out, kTrips, 1.0001f, 0.5f); });
        printf("  %d wavefronts per SIMD: matrix only %.3f, vector only %.3f, both %.3f (sum %.3f, larger %.3f)\n", threads / 256,
               m1, m2, m3, m1 + m2, m1 > m2 ? m1 : m2);
        fflush(stdout);
    }
    CK(hipFree(out));
    return 0;
}
