/*
 * pq_ldsbench.hip -- stand-alone probe of what a table gather costs the LDS of this chip: every lane of a wavefront
 * reads an entry of 4, 8 or 16 bytes whose number it picked at random (fixed per lane, no index arithmetic in the
 * loop), from a compact table (entry e at byte e * size) or from a table with a column per lane (entry e of lane l at
 * row e, column l mod COLS), with all CUs busy (four workgroups of four wavefronts per CU).  Prints the time of one
 * wavefront gather per CU in ns and in cycles of the clock the kernel ran at.
 */
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)
template <int BYTES> struct Vec;
template <> struct Vec<4> { typedef uint32_t T; };
template <> struct Vec<8> { typedef uint2 T; };
template <> struct Vec<16> { typedef uint4 T; };
__device__ inline uint32_t fold(uint32_t v) { return v; }
__device__ inline uint32_t fold(uint2 v) { return v.x ^ v.y; }
__device__ inline uint32_t fold(uint4 v) { return v.x ^ v.y ^ v.z ^ v.w; }

// MODE 0: entry e at byte e*BYTES.  MODE 1: a column per lane: entry e of lane l at byte e*COLS*BYTES + (l % COLS)*BYTES.
template <int BYTES, int N, int MODE, int COLS>
__global__ __launch_bounds__(256) void gather(const uint32_t* seed, uint32_t* out, int iters, long long* clk)
{
    constexpr int kBytes = MODE == 0 ? N * BYTES : N * COLS * BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char tab[kBytes];
    uint32_t* t32 = reinterpret_cast<uint32_t*>(tab);
    for (int i = threadIdx.x; i < kBytes / 4; i += 256) t32[i] = i * 2654435761u;
    __syncthreads();
    uint32_t off[16];
    uint32_t s = seed[threadIdx.x + blockIdx.x * 256];
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        s = s * 1664525u + 1013904223u;
        const uint32_t e = (s >> 9) & (N - 1);
        off[k] = MODE == 0 ? e * BYTES : (e * COLS + (lane % COLS)) * BYTES;
    }
    uint32_t acc = 0;
    typedef typename Vec<BYTES>::T T;
    long long t0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        T v[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) v[k] = *reinterpret_cast<const T*>(tab + off[k]);
#pragma unroll
        for (int k = 0; k < 16; ++k) acc ^= fold(v[k]);
        asm volatile("" ::: "memory");
    }
    long long t1 = clock64(), w1 = wall_clock64();
    out[threadIdx.x + blockIdx.x * 256] = acc;
    if (threadIdx.x == 0 && blockIdx.x == 0) { clk[0] = t1 - t0; clk[1] = w1 - w0; }
}

template <int BYTES, int N, int MODE, int COLS>
void run(const char* what, uint32_t* seed, uint32_t* out, long long* clk)
{
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    const int iters = 2000, blocks = 256 * 4; float best = 1e9f; long long h[2] = {0, 0};
    for (int rep = 0; rep < 3; ++rep) {
        CK(hipEventRecord(e0));
        hipLaunchKernelGGL((gather<BYTES, N, MODE, COLS>), dim3(blocks), dim3(256), 0, 0, seed, out, iters, clk);
        CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
        float ms; CK(hipEventElapsedTime(&ms, e0, e1)); if (ms < best) best = ms;
    }
    CK(hipMemcpy(h, clk, sizeof(h), hipMemcpyDeviceToHost));
    const double mhz = h[1] > 0 ? (double)h[0] / (double)h[1] * 100.0 : 0.0;
    const double ns = best * 1e6 / (16.0 * iters * 16);
    printf("%-34s bytes=%2d N=%5d: %.3f ms  %.2f ns = %.2f cycles per wave-gather per CU (%.0f MHz)\n", what, BYTES, N, best, ns, ns * mhz * 1e-3, mhz);
    fflush(stdout);
}

int main()
{
    const size_t n = 256 * 4 * 256;
    uint32_t *seed, *out; long long* clk;
    CK(hipMalloc(&seed, n * 4)); CK(hipMalloc(&out, n * 4)); CK(hipMalloc(&clk, 16));
    uint32_t* h = (uint32_t*)malloc(n * 4); srand(1); for (size_t i = 0; i < n; ++i) h[i] = (uint32_t)rand() * 2654435761u + (uint32_t)rand();
    CK(hipMemcpy(seed, h, n * 4, hipMemcpyHostToDevice));
    run<4, 1, 0, 1>("b32 broadcast (1 entry)", seed, out, clk);
    run<4, 16, 0, 1>("b32 compact table", seed, out, clk);
    run<4, 32, 0, 1>("b32 compact table", seed, out, clk);
    run<4, 64, 0, 1>("b32 compact table", seed, out, clk);
    run<4, 128, 0, 1>("b32 compact table", seed, out, clk);
    run<4, 1024, 0, 1>("b32 compact table", seed, out, clk);
    run<4, 64, 1, 64>("b32 column per lane, 64 columns", seed, out, clk);
    run<4, 64, 1, 32>("b32 column per lane, 32 columns", seed, out, clk);
    run<8, 1, 0, 1>("b64 broadcast (1 entry)", seed, out, clk);
    run<8, 16, 0, 1>("b64 compact table", seed, out, clk);
    run<8, 32, 0, 1>("b64 compact table", seed, out, clk);
    run<8, 64, 0, 1>("b64 compact table", seed, out, clk);
    run<8, 1024, 0, 1>("b64 compact table", seed, out, clk);
    run<8, 64, 1, 32>("b64 column per lane, 32 columns", seed, out, clk);
    run<8, 64, 1, 16>("b64 column per lane, 16 columns", seed, out, clk);
    run<16, 1, 0, 1>("b128 broadcast (1 entry)", seed, out, clk);
    run<16, 8, 0, 1>("b128 compact table", seed, out, clk);
    run<16, 16, 0, 1>("b128 compact table", seed, out, clk);
    run<16, 64, 0, 1>("b128 compact table", seed, out, clk);
    run<16, 64, 1, 16>("b128 column per lane, 16 columns", seed, out, clk);
    run<16, 64, 1, 8>("b128 column per lane, 8 columns", seed, out, clk);
    return 0;
}
