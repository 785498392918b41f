/*
 * pq_membench.hip -- stand-alone HBM probe used next to the benchmark:
 *   stream_read  plain 16-byte streaming reads of as many bytes as one decode step of the
 *                32k-context benchmark moves (the practical read ceiling of the device)
 *   tile_read    the same bytes fetched with the attention kernel's tile load pattern, no arithmetic
 *   plain_copy   a copy of known size, to calibrate the profiler's FETCH_SIZE / WRITE_SIZE counters
 * Buffers are far larger than the 256 MB last-level cache and are rotated between repetitions.
 */
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)

__global__ __launch_bounds__(256) void stream_read(const uint4* __restrict__ p, size_t n16, uint32_t* out){
  size_t i = (size_t)blockIdx.x*blockDim.x + threadIdx.x, stride=(size_t)gridDim.x*blockDim.x;
  uint32_t acc=0;
  for(; i+3*stride<n16; i+=4*stride){ uint4 a=p[i], b=p[i+stride], c=p[i+2*stride], d=p[i+3*stride]; acc += a.x^b.y^c.z^d.w; }
  for(; i<n16; i+=stride){ uint4 a=p[i]; acc+=a.x; }
  if(acc==0x12345678) out[0]=acc;
}
// tile pattern: each wave handles `ct` consecutive tiles of 3968 B from K and V arrays (codes 2944 + radii 1024)
template<int DEPTH>
__global__ __launch_bounds__(256) void tile_read(const uint8_t* kc, const uint8_t* kr, const uint8_t* vc, const uint8_t* vr, int ct, long ntiles, uint32_t* out){
  int lane=threadIdx.x&63; long item=(long)blockIdx.x*4+(threadIdx.x>>6);
  long t0=item*ct; if(t0>=ntiles) return; long t1 = t0+ct<ntiles? t0+ct: ntiles;
  uint32_t acc=0;
  for(long t=t0;t<t1;++t){
    const uint8_t* c=kc+t*2944; const uint8_t* r=kr+t*1024; const uint8_t* c2=vc+t*2944; const uint8_t* r2=vr+t*1024;
    uint4 a=*(const uint4*)(c+lane*16), b=*(const uint4*)(c+1024+lane*16);
    const uint32_t* g=(const uint32_t*)(c+2048+lane*12); uint32_t g0=g[0],g1=g[1],g2=g[2];
    uint32_t c4=*(const uint16_t*)(c+2816+lane*2); uint4 rr=*(const uint4*)(r+lane*16);
    uint4 a2=*(const uint4*)(c2+lane*16), b2=*(const uint4*)(c2+1024+lane*16);
    const uint32_t* gg=(const uint32_t*)(c2+2048+lane*12); uint32_t h0=gg[0],h1=gg[1],h2=gg[2];
    uint32_t d4=*(const uint32_t*)(c2+2816+(lane>>1)*4); const uint4* r4=(const uint4*)(r2+(lane>>1)*32); uint4 q0=r4[0], q1=r4[1];
    acc += a.x^b.y^g0^g1^g2^c4^rr.z^a2.w^b2.x^h0^h1^h2^d4^q0.y^q1.z;
  }
  if(acc==0x12345678) out[0]=acc;
}
__global__ __launch_bounds__(256) void plain_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16){
  size_t i = (size_t)blockIdx.x*blockDim.x + threadIdx.x, stride=(size_t)gridDim.x*blockDim.x;
  for(; i<n16; i+=stride) dst[i]=src[i];
}
int main(){
  size_t bytes = (size_t)1<<31; // 2 GiB buffer, beyond the 256 MB last-level cache
  uint8_t* buf; uint32_t* out; CK(hipMalloc(&buf, bytes)); CK(hipMalloc(&out, 64)); CK(hipMemset(buf, 1, bytes));
  hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  for(int blocks : {1024, 2048, 4096, 8192, 16384}){
    size_t n16 = (size_t)520093696/16; // same bytes as the benchmark step
    float best=1e9;
    for(int rep=0; rep<6; ++rep){
      const uint4* p = (const uint4*)(buf + (size_t)(rep%3)*600000000);
      CK(hipEventRecord(e0)); hipLaunchKernelGGL(stream_read, dim3(blocks), dim3(256), 0, 0, p, n16, out); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms,e0,e1)); if(rep>=2 && ms<best) best=ms;
    }
    printf("stream_read blocks=%d: %.1f us  %.0f GB/s\n", blocks, best*1e3, 520093696/(best*1e-3)/1e9);
  }
  long ntiles = 16L*8*512; // config 2: 65536 tiles per K and V
  for(int ct : {4, 8, 16, 32}){
    float best=1e9;
    for(int rep=0; rep<6; ++rep){
      uint8_t* base = buf + (size_t)(rep%3)*600000000;
      const uint8_t* kc=base; const uint8_t* kr=base+ntiles*2944; const uint8_t* vc=kr+ntiles*1024; const uint8_t* vr=vc+ntiles*2944;
      long items=(ntiles+ct-1)/ct; int blocks=(int)((items+3)/4);
      CK(hipEventRecord(e0)); hipLaunchKernelGGL(tile_read<1>, dim3(blocks), dim3(256), 0, 0, kc,kr,vc,vr,ct,ntiles,out); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms,e0,e1)); if(rep>=2 && ms<best) best=ms;
    }
    printf("tile_read chunk=%d tiles: %.1f us  %.0f GB/s\n", ct, best*1e3, ntiles*3968.0*2/(best*1e-3)/1e9);
  }
  {
    size_t copy_bytes = (size_t)256<<20; // 256 MiB read + 256 MiB written
    float best=1e9;
    for(int rep=0; rep<5; ++rep){
      const uint4* s = (const uint4*)(buf + (size_t)(rep%2)*600000000); uint4* d = (uint4*)(buf + 1300000000 + (size_t)(rep%2)*300000000);
      CK(hipEventRecord(e0)); hipLaunchKernelGGL(plain_copy, dim3(8192), dim3(256), 0, 0, s, d, copy_bytes/16); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms,e0,e1)); if(rep>=1 && ms<best) best=ms;
    }
    printf("plain_copy 268435456 B read + 268435456 B written: %.1f us  %.0f GB/s (read+write)\n", best*1e3, 2*268435456.0/(best*1e-3)/1e9);
  }
  return 0;
}
