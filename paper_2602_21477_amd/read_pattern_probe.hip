// Read-bandwidth probe for gfx950: what the memory system delivers to (A) fully coalesced
// grid-stride reads and (B) the list-scan kernel's lane -> address map (pages of 128 rows, a
// wave takes 32 rows, lane (l & 15, l >> 4) loads 16 bytes of row l & 15 per instruction), with
// no LDS and no MFMA work.  The scan kernel's achieved bandwidth is read against (B).
//   python -m paper_2602_21477_amd.build        (builds read_pattern_probe.bin beside this file)
//   ./read_pattern_probe.bin        (buffer of constant bytes)
//   ./read_pattern_probe.bin r      (buffer of pseudo-random bytes)
//   ./read_pattern_probe.bin r w    (also: both patterns re-reading a window of 16 MB .. 1 GB that
//                                    wraps around, i.e. served by L2 / Infinity Cache instead of HBM)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CK(x) do{hipError_t e=(x); if(e!=hipSuccess){printf("err %s line %d\n", hipGetErrorString(e), __LINE__); exit(1);} }while(0)

template<int UNROLL>
__global__ __launch_bounds__(256) void readA(const u32x4* p, size_t n16, uint32_t* out, size_t wrap16){
  size_t i = (size_t)blockIdx.x*blockDim.x + threadIdx.x, stride=(size_t)gridDim.x*blockDim.x;
  u32x4 acc = {0,0,0,0};
  for (; i + (UNROLL-1)*stride < n16; i += UNROLL*stride){
    u32x4 v[UNROLL];
    #pragma unroll
    for(int u=0;u<UNROLL;++u) v[u]=p[(i+u*stride) % wrap16];
    #pragma unroll
    for(int u=0;u<UNROLL;++u) acc ^= v[u];
  }
  if ((acc.x^acc.y^acc.z^acc.w)==0x12345678) out[0]=1;
}
// pattern B: page of 128 rows x rowbytes; WG of 4 waves; wave handles 32 rows; lane (ln=l&15, lg=l>>4) loads 16B at row ln (+16), offset it*256 + s*64 + lg*16
template<int DEPTH>
__global__ __launch_bounds__(256) void readB(const char* base, size_t npages, int rowbytes, uint32_t* out, size_t wrap){
  const int lane=threadIdx.x&63, wave=threadIdx.x>>6, ln=lane&15, lg=lane>>4;
  const int nit=rowbytes/256;
  u32x4 acc={0,0,0,0};
  for(size_t pg=blockIdx.x; pg<npages; pg+=gridDim.x){
    const char* p0 = base + (pg % wrap)*(size_t)128*rowbytes + (size_t)(wave*32+ln)*rowbytes + lg*16;
    const char* p1 = p0 + (size_t)16*rowbytes;
    u32x4 buf[DEPTH][8];
    #pragma unroll
    for(int d=0; d<DEPTH-1; ++d){
      #pragma unroll
      for(int s=0;s<4;++s){ buf[d][s]=*(const u32x4*)(p0+d*256+s*64); buf[d][4+s]=*(const u32x4*)(p1+d*256+s*64);} }
    for(int it=0; it<nit; it+=DEPTH){
      #pragma unroll
      for(int d=0; d<DEPTH; ++d){
        const int ld = it+d+DEPTH-1;
        if (ld<nit){
          #pragma unroll
          for(int s=0;s<4;++s){ buf[(d+DEPTH-1)%DEPTH][s]=*(const u32x4*)(p0+ld*256+s*64); buf[(d+DEPTH-1)%DEPTH][4+s]=*(const u32x4*)(p1+ld*256+s*64);} }
        if (it+d<nit){
          #pragma unroll
          for(int s=0;s<8;++s) acc ^= buf[d][s];
        }
      }
    }
  }
  if ((acc.x^acc.y^acc.z^acc.w)==0x12345678) out[0]=1;
}
__global__ void fillrand(uint32_t* p, size_t n){ size_t i=(size_t)blockIdx.x*blockDim.x+threadIdx.x, st=(size_t)gridDim.x*blockDim.x; for(;i<n;i+=st){ uint32_t x=(uint32_t)i*2654435761u; x^=x>>15; x*=2246822519u; x^=x>>13; p[i]=x; } }
int main(int argc, char** argv){
  const size_t bytes = (size_t)12<<30;
  char* d; uint32_t* o; CK(hipMalloc(&d, bytes)); CK(hipMalloc(&o, 4)); CK(hipMemset(d, 1, bytes)); if (argc>1) { hipLaunchKernelGGL(fillrand, dim3(4096), dim3(256),0,0,(uint32_t*)d, bytes/4); CK(hipDeviceSynchronize()); printf("random fill\n"); }
  hipEvent_t e0,e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  auto timeit=[&](const char* name, auto launch){
    launch(); CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0)); for(int r=0;r<5;++r) launch(); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
    float ms; CK(hipEventElapsedTime(&ms,e0,e1)); ms/=5; printf("%-40s %.3f ms  %.0f GB/s\n", name, ms, bytes/ms/1e6); fflush(stdout);
  };
  for (int wgs : {256*8}) {
    char nm[64];
    snprintf(nm,64,"A unroll4 grid=%d",wgs); timeit(nm,[&]{ hipLaunchKernelGGL(readA<4>, dim3(wgs), dim3(256),0,0,(const u32x4*)d, bytes/16, o, bytes/16);});
    snprintf(nm,64,"A unroll8 grid=%d",wgs); timeit(nm,[&]{ hipLaunchKernelGGL(readA<8>, dim3(wgs), dim3(256),0,0,(const u32x4*)d, bytes/16, o, bytes/16);});
  }
  for (int rb : {1536, 3072}) for (int wgs : {256*3,256*8}) {
    size_t npages = bytes/((size_t)128*rb); char nm[64];
    snprintf(nm,64,"B depth2 rowbytes=%d grid=%d",rb,wgs); timeit(nm,[&]{ hipLaunchKernelGGL(readB<2>, dim3(wgs), dim3(256),0,0,d,npages,rb,o,npages);});
    snprintf(nm,64,"B depth3 rowbytes=%d grid=%d",rb,wgs); timeit(nm,[&]{ hipLaunchKernelGGL(readB<3>, dim3(wgs), dim3(256),0,0,d,npages,rb,o,npages);});
  }
  if (argc > 2) {
    const int rb = 1536;
    const size_t npages = bytes/((size_t)128*rb);
    for (size_t mb : {16, 32, 64, 128, 256, 512, 1024}) {
      const size_t wrap = (mb<<20)/((size_t)128*rb); char nm[64];
      snprintf(nm,64,"B depth2 window=%zu MB grid=768",mb); timeit(nm,[&]{ hipLaunchKernelGGL(readB<2>, dim3(768), dim3(256),0,0,d,npages,rb,o,wrap);});
      snprintf(nm,64,"A unroll4 window=%zu MB grid=4096",mb); timeit(nm,[&]{ hipLaunchKernelGGL(readA<4>, dim3(4096), dim3(256),0,0,(const u32x4*)d, bytes/16, o, (mb<<20)/16);});
    }
  }
  return 0;
}
