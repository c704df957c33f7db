// Microbenchmark: sustained L2 -> CU load bandwidth (data resident in L2), register and LDS-DMA paths.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((address_space(3))) void lds_void;
template<int MODE, int UNROLL>
__global__ __launch_bounds__(512) void k(const u32x4* src, unsigned* out, int iters, size_t region_granules){
  __shared__ u32x4 lds[8192];  // 128 KB
  // every WG walks the same region (L2 resident), offset by wave so requests differ within a CU
  const int tid=threadIdx.x, wave=tid>>6;
  u32x4 acc={0,0,0,0};
  size_t base = ((size_t)blockIdx.x*977) % (region_granules/ (512*UNROLL)) * (512*UNROLL);
  unsigned long long a=(unsigned long long)src;
  i32x4 r; r[0]=__builtin_amdgcn_readfirstlane((int)a); r[1]=__builtin_amdgcn_readfirstlane((int)(a>>32)&0xffff); r[2]=__builtin_amdgcn_readfirstlane((int)(region_granules*16)); r[3]=0x00020000;
  unsigned ldsbase=(unsigned)(unsigned long long)(lds_void*)&lds[0];
  for(int it=0; it<iters; ++it){
    size_t g0 = (base + (size_t)it*512*UNROLL) % region_granules;
    if (MODE==0){
      u32x4 v[UNROLL];
#pragma unroll
      for(int u=0;u<UNROLL;u++) v[u]=src[(g0 + u*512 + tid) % region_granules];
#pragma unroll
      for(int u=0;u<UNROLL;u++){ acc[0]^=v[u][0]; acc[1]^=v[u][1]; acc[2]^=v[u][2]; acc[3]^=v[u][3]; }
    } else {
#pragma unroll
      for(int u=0;u<UNROLL;u++){
        unsigned voff = (unsigned)(((g0 + u*512 + tid) % region_granules)*16);
        unsigned la = ldsbase + __builtin_amdgcn_readfirstlane(((u*8+wave)%128)*1024);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" :: "s"(la), "v"(voff), "s"(r) : "memory","m0");
      }
      __builtin_amdgcn_s_waitcnt(0x0070);
    }
  }
  if (MODE==1){ __syncthreads(); acc = lds[tid]; }
  out[blockIdx.x*512+tid]=acc[0]^acc[1]^acc[2]^acc[3];
}
template<int MODE,int UNROLL> void run(const u32x4* s, unsigned* o, size_t rg, const char* name){
  int blocks=256, iters=2000;
  k<MODE,UNROLL><<<blocks,512>>>(s,o,10,rg); hipDeviceSynchronize();
  hipEvent_t e0,e1; hipEventCreate(&e0); hipEventCreate(&e1);
  hipEventRecord(e0); k<MODE,UNROLL><<<blocks,512>>>(s,o,iters,rg); hipEventRecord(e1); hipEventSynchronize(e1);
  float ms; hipEventElapsedTime(&ms,e0,e1);
  double bytes=(double)blocks*iters*512*UNROLL*16;
  printf("%s unroll %d region %zu KB: %.3f ms  %.2f TB/s aggregate, %.1f GB/s per CU\n", name, UNROLL, rg*16/1024, ms, bytes/ms/1e9, bytes/ms/1e6/256);
}
int main(){
  size_t maxg = (64u<<20)/16; u32x4* s; unsigned* o; hipMalloc(&s, maxg*16); hipMalloc(&o, 256*512*4); hipMemset(s, 1, maxg*16);
  for (size_t kb : {512, 2048, 16384}) {
    size_t rg = kb*1024/16;
    run<0,4>(s,o,rg,"vgpr"); run<0,8>(s,o,rg,"vgpr"); run<1,4>(s,o,rg,"lds-dma"); run<1,8>(s,o,rg,"lds-dma");
  }
  printf("%s\n", hipGetErrorString(hipDeviceSynchronize()));
}
