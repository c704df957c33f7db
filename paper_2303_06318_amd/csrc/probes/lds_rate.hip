// Microbenchmark: LDS instruction throughput per CU (8 waves issuing back to back).
#include <hip/hip_runtime.h>
#include <cstdio>
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
template<int MODE>
__global__ __launch_bounds__(512) void k(unsigned* out, int iters, long long* cyc){
  __shared__ __attribute__((aligned(16))) char lds[65536];
  const int tid=threadIdx.x, lane=tid&63, wave=tid>>6;
  for (int i=tid;i<16384;i+=512) ((unsigned*)lds)[i]=i*2654435761u;
  __syncthreads();
  u32x4 acc={0,0,0,0};
  // conflict-free address patterns
  const char* p128 = lds + wave*4096 + lane*16;                 // 1 KB contiguous per wave
  const char* p64  = lds + wave*4096 + lane*8;                  // 512 B contiguous per wave
  long long t0 = clock64();
  for (int it=0; it<iters; ++it){
#pragma unroll
    for (int u=0;u<16;u++){
      if (MODE==0){ u32x4 v; unsigned a=(unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)(p128 + (u&3)*1024); asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(4)" : "=v"(v) : "v"(a)); acc[0]^=v[0]; }
      else if (MODE==1){ s16x4 v=__builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p64 + (u&7)*512)); acc[0]^=(unsigned)v[0]; acc[1]^=(unsigned)v[3]; }
      else if (MODE==2){ unsigned a=(unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)(p128 + (u&3)*1024); asm volatile("ds_write_b128 %0, %1" :: "v"(a), "v"(acc) : "memory"); }
      else if (MODE==3){ unsigned long long v; unsigned a=(unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)(p64 + (u&7)*512); asm volatile("ds_read_b64 %0, %1\n\ts_waitcnt lgkmcnt(4)" : "=v"(v) : "v"(a)); acc[0]^=(unsigned)v; }
    }
  }
  long long t1 = clock64();
  out[blockIdx.x*512+tid]=acc[0]^acc[1]^acc[2]^acc[3];
  if (tid==0 && blockIdx.x==0) *cyc = t1-t0;
}
template<int MODE> void run(unsigned* o, long long* c, const char* name, int bytes_per_lane){
  int iters=2000; k<MODE><<<256,512>>>(o,10,c); hipDeviceSynchronize();
  hipEvent_t e0,e1; hipEventCreate(&e0); hipEventCreate(&e1);
  hipEventRecord(e0); k<MODE><<<256,512>>>(o,iters,c); hipEventRecord(e1); hipEventSynchronize(e1);
  float ms; hipEventElapsedTime(&ms,e0,e1); long long hc; hipMemcpy(&hc,c,8,hipMemcpyDeviceToHost);
  double instr = (double)iters*16*8;   // wave-instructions per CU
  double bytes = instr*64*bytes_per_lane;
  printf("%-12s: %.3f ms; %.1f GB/s per CU; clock64 ticks per wave-instr (per CU) %.2f; bytes/tick %.1f\n", name, ms, bytes/ms/1e6, hc/instr, bytes/hc);
}
int main(){ unsigned* o; long long* c; hipMalloc(&o,256*512*4); hipMalloc(&c,8);
  run<0>(o,c,"read_b128",16); run<1>(o,c,"read_tr_b64",8); run<3>(o,c,"read_b64",8); run<2>(o,c,"write_b128",16);
  printf("%s\n", hipGetErrorString(hipDeviceSynchronize())); }
