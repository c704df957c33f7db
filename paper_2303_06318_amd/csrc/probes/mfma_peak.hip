// Ceiling measurement: back-to-back MFMAs from registers only (no memory), random operand bits.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
template<int NACC>
__global__ __launch_bounds__(512) void k(float* out, int iters, unsigned seed, int constant){
  unsigned r = (threadIdx.x + blockIdx.x*512u)*2654435761u + seed;
  bf16x8 a[4], b[2];
  for (int i=0;i<4;i++){ u32x4 v; for(int j=0;j<4;j++){ r^=r>>15; r*=2246822519u; r^=r>>13; unsigned w = constant? 0x3c003c00u : ((r&0x807f807fu)|0x3c003c00u); v[j]=w;} a[i]=__builtin_bit_cast(bf16x8,v);}
  for (int i=0;i<2;i++){ u32x4 v; for(int j=0;j<4;j++){ r^=r>>15; r*=2246822519u; r^=r>>13; unsigned w = constant? 0x3c003c00u : ((r&0x807f807fu)|0x3c003c00u); v[j]=w;} b[i]=__builtin_bit_cast(bf16x8,v);}
  f32x16 acc[NACC];
  for(int i=0;i<NACC;i++) for(int v=0;v<16;v++) acc[i][v]=0.f;
  for(int it=0; it<iters; ++it){
#pragma unroll
    for(int i=0;i<NACC;i++) acc[i]=__builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i&3], b[i&1], acc[i], 0,0,0);
  }
  float s=0; for(int i=0;i<NACC;i++) for(int v=0;v<16;v++) s+=acc[i][v];
  out[blockIdx.x*512+threadIdx.x]=s;
}
int main(int argc,char**argv){
  int blocks = 256*2; float* o; hipMalloc(&o, blocks*512*4);
  for (int constant=0; constant<2; ++constant) for (int rep=0; rep<2; ++rep){
    int iters = 20000;
    hipEvent_t e0,e1; hipEventCreate(&e0); hipEventCreate(&e1);
    k<8><<<blocks,512>>>(o, 100, 1, constant); hipDeviceSynchronize();
    hipEventRecord(e0); k<8><<<blocks,512>>>(o, iters, 1, constant); hipEventRecord(e1); hipEventSynchronize(e1);
    float ms; hipEventElapsedTime(&ms,e0,e1);
    double fl = (double)blocks*8 /*waves*/ * iters * 8 * 32768.0;
    printf("constant=%d: %.2f ms  %.0f TFLOP/s\n", constant, ms, fl/ms/1e9);
  }
  printf("%s\n", hipGetErrorString(hipDeviceSynchronize()));
}
